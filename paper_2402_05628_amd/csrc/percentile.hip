// Per-channel percentile bounds of X' = norm(x) * gamma + beta (Section "Implementation details": the default
// calibration strategy is "Percentile"; the fractions are parameters because the paper gives no value).  The q-th
// fraction of the n sorted values of a channel sits at h = q (n - 1) and is interpolated linearly between the order
// statistics floor(h) and floor(h) + 1.
//
// One workgroup per channel.  An order statistic is found exactly by a radix select on the order-preserving 64-bit image
// of the float64 values, four bits per pass (16 passes): every pass histograms the digit of the values that share the
// prefix found so far.  The column is not stored: every pass re-reads the float32 input (its 50 KB stay in cache) and
// re-normalizes in float64, which gives the same keys every time.  One more pass yields the next order statistic
// (the same value if it repeats, else the smallest larger one).
#include <cfloat>
#include <cmath>

#include "rq_internal.h"

namespace {

__device__ __forceinline__ unsigned long long to_key(double v) {
  const unsigned long long u = (unsigned long long)__double_as_longlong(v);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ double from_key(unsigned long long k) {
  const unsigned long long u = (k >> 63) ? (k & 0x7FFFFFFFFFFFFFFFull) : ~k;
  return __longlong_as_double((long long)u);
}

__global__ __launch_bounds__(512) void channel_percentile_kernel(const float* __restrict__ x, int64_t T, int D, int64_t ldx,
                                                                 const double* __restrict__ stats, const float* __restrict__ gamma,
                                                                 const float* __restrict__ beta, double q_lo, double q_hi,
                                                                 double* __restrict__ out_lo, double* __restrict__ out_hi) {
  __shared__ unsigned hist[16];
  __shared__ unsigned cnt_le;
  __shared__ unsigned long long next_key;
  const int tid = threadIdx.x, ch = blockIdx.x;
  const double g = gamma ? (double)gamma[ch] : 1.0, b = (gamma && beta) ? (double)beta[ch] : 0.0;
  auto key_of = [&](int64_t row) {
    const double xv = (double)x[row * ldx + ch];
    return to_key(stats ? (xv - stats[2 * row]) * stats[2 * row + 1] * g + b : xv);
  };
  for (int which = 0; which < 2; ++which) {
    const double q = which == 0 ? q_lo : q_hi;
    const double h = q * (double)(T - 1);
    const int64_t k = (int64_t)floor(h);
    const double frac = h - (double)k;
    // ---- the k-th smallest key (0-based), most significant digit first ----
    unsigned long long prefix = 0;
    int64_t rank = k;
    for (int shift = 60; shift >= 0; shift -= 4) {
      if (tid < 16) hist[tid] = 0;
      __syncthreads();
      const unsigned long long mask = shift == 60 ? 0ull : ~0ull << (shift + 4);
      for (int64_t row = tid; row < T; row += 512) {
        const unsigned long long key = key_of(row);
        if ((key & mask) == prefix) atomicAdd(&hist[(unsigned)(key >> shift) & 15u], 1u);
      }
      __syncthreads();
      int digit = 0;
      int64_t before = 0;
      for (; digit < 15; ++digit) {                        // every thread walks the same 16 counters
        const int64_t c = hist[digit];
        if (rank < before + c) break;
        before += c;
      }
      rank -= before;
      prefix |= (unsigned long long)digit << shift;
      __syncthreads();
    }
    // ---- the next order statistic: the same value if it occurs more than rank + 1 times, else the smallest larger one ----
    if (tid == 0) { cnt_le = 0; next_key = ~0ull; }
    __syncthreads();
    unsigned my_le = 0;
    unsigned long long my_next = ~0ull;
    for (int64_t row = tid; row < T; row += 512) {
      const unsigned long long key = key_of(row);
      if (key <= prefix) ++my_le;
      else if (key < my_next) my_next = key;
    }
    atomicAdd(&cnt_le, my_le);
    atomicMin(&next_key, my_next);
    __syncthreads();
    if (tid == 0) {
      const double vk = from_key(prefix);
      const double vk1 = ((int64_t)cnt_le > k + 1 || next_key == ~0ull) ? vk : from_key(next_key);
      const double v = vk + frac * (vk1 - vk);
      if (which == 0) out_lo[ch] = v; else out_hi[ch] = v;
    }
    __syncthreads();
  }
}

}  // namespace

rq_status rq_launch_ln_channel_percentile(rq_ctx* ctx, const float* x, int64_t T, int32_t D, int64_t ldx, int32_t norm_kind,
                                          double eps, const float* gamma, const float* beta, double q_lo, double q_hi,
                                          double* lo, double* hi, void* workspace) {
  double* stats = nullptr;
  if (gamma) {
    stats = static_cast<double*>(workspace);
    const rq_status rc = rq_launch_row_stats(ctx, x, T, D, ldx, norm_kind, eps, stats);      // mean and 1 / sqrt(var + eps) per row
    if (rc != RQ_OK) return rc;
  }
  hipLaunchKernelGGL(channel_percentile_kernel, dim3((unsigned)D), dim3(512), 0, ctx->stream, x, T, D, ldx, stats, gamma, beta, q_lo,
                     q_hi, lo, hi);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}
