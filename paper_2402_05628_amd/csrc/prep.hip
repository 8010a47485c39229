// Preparation kernels (run once per block, not on the timed path): rq_reparam_fold, rq_weight_quant_pack,
// rq_rowsum_i8 and the min/max reductions used by calibration.  All float arithmetic is float64.
#include <cfloat>

#include "rq_internal.h"

namespace {

__device__ __forceinline__ double block_sum_256(double v, double* sm) {
  const int tid = threadIdx.x;
  __syncthreads();
  sm[tid] = v;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) sm[tid] += sm[tid + s];
    __syncthreads();
  }
  return sm[0];
}

// Section "Scale reparameterization for LayerNorm activations": s~, z~, r1, r2 and the folded gamma~, beta~, W~, b~.
// One workgroup per output row of W; every workgroup recomputes the two means in the same order.
__global__ __launch_bounds__(256) void fold_kernel(rq_fold_desc d) {
  __shared__ double sm[256];
  const int tid = threadIdx.x;
  double ss = 0.0, zs = 0.0;
  for (int i = tid; i < d.D; i += 256) {
    ss += (double)d.s_ch[i];
    zs += (double)d.z_ch[i];
  }
  const double s_t = block_sum_256(ss, sm) / (double)d.D;
  const double z_t = rint(block_sum_256(zs, sm) / (double)d.D);
  if (blockIdx.x == 0) {
    if (tid == 0) {
      *d.s_tilde = (float)s_t;
      *d.z_tilde = (int)z_t;
      if (d.s_log_pair) {
        d.s_log_pair[0] = d.s_log;
        d.s_log_pair[1] = (float)((double)d.s_log * 1.4142135623730951);
      }
    }
    for (int i = tid; i < d.D; i += 256) {
      const double s = (double)d.s_ch[i];
      const double r1 = s / s_t;
      const double r2 = (double)d.z_ch[i] - z_t;
      const double beta = d.beta ? (double)d.beta[i] : 0.0;
      d.gamma_t[i] = (float)((double)d.gamma[i] / r1);
      d.beta_t[i] = (float)((beta + s * r2) / r1);
    }
  }
  for (int j = blockIdx.x; j < d.D_out; j += gridDim.x) {
    const float* w = d.W + (int64_t)j * d.D;
    float* wt = d.W_t + (int64_t)j * d.D;
    double acc = 0.0;
    for (int i = tid; i < d.D; i += 256) {
      const double s = (double)d.s_ch[i];
      const double r1 = s / s_t;
      const double r2 = (double)d.z_ch[i] - z_t;
      const double wv = (double)w[i];
      acc = fma(s * r2, wv, acc);
      wt[i] = (float)(r1 * wv);
    }
    const double dot = block_sum_256(acc, sm);
    if (tid == 0) d.b_t[j] = (float)((d.b ? (double)d.b[j] : 0.0) - dot);
  }
}

// Channel-wise weight quantization, one workgroup per output channel (Eq. for s and z, per row of W).  The row's range is
// taken to contain 0 (a row whose weights share one sign is extended to 0), so that the zero-point is a code in
// [0, 2^b - 1]: the packed 4-bit GEMM operands subtract it byte-wise without widening.  A row of zeros gets s = 1.
__global__ __launch_bounds__(256) void weight_quant_kernel(rq_wq_desc d) {
  __shared__ float smin[256], smax[256];
  __shared__ int ssum[256];
  const int tid = threadIdx.x;
  const int n = blockIdx.x;
  const float* w = d.W + (int64_t)n * d.K;
  float lo = 0.f, hi = 0.f;
  for (int k = tid; k < d.K; k += 256) {
    const float v = w[k];
    lo = fminf(lo, v);
    hi = fmaxf(hi, v);
  }
  smin[tid] = lo;
  smax[tid] = hi;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) {
      smin[tid] = fminf(smin[tid], smin[tid + s]);
      smax[tid] = fmaxf(smax[tid], smax[tid + s]);
    }
    __syncthreads();
  }
  const double dlo = (double)smin[0], dhi = (double)smax[0];
  const int qmax = (1 << d.bits) - 1;
  float s_f = (float)((dhi - dlo) / (double)qmax);
  if (!(s_f > 0.f)) s_f = 1.f;
  const double s = (double)s_f;
  const int z = (int)rint(-dlo / s);
  int r = n;   // output row
  if (d.gate_up_rows > 0) {
    const int Dm = d.gate_up_rows;
    const int j = n < Dm ? n : n - Dm;
    r = (j / 32) * 64 + (n < Dm ? 0 : 32) + (j % 32);
  }
  int csum = 0;
  if (d.format == RQ_W_U4) {
    uint8_t* out = static_cast<uint8_t*>(d.w_out) + (int64_t)r * (d.K / 2);
    for (int g = tid; g < d.K / 8; g += 256) {
      int c[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        int q = (int)rint((double)w[g * 8 + e] / s) + z;
        q = q < 0 ? 0 : (q > qmax ? qmax : q);
        c[e] = q;
        csum += q - z;
      }
      const uint32_t pk = (uint32_t)(c[0] | (c[4] << 4)) | ((uint32_t)(c[1] | (c[5] << 4)) << 8) |
                          ((uint32_t)(c[2] | (c[6] << 4)) << 16) | ((uint32_t)(c[3] | (c[7] << 4)) << 24);
      *reinterpret_cast<uint32_t*>(out + g * 4) = pk;
    }
  } else {
    int8_t* out = static_cast<int8_t*>(d.w_out) + (int64_t)r * d.K;
    const int off = d.format == RQ_W_I8_CENTERED ? 128 : z;
    for (int k = tid; k < d.K; k += 256) {
      int q = (int)rint((double)w[k] / s) + z;
      q = q < 0 ? 0 : (q > qmax ? qmax : q);
      out[k] = (int8_t)(q - off);
      csum += q - z;
    }
  }
  ssum[tid] = csum;
  __syncthreads();
  for (int s2 = 128; s2 > 0; s2 >>= 1) {
    if (tid < s2) ssum[tid] += ssum[tid + s2];
    __syncthreads();
  }
  if (tid == 0) {
    d.s_w[r] = s_f;
    d.z_w[r] = z;
    d.colsum_w[r] = ssum[0];
    if (d.bias_out) d.bias_out[r] = d.bias ? d.bias[n] : 0.f;
  }
}

__global__ __launch_bounds__(256) void rowsum_kernel(const int8_t* __restrict__ A, int64_t M, int K, int64_t lda,
                                                     int32_t* __restrict__ rowsum) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const int8_t* a = A + row * lda;
  int s = 0;
  for (int k = lane * 4; k < K; k += 256) {
    const int v = *reinterpret_cast<const int*>(a + k);
    s += (int)(int8_t)(v & 0xFF) + (int)(int8_t)((v >> 8) & 0xFF) + (int)(int8_t)((v >> 16) & 0xFF) + (v >> 24);
  }
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) s += __shfl_xor(s, m, 64);
  if (lane == 0) rowsum[row] = s;
}

// order-preserving map double <-> uint64 so that min/max become unsigned integer atomics
__device__ __forceinline__ unsigned long long enc(double v) {
  const unsigned long long u = (unsigned long long)__double_as_longlong(v);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ double dec(unsigned long long u) {
  const unsigned long long b = (u >> 63) ? (u & 0x7FFFFFFFFFFFFFFFull) : ~u;
  return __longlong_as_double((long long)b);
}

__global__ void minmax_init_kernel(unsigned long long* mn, unsigned long long* mx, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    mn[i] = ~0ull;
    mx[i] = 0ull;
  }
}
__global__ void minmax_decode_kernel(double* mn, double* mx, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    mn[i] = dec(reinterpret_cast<unsigned long long*>(mn)[i]);
    mx[i] = dec(reinterpret_cast<unsigned long long*>(mx)[i]);
  }
}

// Per-channel extremes of LayerNorm(x) * gamma + beta over all tokens (Eqs. for X'_up, X'_low before clipping).
// One wavefront per row; each lane owns channels lane*4 + 256*i.
template <int MAXC>
__global__ __launch_bounds__(256) void ln_channel_minmax_kernel(const float* __restrict__ x, int64_t T, int D, int64_t ldx,
                                                                int norm_kind, double eps, const float* __restrict__ gamma,
                                                                const float* __restrict__ beta, unsigned long long* mn,
                                                                unsigned long long* mx) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t nwave = (int64_t)gridDim.x * 4;
  double lo[MAXC * 4], hi[MAXC * 4];
#pragma unroll
  for (int i = 0; i < MAXC * 4; ++i) { lo[i] = DBL_MAX; hi[i] = -DBL_MAX; }
  const int chunks = D / 4;
  for (int64_t row = wave; row < T; row += nwave) {
    const float* xr = x + row * ldx;
    double s1 = 0.0, s2 = 0.0;
    for (int c = lane; c < chunks; c += 64) {
      const float4 v = *reinterpret_cast<const float4*>(xr + c * 4);
      const double a = v.x, b = v.y, cc = v.z, dd = v.w;
      s1 += (a + b) + (cc + dd);
      s2 = fma(a, a, s2); s2 = fma(b, b, s2); s2 = fma(cc, cc, s2); s2 = fma(dd, dd, s2);
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) { s1 += __shfl_xor(s1, m, 64); s2 += __shfl_xor(s2, m, 64); }
    double mean = 0.0, var;
    if (norm_kind == RQ_NORM_LAYERNORM) {
      mean = s1 / (double)D;
      var = fma(-mean, mean, s2 / (double)D);
      var = var < 0.0 ? 0.0 : var;
    } else {
      var = s2 / (double)D;
    }
    const double rstd = 1.0 / sqrt(var + eps);
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int c = lane + 64 * i;
      if (c < chunks) {
        const float4 v = *reinterpret_cast<const float4*>(xr + c * 4);
        const float xv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int ch = c * 4 + e;
          const double y = ((double)xv[e] - mean) * rstd * (double)gamma[ch] + (beta ? (double)beta[ch] : 0.0);
          lo[i * 4 + e] = fmin(lo[i * 4 + e], y);
          hi[i * 4 + e] = fmax(hi[i * 4 + e], y);
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (lo[i * 4 + e] <= hi[i * 4 + e]) {
          atomicMin(&mn[c * 4 + e], enc(lo[i * 4 + e]));
          atomicMax(&mx[c * 4 + e], enc(hi[i * 4 + e]));
        }
      }
    }
  }
}

__global__ __launch_bounds__(256) void minmax_f32_kernel(const float* __restrict__ v, int64_t rows, int64_t cols, int64_t ld,
                                                         unsigned long long* mn, unsigned long long* mx) {
  double lo = DBL_MAX, hi = -DBL_MAX;
  const int64_t total = rows * cols;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / cols, c = i - r * cols;
    const double y = (double)v[r * ld + c];
    lo = fmin(lo, y);
    hi = fmax(hi, y);
  }
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    lo = fmin(lo, __shfl_xor(lo, m, 64));
    hi = fmax(hi, __shfl_xor(hi, m, 64));
  }
  if ((threadIdx.x & 63) == 0 && lo <= hi) {
    atomicMin(mn, enc(lo));
    atomicMax(mx, enc(hi));
  }
}

// Channel-wise (s, z) from the channel extremes, with the optional dual-clipping contraction factors
// (Eqs. for X'_up, X'_low, then the Eq. for s and z per channel); the scale is stored float32 and z follows it.
__global__ void channel_qparams_kernel(const double* cmin, const double* cmax, const float* clip_up, const float* clip_lo,
                                       int D, int bits, float* s_ch, int32_t* z_ch) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= D) return;
  const double up = cmax[i] * (clip_up ? (double)clip_up[i] : 1.0);
  const double lo = cmin[i] * (clip_lo ? (double)clip_lo[i] : 1.0);
  const float s = (float)((up - lo) / (double)((1 << bits) - 1));
  s_ch[i] = s;
  z_ch[i] = (int)rint(-lo / (double)s);
}

}  // namespace

rq_status rq_launch_channel_qparams(rq_ctx* ctx, const double* cmin, const double* cmax, const float* clip_up,
                                    const float* clip_lo, int D, int bits, float* s_ch, int32_t* z_ch) {
  hipLaunchKernelGGL(channel_qparams_kernel, dim3((D + 255) / 256), dim3(256), 0, ctx->stream, cmin, cmax, clip_up, clip_lo, D, bits,
                     s_ch, z_ch);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

rq_status rq_launch_fold(rq_ctx* ctx, const rq_fold_desc* d) {
  int blocks = d->D_out < 1 ? 1 : d->D_out;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(fold_kernel, dim3(blocks), dim3(256), 0, ctx->stream, *d);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

rq_status rq_launch_weight_quant(rq_ctx* ctx, const rq_wq_desc* d) {
  hipLaunchKernelGGL(weight_quant_kernel, dim3(d->N), dim3(256), 0, ctx->stream, *d);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

rq_status rq_launch_rowsum(rq_ctx* ctx, const int8_t* A, int64_t M, int32_t K, int64_t lda, int32_t* rowsum) {
  hipLaunchKernelGGL(rowsum_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, ctx->stream, A, M, K, lda, rowsum);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

rq_status rq_launch_ln_channel_minmax(rq_ctx* ctx, const float* x, int64_t T, int32_t D, int64_t ldx, int32_t norm_kind,
                                      double eps, const float* gamma, const float* beta, double* cmin, double* cmax) {
  auto* mn = reinterpret_cast<unsigned long long*>(cmin);
  auto* mx = reinterpret_cast<unsigned long long*>(cmax);
  hipLaunchKernelGGL(minmax_init_kernel, dim3((D + 255) / 256), dim3(256), 0, ctx->stream, mn, mx, D);
  int64_t blocks = (T + 3) / 4;
  if (blocks > 1024) blocks = 1024;
  const int chunks_per_lane = (D / 4 + 63) / 64;
  if (chunks_per_lane <= 4)
    hipLaunchKernelGGL(ln_channel_minmax_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, x, T, D, ldx, norm_kind,
                       eps, gamma, beta, mn, mx);
  else if (chunks_per_lane <= 16)
    hipLaunchKernelGGL(ln_channel_minmax_kernel<16>, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, x, T, D, ldx, norm_kind,
                       eps, gamma, beta, mn, mx);
  else
    hipLaunchKernelGGL(ln_channel_minmax_kernel<32>, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, x, T, D, ldx, norm_kind,
                       eps, gamma, beta, mn, mx);
  hipLaunchKernelGGL(minmax_decode_kernel, dim3((D + 255) / 256), dim3(256), 0, ctx->stream, cmin, cmax, D);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

rq_status rq_launch_minmax_f32(rq_ctx* ctx, const float* v, int64_t rows, int64_t cols, int64_t ld, double* out2) {
  auto* mn = reinterpret_cast<unsigned long long*>(out2);
  auto* mx = mn + 1;
  hipLaunchKernelGGL(minmax_init_kernel, dim3(1), dim3(64), 0, ctx->stream, mn, mx, 1);
  hipLaunchKernelGGL(minmax_f32_kernel, dim3(1024), dim3(256), 0, ctx->stream, v, rows, cols, ld, mn, mx);
  hipLaunchKernelGGL(minmax_decode_kernel, dim3(1), dim3(64), 0, ctx->stream, out2, out2 + 1, 1);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}
