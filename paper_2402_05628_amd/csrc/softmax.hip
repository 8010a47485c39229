// rq_softmax_log2_quant: Softmax fused with the log-sqrt2 quantizer in base-2 form
// (Section "Scale reparameterization for Softmax activations", Eq. (3.3-1), second line).
//
// HBM-bound: 4 B (int32 accumulator) read + 1 B (code) written per element.  One row lives in the registers
// of LPR lanes (16, 32 or 64 of a 64-wide wavefront, so short rows of 49..257 keys still fill the wavefront);
// max and sum are wavefront shuffles; codes leave as one dword (4 codes) per lane.  The probability is never
// formed:  -2 log2(softmax_j / s) = 2 (log2 sum_k 2^(t_k) - t_j + log2 s),  t = logit * log2(e).
// Without a bias the row maximum is an integer maximum and t_j - t_max = c * (acc_j - acc_max) exactly;
// the linear part runs in float64 (fp64 is full rate here), only the exponentials run in float32.
#include "rq_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

struct SmParams {
  const int32_t* acc;
  uint8_t* codes;
  const float* bias;
  int64_t rows;       // G * Nq
  int64_t ld;
  int Nq, Nk, H;
  int causal;
  double c1;          // logit_scale * log2(e)
  double log2s;       // log2(s_log)
  int qmax;
};

template <int LPR, int MAXNV, bool HAS_BIAS>
__global__ __launch_bounds__(256) void softmax_kernel(const SmParams p) {
  constexpr int RPW = 64 / LPR;
  const int lane = threadIdx.x & 63;
  const int sub = lane % LPR;
  const int64_t row = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + lane / LPR;
  const bool live = row < p.rows;
  const int64_t r = live ? row : p.rows - 1;
  const int64_t g = r / p.Nq;
  const int i = (int)(r - g * p.Nq);
  const int limit = p.causal ? (i + 1 < p.Nk ? i + 1 : p.Nk) : p.Nk;   // valid keys: j < limit
  const int chunks = (int)(p.ld >> 2);
  const int32_t* arow = p.acc + r * p.ld;
  const float* brow = HAS_BIAS ? p.bias + ((int64_t)(g % p.H) * p.Nq + i) * p.Nk : nullptr;

  v4i a[MAXNV];
  double t[HAS_BIAS ? MAXNV * 4 : 1];
#pragma unroll
  for (int v = 0; v < MAXNV; ++v) {
    const int c = sub + v * LPR;
    a[v] = (c < chunks && c * 4 < limit) ? *reinterpret_cast<const v4i*>(arow + c * 4) : v4i{0, 0, 0, 0};
  }

  const float c1f = (float)p.c1;
  float ssum = 0.f;
  double tmax = -1e300;
  int amax = INT32_MIN;
  if (HAS_BIAS) {
#pragma unroll
    for (int v = 0; v < MAXNV; ++v) {
      const int c = sub + v * LPR;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = c * 4 + e;
        const bool ok = c < chunks && j < limit;
        const double tv = ok ? fma((double)a[v][e], p.c1, (double)brow[ok ? j : 0] * 1.4426950408889634) : -1e300;
        t[v * 4 + e] = tv;
        tmax = fmax(tmax, tv);
      }
    }
#pragma unroll
    for (int m = 1; m < LPR; m <<= 1) tmax = fmax(tmax, __shfl_xor(tmax, m, 64));
#pragma unroll
    for (int v = 0; v < MAXNV; ++v)
#pragma unroll
      for (int e = 0; e < 4; ++e) ssum += __builtin_amdgcn_exp2f((float)(t[v * 4 + e] - tmax));   // exp2(-huge) = 0
  } else {
#pragma unroll
    for (int v = 0; v < MAXNV; ++v) {
      const int c = sub + v * LPR;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool ok = c < chunks && (c * 4 + e) < limit;
        amax = ok ? (a[v][e] > amax ? a[v][e] : amax) : amax;
      }
    }
#pragma unroll
    for (int m = 1; m < LPR; m <<= 1) {
      const int o = __shfl_xor(amax, m, 64);
      amax = o > amax ? o : amax;
    }
#pragma unroll
    for (int v = 0; v < MAXNV; ++v) {
      const int c = sub + v * LPR;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool ok = c < chunks && (c * 4 + e) < limit;
        // acc - amax <= 0 and may wrap below INT32_MIN only if |acc| > 2^30, which the int32 contract excludes
        const float ex = __builtin_amdgcn_exp2f((float)(a[v][e] - amax) * c1f);
        ssum += ok ? ex : 0.f;
      }
    }
  }
#pragma unroll
  for (int m = 1; m < LPR; m <<= 1) ssum += __shfl_xor(ssum, m, 64);
  // code = rint(2 * (log2(sum) - (t_j - t_max) + log2 s))
  const double C0 = 2.0 * ((double)__builtin_amdgcn_logf(ssum) + p.log2s);
  const double m2c = -2.0 * p.c1;

  if (!live) return;
  uint8_t* crow = p.codes + row * p.ld;
#pragma unroll
  for (int v = 0; v < MAXNV; ++v) {
    const int c = sub + v * LPR;
    if (c < chunks) {
      int code[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = c * 4 + e;
        double val;
        if (HAS_BIAS) val = fma(t[v * 4 + e] - tmax, -2.0, C0);
        else val = fma((double)(a[v][e] - amax), m2c, C0);
        int k = (int)rint(val);
        k = k < 0 ? 0 : (k > p.qmax ? p.qmax : k);
        code[e] = j < limit ? k : p.qmax;
      }
      *reinterpret_cast<int*>(crow + c * 4) = rq_pack4(code[0], code[1], code[2], code[3]);
    }
  }
}

template <int LPR, int MAXNV>
void launch(rq_ctx* ctx, const SmParams& p, bool has_bias) {
  const int64_t rows_per_block = 4 * (64 / LPR);
  const unsigned blocks = (unsigned)((p.rows + rows_per_block - 1) / rows_per_block);
  if (has_bias) hipLaunchKernelGGL((softmax_kernel<LPR, MAXNV, true>), dim3(blocks), dim3(256), 0, ctx->stream, p);
  else hipLaunchKernelGGL((softmax_kernel<LPR, MAXNV, false>), dim3(blocks), dim3(256), 0, ctx->stream, p);
}

}  // namespace

rq_status rq_launch_softmax(rq_ctx* ctx, const rq_softmax_desc* d) {
  SmParams p;
  p.acc = d->acc; p.codes = d->codes; p.bias = d->bias;
  p.rows = d->G * d->Nq; p.ld = d->ld; p.Nq = d->Nq; p.Nk = d->Nk; p.H = d->H;
  p.causal = d->mask == RQ_MASK_CAUSAL;
  p.c1 = d->logit_scale * 1.4426950408889634;
  p.log2s = log2((double)d->s_log);
  p.qmax = (1 << d->bits) - 1;
  const int chunks = (int)(d->ld / 4);
  // lanes per row: the choice that wastes the fewest lane slots, smaller groups first
  int best_lpr = 64, best_nv = (chunks + 63) / 64;
  int64_t best_waste = (int64_t)best_nv * 64 - chunks;
  for (int lpr : {32, 16}) {
    const int nv = (chunks + lpr - 1) / lpr;
    const int64_t waste = (int64_t)nv * lpr - chunks;
    if (nv <= 8 && waste <= best_waste) { best_lpr = lpr; best_nv = nv; best_waste = waste; }
  }
  const bool hb = d->bias != nullptr;
#define RQ_SM_CASE(L, N)                         \
  if (best_lpr == L && best_nv <= N) {           \
    launch<L, N>(ctx, p, hb);                    \
    RQ_HIP(hipGetLastError());                   \
    return RQ_OK;                                \
  }
  RQ_SM_CASE(16, 1) RQ_SM_CASE(16, 2) RQ_SM_CASE(16, 4) RQ_SM_CASE(16, 6) RQ_SM_CASE(16, 8)
  RQ_SM_CASE(32, 1) RQ_SM_CASE(32, 2) RQ_SM_CASE(32, 4) RQ_SM_CASE(32, 6) RQ_SM_CASE(32, 8)
  RQ_SM_CASE(64, 1) RQ_SM_CASE(64, 2) RQ_SM_CASE(64, 4) RQ_SM_CASE(64, 8) RQ_SM_CASE(64, 16)
#undef RQ_SM_CASE
  return rq_fail(ctx, RQ_ERR_SHAPE, "rq_softmax_log2_quant: row pitch %lld exceeds the supported 4096", (long long)d->ld);
}
