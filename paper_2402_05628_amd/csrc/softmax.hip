// rq_softmax_log2_quant: Softmax fused with the log-sqrt2 quantizer in base-2 form
// (Section "Scale reparameterization for Softmax activations", Eq. (3.3-1), second line).
//
// HBM-bound: 4 B (int32 accumulator) read + 1 B (code) written per element.  One row lives in the registers
// of LPR lanes (16, 32 or 64 of a 64-wide wavefront, so short rows of 49..257 keys still fill the wavefront);
// max and sum are DPP exchanges inside 16-lane rows plus shuffles across them; codes leave as one dword (4 codes) per lane.  The probability is never
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

// reductions over the LPR lanes of a row group: DPP exchanges inside 16-lane rows, shuffles across them
template <int LPR> __device__ __forceinline__ int group_max_i(int v) {
  v = max(v, __builtin_amdgcn_update_dpp(INT32_MIN, v, 0xB1, 0xF, 0xF, false));   // lane ^ 1
  v = max(v, __builtin_amdgcn_update_dpp(INT32_MIN, v, 0x4E, 0xF, 0xF, false));   // lane ^ 2
  v = max(v, __builtin_amdgcn_update_dpp(INT32_MIN, v, 0x141, 0xF, 0xF, false));  // row_half_mirror
  v = max(v, __builtin_amdgcn_update_dpp(INT32_MIN, v, 0x140, 0xF, 0xF, false));  // row_mirror
  if (LPR >= 32) v = max(v, __shfl_xor(v, 16, 64));
  if (LPR >= 64) v = max(v, __shfl_xor(v, 32, 64));
  return v;
}
template <int LPR> __device__ __forceinline__ float group_sum_f(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
  if (LPR >= 32) v += __shfl_xor(v, 16, 64);
  if (LPR >= 64) v += __shfl_xor(v, 32, 64);
  return v;
}
template <int LPR> __device__ __forceinline__ double group_max_d(double v) {
#pragma unroll
  for (int m = 1; m < LPR; m <<= 1) v = fmax(v, __shfl_xor(v, m, 64));
  return v;
}

// F64CODE: the code's pre-round value 2 (log2 sum - (t_j - t_max) + log2 s) is formed in float64 (used for more than
// 6 bits, where a float32 product could move ~3e-5 of the codes across a rounding boundary); otherwise one float32
// fma.  Rounding to nearest-even, saturation at 0 and byte packing are one v_cvt_pk_u8_f32 per code either way.
template <int LPR, int MAXNV, bool HAS_BIAS, bool F64CODE>
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
  const float qmaxf = (float)p.qmax;
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
    tmax = group_max_d<LPR>(tmax);
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
        a[v][e] = ok ? a[v][e] : INT32_MIN;          // masked and padding keys
        amax = max(amax, a[v][e]);
      }
    }
    amax = group_max_i<LPR>(amax);
#pragma unroll
    for (int v = 0; v < MAXNV; ++v)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        // acc - amax <= 0; INT32_MIN - amax wraps only if amax > 0, to a large positive value, so clamp the masked ones
        const int d = a[v][e] == INT32_MIN ? -0x40000000 : a[v][e] - amax;
        a[v][e] = d;
        ssum += __builtin_amdgcn_exp2f((float)d * c1f);   // exp2(-huge) = 0
      }
  }
  ssum = group_sum_f<LPR>(ssum);
  // code = rint(2 * (log2(sum) - (t_j - t_max) + log2 s))
  const double C0 = 2.0 * ((double)__builtin_amdgcn_logf(ssum) + p.log2s);
  const double m2c = -2.0 * p.c1;
  const float C0f = (float)C0, m2cf = (float)m2c;

  if (!live) return;
  uint8_t* crow = p.codes + row * p.ld;
#pragma unroll
  for (int v = 0; v < MAXNV; ++v) {
    const int c = sub + v * LPR;
    if (c < chunks) {
      unsigned w = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float vf;
        if (HAS_BIAS) {
          const int j = c * 4 + e;
          vf = j < limit ? (float)rint(fma(t[v * 4 + e] - tmax, -2.0, C0)) : qmaxf;
        } else if (F64CODE) {
          vf = (float)rint(fma((double)a[v][e], m2c, C0));       // masked keys: huge positive -> saturates at qmax below
        } else {
          vf = fmaf((float)a[v][e], m2cf, C0f);
        }
        vf = fminf(vf, qmaxf);
        if (e == 0) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 0, w);
        if (e == 1) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 1, w);
        if (e == 2) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 2, w);
        if (e == 3) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 3, w);
      }
      *reinterpret_cast<unsigned*>(crow + c * 4) = w;
    }
  }
}

template <int LPR, int MAXNV>
void launch(rq_ctx* ctx, const SmParams& p, bool has_bias) {
  const int64_t rows_per_block = 4 * (64 / LPR);
  const unsigned blocks = (unsigned)((p.rows + rows_per_block - 1) / rows_per_block);
  if (has_bias) hipLaunchKernelGGL((softmax_kernel<LPR, MAXNV, true, true>), dim3(blocks), dim3(256), 0, ctx->stream, p);
  else if (p.qmax > 63) hipLaunchKernelGGL((softmax_kernel<LPR, MAXNV, false, true>), dim3(blocks), dim3(256), 0, ctx->stream, p);
  else hipLaunchKernelGGL((softmax_kernel<LPR, MAXNV, false, false>), dim3(blocks), dim3(256), 0, ctx->stream, p);
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
