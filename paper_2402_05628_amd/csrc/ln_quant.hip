// rq_ln_quant: LayerNorm / RMSNorm with the folded affine, fused with the layer-wise uniform quantizer
// (Section "Scale reparameterization for LayerNorm activations"; quantizer of Section "Efficient quantizers").
//
// HBM-bound: 4 B read + 1 B written per element.  One row is held in the registers of LPR lanes
// (LPR = 16, 32 or 64 lanes of a 64-wide wavefront); the row statistics are wavefront shuffles; the
// codes leave as one dword (4 codes) per lane, contiguous across lanes.  All arithmetic is float64:
// fp64 runs at the fp32 rate on this chip and the kernel has ALU headroom, so the codes agree with a
// float64 reference except at exact ties.  The next row is fetched while the current one is quantized.
#include <vector>

#include "rq_internal.h"

namespace {

template <int LPR, int NV, bool REG_AFFINE>
__global__ __launch_bounds__(256) void ln_quant_kernel(
    const float* __restrict__ x, int64_t ldx, int64_t T, int D, int norm_kind, double eps,
    const float* __restrict__ gamma_t, const float* __restrict__ beta_t, double inv_s, double zshift,
    int lo, int hi, int8_t* __restrict__ q, int64_t ldq, int32_t* __restrict__ rowsum) {
  constexpr int RPW = 64 / LPR;                 // rows per wavefront
  const int lane = threadIdx.x & 63;
  const int sub = lane % LPR;                   // lane within the row
  const int rsel = lane / LPR;                  // which of the wavefront's rows
  const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int64_t nwave = (int64_t)gridDim.x * (blockDim.x >> 6);
  const int chunks = D >> 2;

  // g = gamma~/s~, h = beta~/s~ + z~ - store_off for this lane's channels
  double g[REG_AFFINE ? NV * 4 : 1], h[REG_AFFINE ? NV * 4 : 1];
  if (REG_AFFINE) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = sub + i * LPR;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int ch = c * 4 + e;
        const bool ok = c < chunks;
        g[i * 4 + e] = ok ? (double)gamma_t[ch] * inv_s : 0.0;
        h[i * 4 + e] = ok ? (beta_t ? (double)beta_t[ch] * inv_s : 0.0) + zshift : 0.0;
      }
    }
  }

  float4 cur[NV], nxt[NV];
  int64_t row = wave * RPW + rsel;
  const int64_t stride = nwave * RPW;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = sub + i * LPR;
    cur[i] = (row < T && c < chunks) ? *reinterpret_cast<const float4*>(x + row * ldx + c * 4) : make_float4(0, 0, 0, 0);
  }
  const double invD = 1.0 / (double)D;
  for (; (row - rsel) < T; row += stride) {       // wavefront-uniform trip count
    const int64_t nrow = row + stride;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = sub + i * LPR;
      nxt[i] = (nrow < T && c < chunks) ? *reinterpret_cast<const float4*>(x + nrow * ldx + c * 4) : make_float4(0, 0, 0, 0);
    }
    double s1 = 0.0, s2 = 0.0;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const double a = cur[i].x, b = cur[i].y, c = cur[i].z, d = cur[i].w;
      s1 += (a + b) + (c + d);
      s2 = fma(a, a, s2); s2 = fma(b, b, s2); s2 = fma(c, c, s2); s2 = fma(d, d, s2);
    }
#pragma unroll
    for (int m = 1; m < LPR; m <<= 1) {
      s1 += __shfl_xor(s1, m, 64);
      s2 += __shfl_xor(s2, m, 64);
    }
    double mean, var;
    if (norm_kind == RQ_NORM_LAYERNORM) {
      mean = s1 * invD;
      var = fma(-mean, mean, s2 * invD);
      var = var < 0.0 ? 0.0 : var;
    } else {
      mean = 0.0;
      var = s2 * invD;
    }
    const double rstd = 1.0 / sqrt(var + eps);
    const double nmr = -mean * rstd;
    int rs = 0;
    if (row < T) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = sub + i * LPR;
        if (c < chunks) {
          const float xv[4] = {cur[i].x, cur[i].y, cur[i].z, cur[i].w};
          int code[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            double gg, hh;
            if (REG_AFFINE) {
              gg = g[i * 4 + e];
              hh = h[i * 4 + e];
            } else {
              const int ch = c * 4 + e;
              gg = (double)gamma_t[ch] * inv_s;
              hh = (beta_t ? (double)beta_t[ch] * inv_s : 0.0) + zshift;
            }
            const double xh = fma((double)xv[e], rstd, nmr);
            const double v = fma(xh, gg, hh);
            int k = (int)rint(v);
            k = k < lo ? lo : (k > hi ? hi : k);
            code[e] = k;
            rs += k;
          }
          *reinterpret_cast<int*>(q + row * ldq + c * 4) = rq_pack4(code[0], code[1], code[2], code[3]);
        }
      }
    }
    if (rowsum) {
#pragma unroll
      for (int m = 1; m < LPR; m <<= 1) rs += __shfl_xor(rs, m, 64);
      if (sub == 0 && row < T) rowsum[row] = rs;
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) cur[i] = nxt[i];
  }
}

template <int LPR, int NV>
void launch(rq_ctx* ctx, const rq_ln_desc* d, double inv_s, double zshift, int lo, int hi) {
  constexpr int RPW = 64 / LPR;
  constexpr bool REG = NV <= 4;
  const int64_t rows_per_block = 4 * RPW;
  int64_t blocks = (d->T + rows_per_block - 1) / rows_per_block;
  const int64_t cap = (int64_t)ctx->num_cu * 8;
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL((ln_quant_kernel<LPR, NV, REG>), dim3((unsigned)blocks), dim3(256), 0, ctx->stream, d->x, d->ldx, d->T,
                     d->D, d->norm_kind, d->eps, d->gamma_t, d->beta_t, inv_s, zshift, lo, hi, d->q, d->ldq, d->rowsum);
}

}  // namespace

rq_status rq_launch_ln_quant(rq_ctx* ctx, const rq_ln_desc* d) {
  const int chunks = d->D / 4;
  const double inv_s = 1.0 / (double)d->s_tilde;
  const double zshift = (double)d->z_tilde - (double)d->store_off;
  const int lo = -d->store_off, hi = (1 << d->bits) - 1 - d->store_off;
  int lpr;
  if (chunks % 64 == 0 || chunks > 128) lpr = 64;
  else if (chunks % 32 == 0 || chunks > 64) lpr = 32;
  else lpr = 16;
  const int nv = (chunks + lpr - 1) / lpr;
#define RQ_LN_CASE(L, N)                                  \
  if (lpr == L && nv <= N) {                              \
    launch<L, N>(ctx, d, inv_s, zshift, lo, hi);          \
    RQ_HIP(hipGetLastError());                            \
    return RQ_OK;                                         \
  }
  RQ_LN_CASE(16, 1) RQ_LN_CASE(16, 2) RQ_LN_CASE(16, 4)
  RQ_LN_CASE(32, 1) RQ_LN_CASE(32, 2) RQ_LN_CASE(32, 3) RQ_LN_CASE(32, 4)
  RQ_LN_CASE(64, 2) RQ_LN_CASE(64, 3) RQ_LN_CASE(64, 4) RQ_LN_CASE(64, 8) RQ_LN_CASE(64, 16) RQ_LN_CASE(64, 32)
#undef RQ_LN_CASE
  return rq_fail(ctx, RQ_ERR_SHAPE, "rq_ln_quant: D = %d exceeds the supported 8192", d->D);
}
