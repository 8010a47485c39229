// Device code shared by the translation units of the weight-mode integer GEMM (rq_qgemm).
#pragma once

#include "rq_internal.h"

namespace rqg {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct GemmParams {
  int64_t M;
  int N, K;
  const int8_t* A;
  int64_t lda;
  const uint8_t* B;
  int64_t ldb;
  const float* s_b;
  const int32_t* z_b;
  const int32_t* colsum_b;
  const int32_t* rowsum_a;
  const float* bias;
  float s_a;
  int da;        // a_off - z_a
  int centered;  // weights stored code - 128: needs (128 - z_b[n]) * rowsum_a[m]
  int act;
  const float* residual;
  int64_t ldr;
  int32_t* out_acc;
  int64_t ldacc;
  float* out_f32;
  int64_t ldf;
  int8_t* out_q;
  int64_t ldq;
  int n_seg, seg_len;
  double inv_so_d[4];   // 1 / s_o in float64 (the exact re-decision of codes near rounding ties)
  float inv_so[4];
  float zo[4];   // z_o - off_o
  float zcode[4];   // z_o
  float qmaxf;
  int off4[4];   // off_o replicated in the four bytes
  int lo[4], hi[4];
  int tiles_m, tiles_n;
  int group_m;      // tile rows walked together: consecutive tiles go down group_m rows before they move to the next column
  int force_rows;   // host only: 64-row groups per tile to take wherever that tile exists (0: choose by shape)
  int no_raw;       // host only: 1 = packed 4-bit weights keep the zero-point subtraction in the unpack even when row sums are
                    // given, -1 = raw nibbles whenever they are given (default: only with a long K loop)
};

__device__ __forceinline__ int swz(int row, int c) {
  return (row >> 1) * 128 + (((((row & 1) << 2) | c) ^ ((row >> 1) & 7)) << 4);
}

// GELU(y) = y Phi(y) = max(y, 0) - |y| erfc(|y| / sqrt 2) / 2.  log2(erfc(a / sqrt 2) / 2) is smooth and close to a parabola;
// a degree-6 polynomial (weighted least squares on [0, 6.5], where the product with |y| matters) reproduces GELU to 2.6e-7
// absolute in float32 -- the same as a rational erf, with one exp2 and no reciprocal.  Beyond 6.5 the term is below 1e-9 |y|.
#define RQ_FMAAK(d, s0, s1, HEX) asm("v_fmaak_f32 %0, %1, %2, " HEX : "=v"(d) : "v"(s0), "v"(s1))
__device__ __forceinline__ float gelu_f(float y) {
  const float ay = fabsf(y);
  const float a = fminf(ay, 6.5f);
  float p = fmaf(3.204148336e-05f, a, -7.530309838e-04f);
  // Horner steps as v_fmaak_f32 (d = s0 * s1 + literal), one instruction each: left to itself the compiler turns about a
  // third of them into a v_mov of the constant plus a v_fmac.  Same fused multiply-add, same rounding.
  RQ_FMAAK(p, p, a, "0x3c03246a");     //  8.004287203e-03
  RQ_FMAAK(p, p, a, "0xbd5a230b");     // -5.325607760e-02
  RQ_FMAAK(p, p, a, "0xbeeaf763");     // -4.589186652e-01
  RQ_FMAAK(p, p, a, "0xbf935899");     // -1.151141279e+00
  RQ_FMAAK(p, p, a, "0xbf800008");     // -1.000001008e+00
  return fmaf(-ay, __builtin_amdgcn_exp2f(p), fmaxf(y, 0.f));
}

// Re-quantization of 8-bit codes: the float32 epilogue carries up to ~1e-4 of a code of rounding error, enough to flip a
// code whose exact value sits that close to a rounding tie -- and a flipped Q or K code can move the winning key of a
// peaked attention row.  Outputs whose float32 pre-round value lies within TIE_GUARD of a tie are therefore decided again in
// float64, in the order the definition states: y = acc * (s_a * s_w[n]) + bias[n] (+ residual), code = round(y / s_o) + z_o
// (the division as a product with the float64 reciprocal: one more rounding of 1e-16).  Inlined: a call from the epilogue
// would park the accumulators in scratch memory.
// (Narrower codes: |value| <= 127 keeps the float32 error below 4e-6 of a code, flips stay inside the tolerated 1e-4 of the
// elements at no cost; activation epilogues feed the MLP, where a flipped code moves one output by one step and no more.)
constexpr float TIE_GUARD = 1.0f / 4096.0f;
__device__ __forceinline__ unsigned requant_exact4(const GemmParams& p, int t0, int t1, int t2, int t3, int n, float r0, float r1, float r2,
                                                   float r3, int seg) {
  const int t[4] = {t0, t1, t2, t3};
  const float r[4] = {r0, r1, r2, r3};
  const double iso = p.inv_so_d[seg], zc = (double)p.zcode[seg], qm = (double)p.qmaxf, sa = (double)p.s_a;
  unsigned w = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int ne = n + e < p.N ? n + e : p.N - 1;
    double y = (double)t[e] * (sa * (double)p.s_b[ne]) + (p.bias ? (double)p.bias[ne] : 0.0);
    y += (double)r[e];
    const double c = fmin(fmax(rint(y * iso) + zc, 0.0), qm);
    w |= (unsigned)(int)c << (8 * e);
  }
  return w;
}

__device__ __forceinline__ float silu_f(float y) {
  return y * __frcp_rn(1.0f + __builtin_amdgcn_exp2f(y * -1.4426950408889634f));
}

// Accumulators start at the zero-point corrections:
//   true = sum a'w' + (a_off - z_a) * colsum_w[n] + (128 - z_w[n]) * rowsum_a'[m]   (second term only for centered weights)
template <int TM, int TN>
__device__ __forceinline__ void init_acc(const GemmParams& p, v16i (&acc)[TN][TM], int64_t m0, int n0, int wm0, int wn0, int lane) {
  const int lcol = lane & 31, lrow4 = (lane >> 5) * 4;
  const bool need_cs = p.da != 0 && p.colsum_b;
  if (!need_cs && !p.centered) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][i][e] = 0;
    return;
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int n = n0 + wn0 + j * 32 + 8 * (e >> 2) + lrow4 + (e & 3);
      n = n < p.N ? n : p.N - 1;
      const int cs = need_cs ? p.da * p.colsum_b[n] : 0;
      const int dw = p.centered ? 128 - p.z_b[n] : 0;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        int64_t m = m0 + wm0 + i * 32 + lcol;
        m = m < p.M ? m : p.M - 1;
        acc[j][i][e] = cs + (p.centered ? dw * p.rowsum_a[m] : 0);
      }
    }
  }
}

// Epilogue: for MFMA tile (j, i) and e-group g the lane holds output channels n..n+3 of token m.
template <int TM, int TN>
__device__ __forceinline__ void epilogue(const GemmParams& p, v16i (&acc)[TN][TM], int64_t m0, int n0, int wm0, int wn0, int lane) {
  const int lcol = lane & 31, lrow4 = (lane >> 5) * 4;
  const bool gated = p.act == RQ_ACT_SILU_GATED;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    if (gated && (j & 1)) continue;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int n = n0 + wn0 + j * 32 + 8 * g + lrow4;
      if (n >= p.N) continue;
      float4 sc = *reinterpret_cast<const float4*>(p.s_b + n);
      sc.x *= p.s_a; sc.y *= p.s_a; sc.z *= p.s_a; sc.w *= p.s_a;
      const float4 bi = p.bias ? *reinterpret_cast<const float4*>(p.bias + n) : make_float4(0.f, 0.f, 0.f, 0.f);
      float4 sc2 = sc, bi2 = bi;
      int no = n;   // output column
      if (gated) {
        sc2 = *reinterpret_cast<const float4*>(p.s_b + n + 32);
        sc2.x *= p.s_a; sc2.y *= p.s_a; sc2.z *= p.s_a; sc2.w *= p.s_a;
        bi2 = p.bias ? *reinterpret_cast<const float4*>(p.bias + n + 32) : make_float4(0.f, 0.f, 0.f, 0.f);
        no = (n0 + wn0 + j * 32) / 2 + 8 * g + lrow4;
      }
      const int sg = (p.out_q && p.n_seg > 1) ? no / p.seg_len : 0;
      const float is = p.inv_so[sg], zz = p.zo[sg];
      const int lo = p.lo[sg], hi = p.hi[sg];
      const bool guard = p.out_q && p.act == RQ_ACT_NONE && p.qmaxf > 127.f;     // 8-bit codes: see TIE_GUARD
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int64_t m = m0 + wm0 + i * 32 + lcol;
        if (m >= p.M) continue;
        if (p.out_acc) {
          v4i t = {acc[j][i][4 * g], acc[j][i][4 * g + 1], acc[j][i][4 * g + 2], acc[j][i][4 * g + 3]};
          *reinterpret_cast<v4i*>(p.out_acc + m * p.ldacc + n) = t;
        }
        float y[4];
        y[0] = fmaf((float)acc[j][i][4 * g + 0], sc.x, bi.x);
        y[1] = fmaf((float)acc[j][i][4 * g + 1], sc.y, bi.y);
        y[2] = fmaf((float)acc[j][i][4 * g + 2], sc.z, bi.z);
        y[3] = fmaf((float)acc[j][i][4 * g + 3], sc.w, bi.w);
        if (p.act == RQ_ACT_GELU) {
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] = gelu_f(y[e]);
        } else if (gated) {
          constexpr int J1 = TN > 1 ? 1 : 0;
          const int ju = (j + J1) < TN ? (j + J1) : j;
          const float u0 = fmaf((float)acc[ju][i][4 * g + 0], sc2.x, bi2.x);
          const float u1 = fmaf((float)acc[ju][i][4 * g + 1], sc2.y, bi2.y);
          const float u2 = fmaf((float)acc[ju][i][4 * g + 2], sc2.z, bi2.z);
          const float u3 = fmaf((float)acc[ju][i][4 * g + 3], sc2.w, bi2.w);
          y[0] = silu_f(y[0]) * u0; y[1] = silu_f(y[1]) * u1; y[2] = silu_f(y[2]) * u2; y[3] = silu_f(y[3]) * u3;
        }
        float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
        if (p.residual) {
          r = *reinterpret_cast<const float4*>(p.residual + m * p.ldr + no);
          y[0] += r.x; y[1] += r.y; y[2] += r.z; y[3] += r.w;
        }
        if (p.out_f32) *reinterpret_cast<float4*>(p.out_f32 + m * p.ldf + no) = make_float4(y[0], y[1], y[2], y[3]);
        if (p.out_q) {
          int c[4];
          bool near_tie = false;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float v = y[e] * is;
            const float rv = __builtin_rintf(v);
            near_tie |= fabsf(v - rv) > 0.5f - TIE_GUARD;
            int k = (int)(rv + zz);
            c[e] = k < lo ? lo : (k > hi ? hi : k);
          }
          if (guard && near_tie) {
            const unsigned w = requant_exact4(p, acc[j][i][4 * g], acc[j][i][4 * g + 1], acc[j][i][4 * g + 2], acc[j][i][4 * g + 3], n, r.x,
                                              r.y, r.z, r.w, sg);
            const int off = (int)p.zcode[sg] - (int)p.zo[sg];      // the storage offset
#pragma unroll
            for (int e = 0; e < 4; ++e) c[e] = (int)((w >> (8 * e)) & 0xFFu) - off;
          }
          *reinterpret_cast<int*>(p.out_q + m * p.ldq + no) = rq_pack4(c[0], c[1], c[2], c[3]);
        }
      }
    }
  }
}

// 4-bit unpack of 16 packed bytes (32 codes, interleaved so that `& 0x0F0F0F0F` and `>> 4 & 0x0F0F0F0F` give 4 consecutive
// codes each) into two 16-byte int8 chunks with the zero-point subtracted: ((x | 0x80) - z) ^ 0x80 is x - z per byte.
__device__ __forceinline__ void unpack_u4(const v4i& pk, int z4, v4i& c0, v4i& c1) {
  int lo, hi;
  lo = pk[0] & 0x0F0F0F0F; hi = (pk[0] >> 4) & 0x0F0F0F0F;
  c0[0] = ((lo | 0x80808080) - z4) ^ 0x80808080; c0[1] = ((hi | 0x80808080) - z4) ^ 0x80808080;
  lo = pk[1] & 0x0F0F0F0F; hi = (pk[1] >> 4) & 0x0F0F0F0F;
  c0[2] = ((lo | 0x80808080) - z4) ^ 0x80808080; c0[3] = ((hi | 0x80808080) - z4) ^ 0x80808080;
  lo = pk[2] & 0x0F0F0F0F; hi = (pk[2] >> 4) & 0x0F0F0F0F;
  c1[0] = ((lo | 0x80808080) - z4) ^ 0x80808080; c1[1] = ((hi | 0x80808080) - z4) ^ 0x80808080;
  lo = pk[3] & 0x0F0F0F0F; hi = (pk[3] >> 4) & 0x0F0F0F0F;
  c1[2] = ((lo | 0x80808080) - z4) ^ 0x80808080; c1[3] = ((hi | 0x80808080) - z4) ^ 0x80808080;
}


}  // namespace rqg
