// Pipelined weight-mode GEMM kernel (256 x 128 tiles, asynchronous global->LDS ring) and its epilogue.
// Included by the per-format instantiation units.
#pragma once

#include <type_traits>

#include "qgemm_common.h"

namespace rqg {

// Per-column epilogue constants.  They are fetched at kernel start (one column per thread), parked in registers
// over the main loop and handed over through the start of the then-idle LDS ring, so that no global or scalar
// memory latency sits in front of the first output of a tile.
template <int BN>
struct EpiLdsT {
  float scale[BN];      // s_a * s_w[n]
  float bias[BN];
  int cs[BN];           // (a_off - z_a) * colsum_w[n]
  int dw[BN];           // 128 - z_w[n] for centered weights, else 0
  float is[BN];         // 1 / s_o of the output column's re-quantization segment
  float zz[BN];         // z_o of that segment
  int off4[BN];         // storage offset of that segment replicated in 4 bytes
};
typedef EpiLdsT<128> EpiLds;

enum { OUT_ACC = 1, OUT_F32 = 2, OUT_RES = 4, OUT_Q = 8, OUT_ANY = 15 };

// Epilogue: for MFMA tile (j, i) and e-group g the lane holds output channels n..n+3 of token m.
//  * OUT selects the outputs at compile time (OUT_ANY: decided by the pointers at run time), CHECK the row bound;
//  * v_cvt_pk_u8_f32 rounds to nearest-even, saturates to 0..255 and packs in one instruction; two
//    v_permlane32_swap exchange dwords between lane l and lane l+32 (which hold interleaved groups of 4 channels of
//    the same token) so that each lane owns 16 consecutive channels and issues one 16-byte store.
//  * Q8 (a separate kernel instantiation, so that narrower codes carry none of its code or registers): 8-bit output codes
//    without an activation are guarded against rounding ties, see TIE_GUARD.
template <int TM, int TN, int ACT, int OUT, bool CHECK, typename EL = EpiLds, bool Q8 = false>
__device__ __forceinline__ void epilogue_wide(const GemmParams& p, v16i (&acc)[TN][TM], const EL* el, const int (&rs)[TM],
                                              int m0, int n0, int wm0, int wn0, int lane) {
  const int lcol = lane & 31, half = lane >> 5, lrow4 = half * 4;
  constexpr bool gated = ACT == RQ_ACT_SILU_GATED;
  constexpr bool FOLD = OUT == OUT_Q && ACT == RQ_ACT_NONE;      // el->scale / el->bias hold the folded constants A, B (see the kernel)
  // everything the stores need, read from the kernel arguments once
  int32_t* const out_acc = (OUT & OUT_ACC) ? p.out_acc : nullptr;
  float* const out_f32 = (OUT & OUT_F32) ? p.out_f32 : nullptr;
  const float* const residual = (OUT & OUT_RES) ? p.residual : nullptr;
  int8_t* const out_q = (OUT & OUT_Q) ? p.out_q : nullptr;
  const bool has_acc = (OUT & OUT_ACC) && (OUT != OUT_ANY || out_acc);
  const bool has_f32 = (OUT & OUT_F32) && (OUT != OUT_ANY || out_f32);
  const bool has_res = (OUT & OUT_RES) && (OUT != OUT_ANY || residual);
  const bool has_q = (OUT & OUT_Q) && (OUT != OUT_ANY || out_q);
  const int64_t ldacc = p.ldacc, ldf = p.ldf, ldr = p.ldr, ldq = p.ldq;
  const int Mi = (int)p.M;
  const float qm = p.qmaxf;
  const bool wide_codes = qm > 127.f;      // 8-bit output codes
  const bool wide_q = has_q && (ldq & 15) == 0 && (reinterpret_cast<uintptr_t>(out_q) & 15) == 0;
  const bool corr = p.da != 0 || p.centered;
  // row bases of this lane's TM tokens
  int32_t* racc[TM]; float* rf32[TM]; const float* rres[TM]; int8_t* rq[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int64_t m = m0 + wm0 + i * 32 + lcol;
    racc[i] = has_acc ? out_acc + m * ldacc : nullptr;
    rf32[i] = has_f32 ? out_f32 + m * ldf : nullptr;
    rres[i] = has_res ? residual + m * ldr : nullptr;
    rq[i] = has_q ? out_q + m * ldq : nullptr;
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    if (gated && (j & 1)) continue;
    const int nb = n0 + wn0 + j * 32;              // first weight row of this MFMA tile
    if (nb >= p.N) continue;                       // N is a multiple of 32 here (checked by the launcher)
    const int nob = gated ? nb / 2 : nb;           // first output column
    unsigned pk[TM][4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int nl = wn0 + j * 32 + 8 * g + lrow4;   // weight row within the tile
      const int nlo = gated ? (wn0 + j * 32) / 2 + 8 * g + lrow4 : nl;   // output column within the tile's outputs
      const int n = n0 + nl;
      const int no = nob + 8 * g + lrow4;
      const float4 sc = *reinterpret_cast<const float4*>(&el->scale[nl]);
      const float4 bi = *reinterpret_cast<const float4*>(&el->bias[nl]);
      float4 sc2 = sc, bi2 = bi;
      if (gated) {
        sc2 = *reinterpret_cast<const float4*>(&el->scale[nl + 32]);
        bi2 = *reinterpret_cast<const float4*>(&el->bias[nl + 32]);
      }
      float is = 0.f, zz = 0.f;
      unsigned o4 = 0;
      if (has_q) { is = el->is[nlo]; zz = el->zz[nlo]; o4 = (unsigned)el->off4[nlo]; }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm0 + i * 32 + lcol;
        const bool live = !CHECK || m < Mi;
        int t[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = acc[j][i][4 * g + e];
        if (corr) {      // the correction constants are read inside the branch: no registers, no zeroing without it
          const v4i cs = *reinterpret_cast<const v4i*>(&el->cs[nl]), dw = *reinterpret_cast<const v4i*>(&el->dw[nl]);
#pragma unroll
          for (int e = 0; e < 4; ++e) t[e] += cs[e] + dw[e] * rs[i];
        }
        if (has_acc && live) {
          v4i tv = {t[0], t[1], t[2], t[3]};
          *reinterpret_cast<v4i*>(racc[i] + n) = tv;
        }
        float y[4];
        y[0] = fmaf((float)t[0], sc.x, bi.x);
        y[1] = fmaf((float)t[1], sc.y, bi.y);
        y[2] = fmaf((float)t[2], sc.z, bi.z);
        y[3] = fmaf((float)t[3], sc.w, bi.w);
        if (ACT == RQ_ACT_GELU) {
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] = gelu_f(y[e]);
        } else if (gated) {
          constexpr int J1 = TN > 1 ? 1 : 0;
          const int ju = (j + J1) < TN ? (j + J1) : j;
          int u[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) u[e] = acc[ju][i][4 * g + e];
          if (corr) {
            const v4i cs2 = *reinterpret_cast<const v4i*>(&el->cs[nl + 32]), dw2 = *reinterpret_cast<const v4i*>(&el->dw[nl + 32]);
#pragma unroll
            for (int e = 0; e < 4; ++e) u[e] += cs2[e] + dw2[e] * rs[i];
          }
          y[0] = silu_f(y[0]) * fmaf((float)u[0], sc2.x, bi2.x);
          y[1] = silu_f(y[1]) * fmaf((float)u[1], sc2.y, bi2.y);
          y[2] = silu_f(y[2]) * fmaf((float)u[2], sc2.z, bi2.z);
          y[3] = silu_f(y[3]) * fmaf((float)u[3], sc2.w, bi2.w);
        }
        float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
        if (has_res && live) {
          r = *reinterpret_cast<const float4*>(rres[i] + no);
          y[0] += r.x; y[1] += r.y; y[2] += r.z; y[3] += r.w;
        }
        if (has_f32 && live) *reinterpret_cast<float4*>(rf32[i] + no) = make_float4(y[0], y[1], y[2], y[3]);
        if (has_q) {
          unsigned w = 0;
          if (FOLD && Q8) {      // y is the pre-round code already; the same guard with the tie distance added to it
            unsigned wl = 0;
            w = __builtin_amdgcn_cvt_pk_u8_f32(y[0] + TIE_GUARD, 0, w);
            w = __builtin_amdgcn_cvt_pk_u8_f32(y[1] + TIE_GUARD, 1, w);
            w = __builtin_amdgcn_cvt_pk_u8_f32(y[2] + TIE_GUARD, 2, w);
            w = __builtin_amdgcn_cvt_pk_u8_f32(y[3] + TIE_GUARD, 3, w);
            wl = __builtin_amdgcn_cvt_pk_u8_f32(y[0] - TIE_GUARD, 0, wl);
            wl = __builtin_amdgcn_cvt_pk_u8_f32(y[1] - TIE_GUARD, 1, wl);
            wl = __builtin_amdgcn_cvt_pk_u8_f32(y[2] - TIE_GUARD, 2, wl);
            wl = __builtin_amdgcn_cvt_pk_u8_f32(y[3] - TIE_GUARD, 3, wl);
            if (w != wl) {
              int sg = p.n_seg > 1 ? no / p.seg_len : 0;
              sg = sg < p.n_seg ? sg : p.n_seg - 1;
              w = requant_exact4(p, t[0], t[1], t[2], t[3], n, r.x, r.y, r.z, r.w, sg);
            }
          } else if (FOLD) {
            w = __builtin_amdgcn_cvt_pk_u8_f32(fminf(y[0], qm), 0, w);
            w = __builtin_amdgcn_cvt_pk_u8_f32(fminf(y[1], qm), 1, w);
            w = __builtin_amdgcn_cvt_pk_u8_f32(fminf(y[2], qm), 2, w);
            w = __builtin_amdgcn_cvt_pk_u8_f32(fminf(y[3], qm), 3, w);
          } else if (Q8 && ACT == RQ_ACT_NONE) {      // 8-bit codes: the packed convert saturates at 255 by itself
            // the codes taken TIE_GUARD above and below agree unless the value sits that close to a rounding tie
            const float zp = zz + TIE_GUARD, zm = zz - TIE_GUARD;
            unsigned wl = 0;
            w = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(y[0], is, zp), 0, w);
            w = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(y[1], is, zp), 1, w);
            w = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(y[2], is, zp), 2, w);
            w = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(y[3], is, zp), 3, w);
            wl = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(y[0], is, zm), 0, wl);
            wl = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(y[1], is, zm), 1, wl);
            wl = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(y[2], is, zm), 2, wl);
            wl = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(y[3], is, zm), 3, wl);
            if (w != wl) {
              int sg = p.n_seg > 1 ? no / p.seg_len : 0;
              sg = sg < p.n_seg ? sg : p.n_seg - 1;
              w = requant_exact4(p, t[0], t[1], t[2], t[3], n, r.x, r.y, r.z, r.w, sg);
            }
          } else {
          w = __builtin_amdgcn_cvt_pk_u8_f32(fminf(fmaf(y[0], is, zz), qm), 0, w);
          w = __builtin_amdgcn_cvt_pk_u8_f32(fminf(fmaf(y[1], is, zz), qm), 1, w);
          w = __builtin_amdgcn_cvt_pk_u8_f32(fminf(fmaf(y[2], is, zz), qm), 2, w);
          w = __builtin_amdgcn_cvt_pk_u8_f32(fminf(fmaf(y[3], is, zz), qm), 3, w);
          }
          // stored = code - off per byte.  Codes of 8 bits are stored with offset 128 (nothing else fits int8): flip the sign
          // bits.  Narrower codes leave bit 7 free: with it set no byte borrows from its neighbour (off <= 128).
          w = wide_codes ? w ^ 0x80808080u : ((w | 0x80808080u) - o4) ^ 0x80808080u;
          pk[i][g] = w;
          if (!wide_q && live) *reinterpret_cast<unsigned*>(rq[i] + no) = w;
        }
      }
    }
    if (wide_q) {
      // lanes l (half 0) and l+32 (half 1) hold channel groups {0,8,16,24}+{0..3} and {4,12,20,28}+{0..3}:
      // after the two swaps lane l owns channels 0..15 and lane l+32 channels 16..31 of the same token
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm0 + i * 32 + lcol;
        auto s02 = __builtin_amdgcn_permlane32_swap(pk[i][0], pk[i][2], false, false);
        auto s13 = __builtin_amdgcn_permlane32_swap(pk[i][1], pk[i][3], false, false);
        if (!CHECK || m < Mi) {
          v4i tv = {(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
          *reinterpret_cast<v4i*>(rq[i] + nob + half * 16) = tv;
        }
      }
    }
  }
}

// Epilogue for float outputs with a residual (proj, FC2): y = s_a s_w[n] (acc + corrections) + b[n] + residual.
// In the accumulator layout a lane owns 4 consecutive channels of one token, so direct stores would touch 32-byte
// pieces of 32 different rows per instruction.  Each wavefront instead passes 32 x 64 outputs at a time through its
// own 8.5 KB of the idle ring (row pitch 68 floats: conflict-free both ways) and then reads, adds and writes whole
// 256-byte row segments, 16 lanes per row; the residual segments are requested before the LDS round trip.
template <int TM, int TN, bool CHECK, typename EL = EpiLds>
__device__ __forceinline__ void epilogue_rows_f32(const GemmParams& p, v16i (&acc)[TN][TM], const EL* el, const int (&rs)[TM],
                                                  float* stage, int m0, int n0, int wm0, int wn0, int lane) {
  static_assert(TN % 2 == 0, "64 output columns per wavefront and pass");
  constexpr int PITCH = 68;
  const int l32 = lane & 31, half = lane >> 5;
  const int rrow = lane >> 4, rcol = (lane & 15) * 4;        // read-back: 4 rows x 16 float4 per pass
  const bool corr = p.da != 0 || p.centered;
  const int Mi = (int)p.M;
  const float* const residual = p.residual;
  float* const out = p.out_f32;
  const int64_t ldr = p.ldr, ldf = p.ldf;
#pragma unroll
  for (int jh = 0; jh < TN; jh += 2) {       // 64 columns at a time
    const int ncol = n0 + wn0 + jh * 32 + rcol;
    const bool col_ok = ncol < p.N;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int mb = m0 + wm0 + i * 32;
      float4 res[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int m = mb + r * 4 + rrow;
        res[r] = (col_ok && (!CHECK || m < Mi)) ? *reinterpret_cast<const float4*>(residual + (int64_t)m * ldr + ncol)
                                                : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int j = jh + jj;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int nl = wn0 + j * 32 + 8 * g + half * 4;
          const float4 sc = *reinterpret_cast<const float4*>(&el->scale[nl]);
          const float4 bi = *reinterpret_cast<const float4*>(&el->bias[nl]);
          int t[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) t[e] = acc[j][i][4 * g + e];
          if (corr) {
            const v4i cs = *reinterpret_cast<const v4i*>(&el->cs[nl]);
            const v4i dw = *reinterpret_cast<const v4i*>(&el->dw[nl]);
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] += cs[e] + dw[e] * rs[i];
          }
          const float4 y = make_float4(fmaf((float)t[0], sc.x, bi.x), fmaf((float)t[1], sc.y, bi.y), fmaf((float)t[2], sc.z, bi.z),
                                       fmaf((float)t[3], sc.w, bi.w));
          *reinterpret_cast<float4*>(stage + l32 * PITCH + jj * 32 + 8 * g + half * 4) = y;
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // this wavefront's own writes; no other wavefront touches `stage`
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int m = mb + r * 4 + rrow;
        const float4 y = *reinterpret_cast<const float4*>(stage + (r * 4 + rrow) * PITCH + rcol);
        if (col_ok && (!CHECK || m < Mi))
          *reinterpret_cast<float4*>(out + (int64_t)m * ldf + ncol) = make_float4(y.x + res[r].x, y.y + res[r].y, y.z + res[r].z, y.w + res[r].w);
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // reads done before the next pass overwrites the region
    }
  }
}

// ---- pipelined kernel ------------------------------------------------------------------------------------------------
// One workgroup (4 wavefronts) owns one 256 x 128 output tile (wavefront tile 128 x 64) and walks K in steps of 64
// through an S-stage LDS ring.
//  * Every load is asynchronous and goes global -> LDS directly (global_load_lds_dwordx4: each lane deposits 16
//    bytes at ring_base + lane*16); no in-flight load is held in a register.  The bank swizzle of the int8 tiles is
//    applied on the GLOBAL side: lane l fetches the chunk that belongs at LDS slot l.  Row r (64 B) keeps its four
//    16-byte chunks rotated by (r >> 2), which makes the 32-row MFMA operand reads conflict-free.
//  * 4-bit weights stay PACKED in LDS (32 bytes per row and k-step); each lane reads the 16-byte packet that holds
//    its 32 codes of the k-step once and unpacks the nibbles in registers, zero-point subtracted, right before they
//    enter the MFMA (the k assignment gives lane half h the chunks 2h and 2h+1, so the packet is contiguous).
//  * Each activation fragment is refilled for the NEXT sub-step right after its own MFMAs are issued, so the LDS
//    latency hides behind the remaining MFMAs; the barrier + refill of the ring sit inside the second sub-step.
//  * One bare s_barrier per k-step (no fence: __syncthreads() would drain the asynchronous loads in flight).
// Two workgroups share a CU, so one runs its epilogue / prologue while the other feeds the matrix cores.  Tiles are
// dealt to the 8 XCDs in contiguous ranges (workgroup b runs on XCD b % 8) so that the tiles in flight on one XCD
// share activation rows and weight columns in that XCD's L2.
template <int R, class F> __device__ __forceinline__ void static_for_down(F&& f) {   // f(R), f(R-1), ..., f(0), each a constant
  if constexpr (R >= 0) {
    f(std::integral_constant<int, R>{});
    static_for_down<R - 1>(f);
  }
}

template <int N> __device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);   // vmcnt <= N, other counters unconstrained
}

// workgroups (= wavefronts per SIMD) a CU is meant to hold: bounds the registers the compiler may take
constexpr int pipe_occupancy(int TM, int OUT) {
  return TM <= 2 ? 4 : (TM == 3 ? 3 : (TM == 4 ? 2 : 1));
}
// the same for every tile shape: 256-column tiles and the eight-wavefront grid own their CU
constexpr int pipe_wgs_per_cu(int TM, int TN, int WN, int OUT) {
  return (TN == 4 || WN == 4) ? 1 : pipe_occupancy(TM, OUT);
}

// TN = 2: tiles 128 columns wide (wavefront tile 32 TM x 64); TN = 4: 256 columns (wavefront tile 32 TM x 128, one workgroup
// per CU): per MFMA half the bytes through the CU's load path and the LDS, for large products with a long K loop.
// WN = 4: eight wavefronts in a 2 x 4 grid (two per SIMD, each with the 32 TM x 32 TN tile) on a tile 32 TN * 4 columns wide:
// the operand bytes per MFMA of the 256 x 256 tile, with a second wavefront on every SIMD to cover the first one's waits.
// RAW (packed 4-bit weights with the row sums of the stored activations given): the nibbles enter the MFMA as the raw codes
// 0 .. 15 -- one AND per operand dword, one shift more for the high nibbles, instead of the byte-wise zero-point
// subtraction -- and the zero-point term -z_w[n] * rowsum_a[m] is what the accumulators START from:
//   sum_k a'[m,k] (code[n,k] - z_w[n]) = sum_k a'[m,k] code[n,k] - z_w[n] sum_k a'[m,k],
// the same exact integers.  It more than halves the vector instructions of the K loop.
template <bool W4, int S, int ACT, int OUT, int TM, int TN = 2, int WN = 2, bool Q8 = false, bool RAW = false>
__global__ __launch_bounds__(128 * WN, pipe_wgs_per_cu(TM, TN, WN, OUT)) void qgemm_pipe_kernel(const GemmParams p) {
  static_assert(!RAW || (W4 && TN == 2), "raw nibbles: packed weights, two column tiles per wavefront");
  constexpr int NT = 128 * WN;                        // threads: 2 x WN wavefronts
  constexpr int BM = 64 * TM, BN = 32 * TN * WN;      // TM = 4: 256-row tiles, two workgroups per CU; TM = 5: 320 rows, one
  constexpr int A_BYTES = BM * 64;
  constexpr int B_BYTES = W4 ? BN * 32 : BN * 64;
  constexpr int STAGE = A_BYTES + B_BYTES;
  constexpr int AL = BM * 4 / NT;                     // activation loads per thread and stage (16 bytes each)
  constexpr int BL = (W4 ? BN * 2 : BN * 4) / NT;     // weight loads per thread and stage
  static_assert(AL * NT == BM * 4 && BL >= 1, "the loads of a stage divide evenly over the threads");
  constexpr int LPS = AL + BL;                        // loads per thread and stage
  typedef EpiLdsT<BN> EL;
  constexpr int EPI_BYTES = BN == 128 ? 4096 : 8192;  // the epilogue constants at the start of the idle ring
  static_assert(sizeof(EL) <= EPI_BYTES, "epilogue constants");
  static_assert(S >= 2 && (S - 1) * LPS <= 63, "ring depth (the load counter holds 63)");
  extern __shared__ __align__(16) int8_t ring[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave / WN) * (32 * TM), wn0 = (wave % WN) * (32 * TN);
  const int l32 = lane & 31, half = lane >> 5;

  // tile of this workgroup: XCD b % 8 gets the contiguous range [xcd * per_xcd, ...) of the tile list (n fastest), i.e. a few
  // whole tile rows and every column.  (Cutting the tile grid into one rectangle of tile rows x tile columns per XCD, which
  // on paper halves the operand bytes an XCD's L2 pulls in for launches with few tile rows and many tile columns, measured
  // no faster -- 2048 x 12288 x 4096: 0.119 ms either way, 8192^3: 0.49 - 0.51 ms either way -- and raised the counted L2
  // fetches from 129 to 181 MB per launch at the first shape; it is not used.)
  const unsigned tiles_n = (unsigned)p.tiles_n;
  const unsigned ntiles = (unsigned)p.tiles_m * tiles_n;
  const unsigned per_xcd = (ntiles + 7u) / 8u;
  const unsigned t = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || t >= ntiles) return;
  // Within that range the tiles are walked in bands of group_m tile rows, down a band's rows first: the tiles that are
  // in flight on an XCD at one time then cover a block of rows x columns instead of one long row of tiles, and the
  // operand bytes its L2 has to pull in per k-step shrink accordingly.
  const unsigned band = (unsigned)p.group_m * tiles_n;
  const unsigned bi = t / band, br = t - bi * band;
  const unsigned first_m = bi * (unsigned)p.group_m;
  const unsigned left_m = (unsigned)p.tiles_m - first_m;
  const unsigned gm = left_m < (unsigned)p.group_m ? left_m : (unsigned)p.group_m;
  const unsigned tcol = br / gm;
  const int tm = (int)(first_m + (br - tcol * gm)), tn = (int)tcol;
  const int m0 = tm * BM, n0 = tn * BN;
  const int nk = p.K / 64;
  // ---- asynchronous loads: 32-bit byte offsets from the tensor bases (the launcher checks both are < 4 GiB) ----
  // lane l lands at 16-byte slot l of a 1 KB block = 16 tile rows of 64 B; the chunk that belongs at position
  // (lane & 3) of row (lane >> 2) is chunk ((lane & 3) - (row >> 2)) & 3
  unsigned aofs[AL], bofs[BL];
  {
    const int dl_row = lane >> 2;
    const int dl_c = ((lane & 3) - (dl_row >> 2)) & 3;
    const int Mi = (int)p.M;
#pragma unroll
    for (int i = 0; i < AL; ++i) {
      int m = m0 + (wave * AL + i) * 16 + dl_row;
      m = m < Mi ? m : Mi - 1;
      aofs[i] = (unsigned)m * (unsigned)p.lda + (unsigned)(dl_c * 16);
    }
    if (W4) {
#pragma unroll
      for (int u = 0; u < BL; ++u) {       // NT / 2 weight rows (32 bytes each) per load of the workgroup
        const int row = u * (NT / 2) + (tid >> 1);
        int n = n0 + row;
        n = n < p.N ? n : p.N - 1;
        bofs[u] = (unsigned)n * (unsigned)p.ldb + (unsigned)(((tid & 1) ^ ((row >> 3) & 1)) * 16);
      }
    } else {
#pragma unroll
      for (int i = 0; i < BL; ++i) {
        int n = n0 + wave * (16 * BL) + i * 16 + dl_row;
        n = n < p.N ? n : p.N - 1;
        bofs[i] = (unsigned)n * (unsigned)p.ldb + (unsigned)(dl_c * 16);
      }
    }
  }
  const int8_t* const gA = p.A;
  const uint8_t* const gB = p.B;
  auto issue = [&](int slot, int kt) {
    int8_t* la = ring + slot * STAGE;
    int8_t* lb = la + A_BYTES;
#pragma unroll
    for (int i = 0; i < AL; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gA + (aofs[i] + (unsigned)kt * 64u)),
                                       (__attribute__((address_space(3))) void*)(la + (wave * AL + i) * 1024), 16, 0, 0);
    if (W4) {
#pragma unroll
      for (int u = 0; u < BL; ++u)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gB + (bofs[u] + (unsigned)kt * 32u)),
                                         (__attribute__((address_space(3))) void*)(lb + u * (NT * 16) + wave * 1024), 16, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < BL; ++i)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gB + (bofs[i] + (unsigned)kt * 64u)),
                                         (__attribute__((address_space(3))) void*)(lb + (wave * BL + i) * 1024), 16, 0, 0);
    }
  };
  // The weight zero-points are needed by the first unpack.  Loads return in order, so they are requested BEFORE the ring
  // loads (and first used after them): their wait then does not include the ring's first stages.
  int zraw[TN] = {};
  if (W4 && !RAW) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      int n = n0 + wn0 + j * 32 + l32;
      n = n < p.N ? n : p.N - 1;
      zraw[j] = p.z_b[n];
    }
  }
  // RAW: the zero-points of this lane's 16 output columns per column tile and the row sums of its TM rows, for the
  // accumulators' start values (requested ahead of the ring like the zero-points above)
  v4i zcol[RAW ? TN : 1][4];
  int rsa[RAW ? TM : 1];
  if (RAW) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        int n = n0 + wn0 + j * 32 + 8 * g + 4 * half;
        n = n + 4 <= p.N ? n : p.N - 4;
        zcol[RAW ? j : 0][g] = *reinterpret_cast<const v4i*>(p.z_b + n);
      }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      int m = m0 + wm0 + i * 32 + l32;
      m = m < (int)p.M ? m : (int)p.M - 1;
      rsa[RAW ? i : 0] = p.rowsum_a[m];
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  // ---- prologue ----
  // A CU takes loads in at a bounded rate, so filling the whole ring first would keep the matrix cores waiting for bytes
  // they do not need yet: with more than S k-steps only two stages are requested now and the rest of the ring during the
  // first k-step (RAMP below); a shorter K requests everything at once.
  const bool ramp = nk > S && S > 2;
#pragma unroll
  for (int s = 0; s < S; ++s)
    if (s < nk && (s < 2 || !ramp)) issue(s, s);
  __builtin_amdgcn_sched_barrier(0);

  // ---- MFMA operand fragments ----
  int a_off[2];                                                    // MFMA tile i adds i * 2048
#pragma unroll
  for (int s = 0; s < 2; ++s) a_off[s] = (wm0 + l32) * 64 + (((2 * half + s + (l32 >> 2)) & 3) * 16);
  int b_off[TN][W4 ? 1 : 2];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = wn0 + j * 32 + l32;
#pragma unroll
    for (int s = 0; s < (W4 ? 1 : 2); ++s)
      b_off[j][s] = A_BYTES + (W4 ? n * 32 + ((half ^ ((n >> 3) & 1)) * 16) : n * 64 + (((2 * half + s + (n >> 2)) & 3) * 16));
  }
  int zb4[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) zb4[j] = (int)((unsigned)(zraw[j] * 0x01010101) - 0x80808080u);   // z - 0x80 per byte (mod 2^32)
  v4i fa[TM];      // activation fragments of the sub-step being multiplied
  v4i fb[TN];      // weight fragments of sub-step 0 (of the current, later of the next k-step)
  v4i fbn[TN];     // weight fragments of sub-step 1
  v4i bpk[TN];     // W4: the 16-byte packet that holds this lane's 32 codes of the k-step
  auto load_a = [&](int slot, int s, int i) { fa[i] = *reinterpret_cast<const v4i*>(ring + slot * STAGE + a_off[s] + i * 2048); };
  // weights of sub-step s of the stage in `slot` -> dst; W4: s == 0 also fetches the packet, s == 1 reuses it
  auto unpack = [&](v4i (&dst)[TN], int s) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int d0 = bpk[j][2 * s], d1 = bpk[j][2 * s + 1], z4 = zb4[j];
      if (RAW) {
        dst[j][0] = d0 & 0x0F0F0F0F; dst[j][1] = (d0 >> 4) & 0x0F0F0F0F;
        dst[j][2] = d1 & 0x0F0F0F0F; dst[j][3] = (d1 >> 4) & 0x0F0F0F0F;
        continue;
      }
      dst[j][0] = (int)((unsigned)(d0 & 0x0F0F0F0F) - (unsigned)z4) ^ 0x80808080;
      dst[j][1] = (int)((unsigned)((d0 >> 4) & 0x0F0F0F0F) - (unsigned)z4) ^ 0x80808080;
      dst[j][2] = (int)((unsigned)(d1 & 0x0F0F0F0F) - (unsigned)z4) ^ 0x80808080;
      dst[j][3] = (int)((unsigned)((d1 >> 4) & 0x0F0F0F0F) - (unsigned)z4) ^ 0x80808080;
    }
  };
  auto unpack_dword = [&](v4i (&dst)[TN], int s, int idx) {   // one of the 8 operand dwords: idx = j * 4 + c
    const int j = idx >> 2, c = idx & 3;
    const int d = bpk[j][2 * s + (c >> 1)];
    // per byte: code - z without borrow across bytes = ((code | 0x80) - z) ^ 0x80, with 0x80 - z folded into zb4
    if (RAW) dst[j][c] = ((c & 1) ? (d >> 4) : d) & 0x0F0F0F0F;
    else dst[j][c] = (int)((unsigned)(((c & 1) ? (d >> 4) : d) & 0x0F0F0F0F) - (unsigned)zb4[j]) ^ 0x80808080;
  };
  auto fetch_b = [&](int slot, int s, v4i (&dst)[TN]) {   // int8 weights: fragments straight from LDS; W4: the packet (s == 0 only)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if (W4) bpk[j] = *reinterpret_cast<const v4i*>(ring + slot * STAGE + b_off[j][0]);
      else dst[j] = *reinterpret_cast<const v4i*>(ring + slot * STAGE + b_off[j][W4 ? 0 : s]);
    }
  };
  v16i acc[TN][TM];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e)      // RAW: |z_w| <= 15 and |rowsum_a| <= 128 K fit the 24-bit multiply (K <= 32768: launcher)
        acc[j][i][e] = RAW ? -__mul24(zcol[RAW ? j : 0][e >> 2][e & 3], rsa[RAW ? i : 0]) : 0;
  // per-column epilogue constants: one column per thread pair, fetched now, parked in two registers over the main loop
  // (wide tiles: CPT columns per thread, 128 apart)
  constexpr int CPT = BN / 128;      // (threads beyond the first 256 repeat the second 128's columns)
  float ep_f[CPT], ep_is[CPT], ep_zz[CPT]; int ep_i[CPT], ep_off[CPT];
#pragma unroll
  for (int u = 0; u < CPT; ++u) {
    ep_is[u] = 0.f; ep_zz[u] = 0.f; ep_off[u] = 0;
    const int col = (tid & 127) + 128 * u;
    int n = n0 + col;
    n = n < p.N ? n : p.N - 1;
    // Codes as the only output and no activation (QKV): scale and re-quantization fold into one multiply-add per output,
    // code = rne(acc * A[n] + B[n]) with A = s_a s_w[n] / s_o and B = b[n] / s_o + z_o formed in float64 and rounded once
    // (one rounding less than scale-then-requantize, and one instruction less per output)
    constexpr bool FOLD = OUT == OUT_Q && ACT == RQ_ACT_NONE;
    int sg = 0;
    if ((OUT & OUT_Q) && p.out_q) {   // re-quantization segment of output column col of this tile
      const int no = (ACT == RQ_ACT_SILU_GATED ? n0 / 2 : n0) + col;
      sg = p.n_seg > 1 ? no / p.seg_len : 0;
      sg = sg < p.n_seg ? sg : p.n_seg - 1;
    }
    if (tid < 128) {
      ep_f[u] = FOLD ? (float)((double)p.s_a * (double)p.s_b[n] * p.inv_so_d[sg]) : p.s_a * p.s_b[n];
      ep_i[u] = (p.da != 0 && p.colsum_b) ? p.da * p.colsum_b[n] : 0;
      if ((OUT & OUT_Q) && p.out_q) { ep_is[u] = p.inv_so[sg]; ep_zz[u] = p.zcode[sg]; ep_off[u] = p.off4[sg]; }
    } else {
      const float bn = p.bias ? p.bias[n] : 0.f;
      ep_f[u] = FOLD ? (float)((double)bn * p.inv_so_d[sg] + (double)p.zcode[sg]) : bn;
      ep_i[u] = p.centered ? 128 - p.z_b[n] : 0;
    }
  }
  int rs[TM] = {};
  if (!W4 && p.centered) {      // (packed 4-bit weights are never stored centered: no registers parked for them)
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      int m = m0 + wm0 + i * 32 + l32;
      m = m < (int)p.M ? m : (int)p.M - 1;
      rs[i] = p.rowsum_a[m];
    }
  }

  // stage 0 has landed when at most the loads of stages 1 .. S-1 are outstanding
  {
    const int later = ramp ? 1 : (nk - 1 < S - 1 ? nk - 1 : S - 1);
    static_for_down<S - 1>([&](auto RC) {
      constexpr int r = decltype(RC)::value;
      if (later == r) wait_vm<r * LPS>();
    });
  }
  asm volatile("s_barrier" ::: "memory");
  fetch_b(0, 0, fb);
#pragma unroll
  for (int i = 0; i < TM; ++i) load_a(0, 0, i);
  if (W4) unpack(fb, 0);
  int slot = 0;
  // One k-step.  WAIT = stages that may still be in flight behind stage kt+1, ISSUE = refill the slot with stage kt+S,
  // MORE = a next k-step exists.  While the MFMAs of sub-step 0 run, the weights of sub-step 1 are unpacked into fbn and the
  // activation fragments are replaced one by one; while those of sub-step 1 run, the ring is refilled and the fragments
  // (and unpacked weights) of the next k-step's sub-step 0 are fetched.
  auto step = [&](auto WAITC, auto ISSUEC, auto MOREC, auto RAMPC, int kt) {
    constexpr int WAIT = decltype(WAITC)::value;
    constexpr bool ISSUE = decltype(ISSUEC)::value, MORE = decltype(MOREC)::value, RAMP = decltype(RAMPC)::value;
    const int nslot = slot + 1 == S ? 0 : slot + 1;
    // The issue order below is pinned with scheduling fences: each MFMA is followed by the small piece of VALU / LDS work
    // that hides behind it, so the matrix pipe never waits for the unpacking.
    // ---- sub-step 0: multiply with fb; meanwhile build fbn (sub-step 1 weights) and replace the activation fragments ----
#pragma unroll
    for (int q = 0; q < TM * TN; ++q) {
      const int i = q / TN, j = q % TN;
      acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[j], fa[i], acc[j][i], 0, 0, 0);
      if (W4) {
        constexpr int NDW = TN * 4;      // operand dwords of a sub-step
        if (TM * TN >= NDW) { if (q < NDW) unpack_dword(fbn, 1, q); }
        else {     // fewer MFMAs than operand dwords: spread the pieces over all of them
#pragma unroll
          for (int d = q * NDW / (TM * TN); d < (q + 1) * NDW / (TM * TN); ++d) unpack_dword(fbn, 1, d);
        }
      }
      else if (q < TN) fbn[q] = *reinterpret_cast<const v4i*>(ring + slot * STAGE + b_off[q][W4 ? 0 : 1]);
      if (j == TN - 1) load_a(slot, 1, i);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (MORE) {
      wait_vm<WAIT * LPS>();     // stage kt+1 has landed (this wavefront's share)
      // every read of stage kt by this wavefront has been issued; once they have returned (lgkmcnt) and all wavefronts
      // are here, the slot may be refilled and stage kt+1 (landed everywhere) may be read
      // (the wait as a builtin: the compiler's own wait-count pass cannot see into inline assembly, would take the reads
      // above for still outstanding behind the barrier and drain the counter again -- with the next stage's weight packets
      // just requested -- in front of the first MFMA of sub-step 1)
      __builtin_amdgcn_s_waitcnt(0xC07F);                    // lgkmcnt(0)
      asm volatile("s_barrier" ::: "memory");
      fetch_b(nslot, 0, fb);
      if (RAMP) {          // first k-step of a ramped start: the untouched slots 2 .. S-1 get their first stages now
#pragma unroll
        for (int s = 2; s < S; ++s) issue(s, s);
      }
      if (ISSUE) issue(slot, kt + S);
      __builtin_amdgcn_sched_barrier(0);
    }
    // ---- sub-step 1: multiply with fbn; meanwhile fetch the next k-step's sub-step 0 operands ----
#pragma unroll
    for (int q = 0; q < TM * TN; ++q) {
      const int i = q / TN, j = q % TN;
      acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fbn[j], fa[i], acc[j][i], 0, 0, 0);
      if (MORE) {
        if (W4) {     // the packet was requested before MFMA 0; unpack it behind the later MFMAs
          if (TN == 4) {     // 16 pieces behind the MFMAs after the second one
            constexpr int Q0 = 2, NS = TM * TN - Q0;
            if (q >= Q0) {
#pragma unroll
              for (int d = (q - Q0) * 16 / NS; d < (q - Q0 + 1) * 16 / NS; ++d) unpack_dword(fb, 0, d);
            }
          } else if (TM * TN >= 10) {
            if (q >= 2 && q < 10) unpack_dword(fb, 0, q - 2);
          } else if (TM * TN < 8) {     // the 8 pieces behind the MFMAs after the second one (behind the last, if there are two)
            constexpr int Q0 = TM * TN > 2 ? 2 : TM * TN - 1, NS = TM * TN - Q0;
            if (q >= Q0) {
#pragma unroll
              for (int d = (q - Q0) * 8 / NS; d < (q - Q0 + 1) * 8 / NS; ++d) unpack_dword(fb, 0, d);
            }
          } else {
            if (q >= 2 && q < 6) unpack_dword(fb, 0, q - 2);
            if (q >= 6) { unpack_dword(fb, 0, 4 + 2 * (q - 6)); unpack_dword(fb, 0, 5 + 2 * (q - 6)); }
          }
        }
        if (j == TN - 1) load_a(nslot, 0, i);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    slot = nslot;
  };
  using std::integral_constant;
  int kt = 0;
  using T_ = integral_constant<bool, true>;
  using F_ = integral_constant<bool, false>;
  if (ramp) {     // k-step 0 with only stage 1 behind it
    step(integral_constant<int, 0>{}, T_{}, T_{}, T_{}, 0);
    kt = 1;
  }
  for (; kt + S < nk; ++kt) step(integral_constant<int, S - 2>{}, T_{}, T_{}, F_{}, kt);
  // the last min(S, nk) k-steps: nothing left to issue, fewer and fewer stages in flight (r = k-steps after this one)
  static_for_down<S - 1>([&](auto RC) {
    constexpr int r = decltype(RC)::value;
    if (r < nk) {     // uniform
      step(integral_constant<int, (r > 0 ? r - 1 : 0)>{}, F_{}, integral_constant<bool, (r > 0)>{}, F_{}, kt);
      ++kt;
    }
  });
  // the ring is idle now: hand the per-column constants over through its first bytes
  EL* el = reinterpret_cast<EL*>(ring);
  __syncthreads();
#pragma unroll
  for (int u = 0; u < CPT; ++u) {
    const int col = (tid & 127) + 128 * u;
    if (tid < 128) { el->scale[col] = ep_f[u]; el->cs[col] = ep_i[u]; el->is[col] = ep_is[u]; el->zz[col] = ep_zz[u]; el->off4[col] = ep_off[u]; }
    else { el->bias[col] = ep_f[u]; el->dw[col] = ep_i[u]; }
  }
  __syncthreads();
  if (OUT == (OUT_F32 | OUT_RES) && ACT == RQ_ACT_NONE) {
    float* stage = reinterpret_cast<float*>(ring + EPI_BYTES + wave * (32 * 68 * 4));
    if (m0 + BM <= (int)p.M) epilogue_rows_f32<TM, TN, false, EL>(p, acc, el, rs, stage, m0, n0, wm0, wn0, lane);
    else epilogue_rows_f32<TM, TN, true, EL>(p, acc, el, rs, stage, m0, n0, wm0, wn0, lane);
  } else if (m0 + BM <= (int)p.M) epilogue_wide<TM, TN, ACT, OUT, false, EL, Q8>(p, acc, el, rs, m0, n0, wm0, wn0, lane);
  else epilogue_wide<TM, TN, ACT, OUT, true, EL, Q8>(p, acc, el, rs, m0, n0, wm0, wn0, lane);
}


// host side: one instantiation set per weight format lives in its own translation unit
template <bool W4, int S, int ACT, int OUT, int TM, int TN = 2, int WN = 2, bool Q8 = false, bool RAW = false>
rq_status launch_pipe_one(rq_ctx* ctx, GemmParams& p) {
  if constexpr (!Q8 && ACT == RQ_ACT_NONE && (OUT & OUT_Q) != 0) {      // 8-bit output codes: the tie-guarded instantiation
    if (p.out_q && p.qmaxf > 127.f) return launch_pipe_one<W4, S, ACT, OUT, TM, TN, WN, true, RAW>(ctx, p);
  }
  // Row sums of the activations at hand and a K loop long enough for the cheaper unpack (25 vector instructions per k-step)
  // to outweigh the start values (about 250 per tile): raw nibbles, see the kernel.  Measured: 8192^3 0.544 -> 0.500 ms; with
  // K = 1024 it is 2 % slower (QKV 0.119 -> 0.121, FC1 0.175 -> 0.178 ms at 32896 rows): the K loop there is not bound by its
  // vector instructions and the start values come on top.
  if constexpr (!RAW && W4 && TN == 2) {
    if (p.rowsum_a && p.no_raw <= 0 && (p.K >= 2048 || p.no_raw < 0) && p.K <= 32768 && (reinterpret_cast<uintptr_t>(p.z_b) & 15) == 0 && p.N >= 4)
      return launch_pipe_one<W4, S, ACT, OUT, TM, TN, WN, Q8, true>(ctx, p);
  }
  constexpr int BN = 32 * TN * WN;
  p.tiles_m = (int)((p.M + 64 * TM - 1) / (64 * TM));
  p.tiles_n = (p.N + BN - 1) / BN;
  const int64_t ntiles = (int64_t)p.tiles_m * p.tiles_n;
  {
    // tiles in flight on one XCD (an eighth of the CUs, OCC workgroups each) as g rows x (inflight / g) columns:
    // pick the g that needs the fewest operand bytes per k-step
    constexpr int OCC = pipe_wgs_per_cu(TM, TN, WN, OUT);
    const int cu = ctx->num_cu > 0 ? ctx->num_cu : 256;
    const int inflight = (cu / 8 > 0 ? cu / 8 : 1) * OCC;
    int64_t best = -1;
    p.group_m = 1;
    for (int g = 1; g <= 16; g *= 2) {
      if (g > p.tiles_m && g > 1) break;
      int cols = (inflight + g - 1) / g;
      cols = cols < p.tiles_n ? cols : p.tiles_n;
      const int64_t bytes = (int64_t)g * (64 * TM * 64) + (int64_t)cols * (W4 ? BN * 32 : BN * 64);
      if (best < 0 || bytes < best) { best = bytes; p.group_m = g; }
    }
  }
  constexpr int lds_bytes = S * (64 * TM * 64 + (W4 ? BN * 32 : BN * 64));
  constexpr bool row_staging = OUT == (OUT_F32 | OUT_RES) && ACT == RQ_ACT_NONE;
  constexpr int epi_bytes = BN == 128 ? 4096 : 8192;
  static_assert(sizeof(EpiLdsT<BN>) <= epi_bytes && lds_bytes >= epi_bytes + (row_staging ? 2 * WN * 32 * 68 * 4 : 0) && lds_bytes <= 160 * 1024,
                "the idle ring holds the epilogue constants and, for float rows, the row staging");
  static rq_once_per_device lds_attr;
  RQ_HIP(rq_allow_dynamic_lds(ctx, lds_attr, reinterpret_cast<const void*>(&qgemm_pipe_kernel<W4, S, ACT, OUT, TM, TN, WN, Q8, RAW>), lds_bytes));
  const int64_t blocks = (ntiles + 7) / 8 * 8;
  hipLaunchKernelGGL((qgemm_pipe_kernel<W4, S, ACT, OUT, TM, TN, WN, Q8, RAW>), dim3((unsigned)blocks), dim3(128 * WN), lds_bytes, ctx->stream, p);
  return RQ_OK;
}

// Tile height for the float + residual outputs.  In units of the time one 256-row tile takes alone on a CU, two co-resident
// 256-row tiles take about 1.5, a 320-row tile (which owns its CU) 1.25, two co-resident 192-row tiles 1.125 and three 1.7; pick what
// finishes the busiest CU first.  The 192-row tile only pays while the K loop is short (the epilogue's memory phase then
// weighs as much as the loop and two smaller workgroups overlap it better); with a long loop it measures no faster.
// Returns the number of 64-row groups per tile: 3, 4 or 5.
inline int pick_rows_f32(const rq_ctx* ctx, const GemmParams& p) {
  if (p.force_rows >= 3 && p.force_rows <= 5) return p.force_rows;
  const int64_t cu = ctx->num_cu > 0 ? ctx->num_cu : 256;
  const int64_t tn = (p.N + 127) / 128;
  const int64_t t192 = ((p.M + 191) / 192) * tn, t256 = ((p.M + 255) / 256) * tn, t320 = ((p.M + 319) / 320) * tn;
  // (192-row tiles: up to three per CU; a round of three costs about 1.7, and the last round what its fill costs)
  const int64_t r192 = t192 % (3 * cu);
  const double c192 = 1.69 * (double)(t192 / (3 * cu)) + (r192 == 0 ? 0.0 : r192 <= cu ? 0.75 : r192 <= 2 * cu ? 1.125 : 1.69);
  const double c256 = t256 <= cu ? 1.0 : 1.5 * (double)((t256 + 2 * cu - 1) / (2 * cu));
  const double c320 = 1.25 * (double)((t320 + cu - 1) / cu);
  const double other = c320 < c256 ? c320 : c256;
  if (c192 < other && (p.K <= 1024 || c192 < 0.8 * other)) return 3;      // (a long loop: only where the tile count clearly favours it)
  return c320 < c256 ? 5 : 4;
}

// 256 x 256 tiles (one workgroup per CU): per MFMA they move 192 bytes through the CU's load path instead of the 320 of a
// 256 x 128 tile.  They pay for products that give every CU at least two such tiles
// and have a long K loop (8192^3 with re-quantized output: 1.57 -> 2.04 POP/s); with fewer
// tiles the coarser grid costs more than it saves (2048 x 12288 x 4096, 384 tiles: 0.103 -> 0.105 ms; 2048 x 22016 x 4096 with
// the gated epilogue, 688 tiles: 0.191 -> 0.173 ms).  int8 weight storage gains as much (8192^3: 0.677 -> 0.54 ms) and ends up hardly
// faster than the packed format: without the unpacking its wavefronts wait for operands instead (32 KB per k-step through
// the CU's load path against 24 KB).
template <bool W4>
inline bool wide_tiles(const rq_ctx* ctx, const GemmParams& p) {
  if (p.force_rows) return p.force_rows == 6;
  const int64_t cu = ctx->num_cu > 0 ? ctx->num_cu : 256;
  return p.K >= 2048 && p.M >= 2048 && ((p.M + 255) / 256) * (int64_t)((p.N + 255) / 256) >= 2 * cu;
}

template <bool W4, int S, int ACT>
rq_status launch_pipe_out(rq_ctx* ctx, GemmParams& p) {
  const bool q = p.out_q, f = p.out_f32, r = p.residual, a = p.out_acc;
  if (wide_tiles<W4>(ctx, p)) {
    // re-quantized codes: eight wavefronts (2 x 4, each 128 x 64), two per SIMD -- 8192^3: 0.555 ms against 0.587 ms with four
    // wavefronts of 128 x 128 (a deeper ring changes nothing: 6 stages 0.556 ms)
    if (q && !f && !r && !a) return launch_pipe_one<W4, 4, ACT, OUT_Q, 4, 2, 4>(ctx, p);
    // float output + residual: only on request -- the 320 x 128 tile measures faster there (32896 x 1024 x 4096: 0.187 ms
    // against 0.224 ms)
    if constexpr (W4) {
      if (p.force_rows == 6 && ACT == RQ_ACT_NONE && f && r && !q && !a)
        return launch_pipe_one<W4, 4, RQ_ACT_NONE, OUT_F32 | OUT_RES, 4, 4>(ctx, p);
    }
  }
  if (q && !f && !r && !a) {
    // Re-quantized codes only (QKV, FC1).  With a short K loop the prologue and the epilogue weigh as much as the loop
    // itself, and more, smaller workgroups per CU (three of 192 rows, four of 128 rows) overlap those phases better than
    // two of 256 rows; with a long loop the large tile's operand reuse wins.  Measured on the four workloads' shapes.
    const int rows = p.force_rows ? p.force_rows : (p.K <= 256 ? 2 : (p.K <= 1024 ? 3 : 4));
    if (rows == 2) return launch_pipe_one<W4, 3, ACT, OUT_Q, 2>(ctx, p);
    if (rows == 3) return launch_pipe_one<W4, 3, ACT, OUT_Q, 3>(ctx, p);
    return launch_pipe_one<W4, S, ACT, OUT_Q, 4>(ctx, p);
  }
  if (ACT == RQ_ACT_NONE && f && r && !q && !a) {
    constexpr int S_TALL = W4 ? 6 : 5;       // one workgroup per CU: the ring may take most of the LDS
    const int rows = pick_rows_f32(ctx, p);
    if (rows == 3) return launch_pipe_one<W4, 3, RQ_ACT_NONE, OUT_F32 | OUT_RES, 3>(ctx, p);
    if (rows == 5) return launch_pipe_one<W4, S_TALL, RQ_ACT_NONE, OUT_F32 | OUT_RES, 5>(ctx, p);
    return launch_pipe_one<W4, S, ACT, OUT_F32 | OUT_RES, 4>(ctx, p);
  }
  return launch_pipe_one<W4, S, ACT, OUT_ANY, 4>(ctx, p);
}

template <bool W4, int S>
rq_status launch_pipe(rq_ctx* ctx, GemmParams& p) {
  switch (p.act) {
    case RQ_ACT_GELU: return launch_pipe_out<W4, S, RQ_ACT_GELU>(ctx, p);
    case RQ_ACT_SILU_GATED: return launch_pipe_out<W4, S, RQ_ACT_SILU_GATED>(ctx, p);
    default: return launch_pipe_out<W4, S, RQ_ACT_NONE>(ctx, p);
  }
}

}  // namespace rqg
