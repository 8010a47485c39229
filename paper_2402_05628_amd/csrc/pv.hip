// rq_attn_pv: P.V with shift de-quantized log-sqrt2 probabilities
// (Section "Scale reparameterization for Softmax activations": case analysis before Eq. (3.3-2), Eq. (3.3-2)).
//
//   A^[i, j] = s~(code) * 2^floor(-code/2),  s~ = s (even code) | s*sqrt2 (odd code)
//            = s * 2^-k            (even, k = code >> 1)
//            = (s / sqrt2) * 2^-k  (odd,  k = code >> 1)
// The power of two is an integer shift: inside a window of 8 shifts the probability is the int8 value
// -(128 >> (k & 7)) = -2^(7 - k%8), looked up with one byte-permute per 4 codes.  Even and odd codes go to
// separate exact int32 accumulators on the int8 matrix cores (v_mfma_i32_32x32x32_i8); the parity scale is
// applied once per output.  Codes wider than 4 bits span several windows (k >= 8): shifts are then taken relative to
// the row's smallest shift (whose power of two multiplies the finished row), the windows of 8 relative shifts are
// visited one at a time, only if present, each contributing 2^(-8 w) times its exact integer sum, and relative shifts
// of 40 or more (below 2^-40 of the row's largest probability) are dropped.
// (Rows of more than 256 keys with such codes take pv_long_kernel below instead: powers of two as bfloat16, one pass.)
// V^T is staged per 256 keys in LDS (whole key rows read, bytes transposed in registers) as the ROW operand; the codes go straight from
// global memory into the COLUMN operand (each lane owns 16 consecutive keys of one query row), so a lane ends up
// with 4 consecutive channels of one token.
#include "rq_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct PvParams {
  const uint8_t* codes;
  const int8_t* V;
  int64_t ld, ldv;
  int H, Nq, Nk;
  int causal;
  int wmax;            // last window index: (2^bits - 1) >> 4
  double a_even, a_odd;   // s_log*s_v*(-1/128), s_log*s_v/sqrt2*(-1/128)
  int dv;              // v_off - z_v
  float* out_f32;
  int64_t ldf;
  int8_t* out_q;
  int64_t ldq;
  double inv_so;
  int zo, lo, hi;      // z_o - off_o, clamp bounds of the stored code
  int tiles_i;
  int num_cu;          // causal: every second round of workgroups walks its group's query tiles backwards
  int zero_max;        // RQ_LOG_ZERO_AT_MAX_CODE: keys whose code is the largest one contribute nothing
  unsigned qmax4;      // the largest code in each of the four bytes
};

constexpr int JB = 256;          // keys staged per LDS block (288 for rows of 257 .. 288 keys)

// table of -(128 >> k), k = 0..7, as the 8 bytes {lo dword, hi dword} for v_perm_b32
constexpr unsigned TAB_LO = 0xF0E0C080u, TAB_HI = 0xFFFEFCF8u;

__device__ __forceinline__ unsigned byte_eq_mask(unsigned x, unsigned ref4) {
  // 0xFF in every byte of x equal to the matching byte of ref4 (bytes are < 0x80)
  const unsigned d = x ^ ref4;
  const unsigned nz = ((d + 0x7F7F7F7Fu) | d) & 0x80808080u;   // 0x80 where byte != 0
  const unsigned z = (~nz) & 0x80808080u;                      // 0x80 where byte == 0
  return (z >> 7) * 0xFFu;
}

// WIDE: codes wider than 4 bits (several windows); rows of more than 256 keys with such codes go to pv_long_kernel.
// JBK: keys staged per LDS block, 256, or 288 for rows of 257 .. 288 keys (one block instead of a second one for a few keys:
// every block costs a load -> transpose -> barrier round trip that the few MFMAs of a short row do not hide).
template <int DH, bool WIDE, int JBK>
__global__ __launch_bounds__(256) void pv_kernel(const PvParams p) {
  constexpr int JB = JBK, VT_PITCH = JBK + 16;      // bytes per V^T row (skewed: 68 / 76 dwords -> conflict-free 16-byte reads)
  constexpr int TC = DH / 32;
  constexpr int CP = DH / 16;          // 16-byte pieces per key row
  // V^T: channel r at byte r * VT_PITCH + (r / 16) * 16 -- the extra 16 bytes per 16 channels spread the transposing
  // writes of a wavefront (8 pieces of a key row side by side) over the banks
  __shared__ __align__(16) int8_t vt[DH * VT_PITCH + CP * 16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int blocks_per_group = (p.tiles_i + 3) / 4;
  const int64_t g = blockIdx.x / blocks_per_group;
  // With a causal mask the work of a workgroup grows with its query tile.  Workgroups b and b + (number of CUs) tend to
  // share a CU, so every second round takes the tiles of its groups in reverse: a long one then sits next to a short one.
  int blk = blockIdx.x % blocks_per_group;
  if (p.causal && ((blockIdx.x / (unsigned)p.num_cu) & 1u)) blk = blocks_per_group - 1 - blk;
  const int it = blk * 4 + wave;
  const bool wave_live = it < p.tiles_i;
  const int64_t b = g / p.H;
  const int h = (int)(g % p.H);
  const int8_t* Vg = p.V + b * p.Nk * p.ldv + h * DH;
  const uint8_t* Cg = p.codes + g * p.Nq * p.ld;
  const int qi = it * 32 + l32;
  const int qi_ld = qi < p.Nq ? (wave_live ? qi : 0) : p.Nq - 1;
  const uint8_t* crow = Cg + (int64_t)qi_ld * p.ld;
  const int limit = p.causal ? (qi_ld + 1 < p.Nk ? qi_ld + 1 : p.Nk) : p.Nk;
  // keys this workgroup needs: up to the last row of its last tile when causal
  int blk_rows_end = (blk * 4 + 4) * 32;
  blk_rows_end = blk_rows_end < p.Nq ? blk_rows_end : p.Nq;
  const int nk_block = p.causal ? (blk_rows_end < p.Nk ? blk_rows_end : p.Nk) : p.Nk;
  int wave_rows_end = (it + 1) * 32;
  wave_rows_end = wave_rows_end < p.Nq ? wave_rows_end : p.Nq;
  const int nk_wave = wave_live ? (p.causal ? (wave_rows_end < p.Nk ? wave_rows_end : p.Nk) : p.Nk) : 0;

  // WIDE (codes wider than 4 bits): shifts are taken relative to the row's smallest one, kmin = min over valid keys of
  // code >> 1, and the power 2^-kmin is applied to the finished row.  Relative shifts of 40 or more (terms below 2^-40 of
  // the row's largest probability; at most 4096 of them) are dropped: their sum is below 4e-9 of the result.  Windows of
  // 8 relative shifts are visited one at a time, only if some row of the wavefront has a key in them.
  constexpr int WINDOWS = 5;
  int kmin = 0;
  unsigned kmin4 = 0;
  unsigned present = 1u;
  if (WIDE && wave_live) {
    int km = 127;
    for (int j0 = half * 16; j0 < nk_wave; j0 += 32) {
      const v4i cw = *reinterpret_cast<const v4i*>(crow + j0);
#pragma unroll
      for (int d4 = 0; d4 < 4; ++d4) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = j0 + d4 * 4 + e;
          const int k = (int)(((unsigned)cw[d4] >> (8 * e + 1)) & 0x7Fu);
          km = (j < limit && k < km) ? k : km;
        }
      }
    }
    const int other = __shfl_xor(km, 32, 64);      // the other half of the wavefront holds the other keys of the same row
    kmin = km < other ? km : other;
    kmin4 = (unsigned)kmin * 0x01010101u;
    unsigned pm = 0;
    for (int j0 = half * 16; j0 < nk_wave; j0 += 32) {
      const v4i cw = *reinterpret_cast<const v4i*>(crow + j0);
#pragma unroll
      for (int d4 = 0; d4 < 4; ++d4) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = j0 + d4 * 4 + e;
          const int kr = (int)(((unsigned)cw[d4] >> (8 * e + 1)) & 0x7Fu) - kmin;
          pm |= (j < limit && kr < 8 * WINDOWS) ? (1u << (kr >> 3)) : 0u;
        }
      }
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) pm |= __shfl_xor(pm, m, 64);
    present = pm;
  }
  present = __builtin_amdgcn_readfirstlane(present);

  // WIDE: per-window exact integer sums are folded into float64 running sums (each window has its own power of
  // two); otherwise one window, and the int32 accumulators simply run over all keys.
  // (float32 is enough: each window's exact integer sum is rounded once, to 2^-24 of itself, far inside the 1e-4 code budget)
  float outE[WIDE ? TC : 1][16], outO[WIDE ? TC : 1][16];
  double psE = 0.0, psO = 0.0;
  v16i E[TC], O[TC];
  int se = 0, so = 0;
#pragma unroll
  for (int c = 0; c < TC; ++c)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      E[c][e] = 0; O[c][e] = 0;
      if (WIDE) { outE[c][e] = 0.f; outO[c][e] = 0.f; }
    }

  for (int jb = 0; jb < nk_block; jb += JB) {
    // this wavefront's keys of the block, and (narrow codes) the codes of its first two key tiles, requested before the
    // values are staged so that the two latencies overlap
    int jend = nk_wave - jb;
    jend = jend < JB ? jend : JB;
    auto codes_of = [&](int js) {
      const int j0 = jb + js + half * 16;
      return (js < jend && j0 < p.ld) ? *reinterpret_cast<const v4i*>(crow + j0) : v4i{0, 0, 0, 0};
    };
    v4i c0 = {0, 0, 0, 0}, c1 = {0, 0, 0, 0};
    if (!WIDE) { c0 = codes_of(0); c1 = codes_of(32); }
    __syncthreads();
    // ---- stage V^T for keys jb .. jb+JB-1: thread -> (4 keys, 16 channels); the lanes of a wavefront read whole key
    // rows (16 bytes each), the bytes are transposed in registers, and every channel's 4 keys go out as one dword ----
    // (keys past the last one this workgroup needs are not staged: their probabilities are masked to zero, so whatever
    // the LDS holds there contributes nothing)
    const int nj4 = ((nk_block - jb < JB ? nk_block - jb : JB) + 3) / 4;
    for (int id = tid; id < nj4 * CP; id += 256) {
      const int c16 = id % CP, j4 = id / CP;
      v4i r[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = jb + j4 * 4 + e;
        r[e] = j < p.Nk ? *reinterpret_cast<const v4i*>(Vg + (int64_t)j * p.ldv + c16 * 16) : v4i{0, 0, 0, 0};
      }
      int8_t* const dst = vt + (c16 * 16) * VT_PITCH + c16 * 16 + j4 * 4;     // row c16*16 of the skewed layout
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const unsigned r0 = (unsigned)r[0][d], r1 = (unsigned)r[1][d], r2 = (unsigned)r[2][d], r3 = (unsigned)r[3][d];
        const unsigned lo01 = __builtin_amdgcn_perm(r1, r0, 0x05010400u);   // r0.b0 r1.b0 r0.b1 r1.b1
        const unsigned hi01 = __builtin_amdgcn_perm(r1, r0, 0x07030602u);   // r0.b2 r1.b2 r0.b3 r1.b3
        const unsigned lo23 = __builtin_amdgcn_perm(r3, r2, 0x05010400u);
        const unsigned hi23 = __builtin_amdgcn_perm(r3, r2, 0x07030602u);
        *reinterpret_cast<unsigned*>(dst + (4 * d + 0) * VT_PITCH) = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);   // channel 4d of keys 0..3
        *reinterpret_cast<unsigned*>(dst + (4 * d + 1) * VT_PITCH) = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
        *reinterpret_cast<unsigned*>(dst + (4 * d + 2) * VT_PITCH) = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
        *reinterpret_cast<unsigned*>(dst + (4 * d + 3) * VT_PITCH) = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
      }
    }
    __syncthreads();
    if (jb >= nk_wave) continue;
    for (int w = 0; w < (WIDE ? WINDOWS : 1); ++w) {
      if (WIDE && !((present >> w) & 1u)) continue;
      if (WIDE) {
#pragma unroll
        for (int c = 0; c < TC; ++c)
#pragma unroll
          for (int e = 0; e < 16; ++e) { E[c][e] = 0; O[c][e] = 0; }
        se = 0; so = 0;
      }
      const unsigned wref = (unsigned)w * 0x01010101u;
      // one key tile: its 16 codes per lane -> even / odd operands of this window -> the P.V products
      auto key_tile = [&](int js, const v4i& cw) {
        const int j0 = jb + js + half * 16;
        v4i pe, po;
#pragma unroll
        for (int d4 = 0; d4 < 4; ++d4) {
          // validity of the 4 keys j0+4*d4 .. +3 (padding and causal mask)
          int nv = limit - (j0 + d4 * 4);
          nv = nv < 0 ? 0 : (nv > 4 ? 4 : nv);
          const unsigned vm = nv == 4 ? 0xFFFFFFFFu : ((1u << (8 * nv)) - 1u);
          const unsigned c = (unsigned)cw[d4] | (WIDE ? ~vm : 0u);     // WIDE: invalid positions read as the largest code
          // per byte: relative shift (code >> 1) - kmin; no borrow between bytes because every byte is >= kmin
          const unsigned kr = WIDE ? ((c >> 1) & 0x7F7F7F7Fu) - kmin4 : (c >> 1);
          const unsigned sel = kr & 0x07070707u;
          unsigned pall = __builtin_amdgcn_perm(TAB_HI, TAB_LO, sel);
          if (WIDE) pall &= byte_eq_mask((kr >> 3) & 0x1F1F1F1Fu, wref);
          pall &= vm;
          if (p.zero_max) pall &= ~rq_byte_eq_mask(c, p.qmax4);      // uniform branch
          const unsigned odd = (c & 0x01010101u) * 0xFFu;
          po[d4] = (int)(pall & odd);
          pe[d4] = (int)(pall & ~odd);
        }
        if (p.dv != 0) {
#pragma unroll
          for (int d4 = 0; d4 < 4; ++d4) {
            se = __builtin_amdgcn_sdot4(pe[d4], 0x01010101, se, false);
            so = __builtin_amdgcn_sdot4(po[d4], 0x01010101, so, false);
          }
        }
#pragma unroll
        for (int c = 0; c < TC; ++c) {
          const v4i fv = *reinterpret_cast<const v4i*>(vt + (c * 32 + l32) * VT_PITCH + ((c * 32 + l32) >> 4) * 16 + js + half * 16);
          E[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fv, pe, E[c], 0, 0, 0);
          O[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fv, po, O[c], 0, 0, 0);
        }
      };
      if (WIDE) {       // short rows, visited once per window: the extra registers would cost a wavefront per SIMD
        for (int js = 0; js < jend; js += 32) key_tile(js, codes_of(js));
      } else {
        for (int js = 0; js < jend; js += 32) {
          const v4i c2 = codes_of(js + 64);
          key_tile(js, c0);
          c0 = c1; c1 = c2;
        }
      }
      if (WIDE) {
        const float wsf = __builtin_ldexpf(1.0f, -8 * w);
        // the zero-point term dv * sum(p) is added to the integer sums BEFORE the conversion, so that the large
        // cancellation between the two happens exactly (all of it fits int32: |E| < 2^27, dv * sum(p) < 2^26)
        int ce = 0, co = 0;
        if (p.dv != 0) {     // uniform; the two halves of the wavefront saw different keys of the same row
          ce = p.dv * (se + __shfl_xor(se, 32, 64));
          co = p.dv * (so + __shfl_xor(so, 32, 64));
        }
#pragma unroll
        for (int c = 0; c < TC; ++c)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            outE[c][e] = fmaf((float)(E[c][e] + ce), wsf, outE[c][e]);
            outO[c][e] = fmaf((float)(O[c][e] + co), wsf, outO[c][e]);
          }
      }
    }
  }
  if (!WIDE) { psE = (double)se; psO = (double)so; }
  if (!wave_live) return;
  if (!WIDE && p.dv != 0) {   // the two halves of the wavefront saw different keys of the same row
    psE += __shfl_xor(psE, 32, 64);
    psO += __shfl_xor(psO, 32, 64);
  }
  if (qi >= p.Nq) return;
  const int64_t tok = b * p.Nq + qi;
  const double rowscale = WIDE ? __builtin_ldexp(1.0, -kmin) : 1.0;
  const double corr = WIDE ? 0.0 : (double)p.dv * (p.a_even * psE + p.a_odd * psO);
#pragma unroll
  for (int c = 0; c < TC; ++c) {
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const int col = h * DH + c * 32 + 8 * gq + half * 4;
      double y[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const double ve = WIDE ? (double)outE[WIDE ? c : 0][4 * gq + e] : (double)E[c][4 * gq + e];
        const double vo = WIDE ? (double)outO[WIDE ? c : 0][4 * gq + e] : (double)O[c][4 * gq + e];
        y[e] = (p.a_even * ve + p.a_odd * vo + corr) * rowscale;
      }
      if (p.out_f32)
        *reinterpret_cast<float4*>(p.out_f32 + tok * p.ldf + col) = make_float4((float)y[0], (float)y[1], (float)y[2], (float)y[3]);
      if (p.out_q) {
        int k[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          int q = (int)rint(y[e] * p.inv_so) + p.zo;
          k[e] = q < p.lo ? p.lo : (q > p.hi ? p.hi : q);
        }
        *reinterpret_cast<int*>(p.out_q + tok * p.ldq + col) = rq_pack4(k[0], k[1], k[2], k[3]);
      }
    }
  }
}

// ---- long rows of wide codes: one pass on the bf16 matrix cores ------------------------------------------------------
// With codes wider than 4 bits the int8 scheme above visits every window of 8 shifts separately, after a pass over the
// row's codes for its smallest shift.  A power of two 2^-k (k = 0..127) is exact in bfloat16 whatever k is, and so is
// code - z_v (|.| <= 255: 8 significant bits), so for long rows the probabilities go to the matrix cores as bfloat16
// instead: no windows, no reference shift, one MFMA pass with float32 accumulation (products exact; the sums round like
// any float32 dot product, about 2^-24 per term, far inside the tolerance of the codes).  Even and odd codes still
// accumulate separately; the parity scale is applied once per output.
//  * V^T is staged per 128 keys as bfloat16 of (code - z_v), double-buffered, one barrier per block; the zero-point
//    term therefore needs no separate sum.
//  * A workgroup of 8 wavefronts serves 8 query tiles of one (batch item, head); wavefronts w and w + 4 take tiles from
//    the two ends of the group, which evens out the work under a causal mask.
//  * Contraction index of an MFMA k-step s (16 keys): lane half h, element e <-> key 16 h + 8 s + e of the 32-key tile,
//    for both operands: a lane's 16 codes are one 16-byte load, its V^T piece one 16-byte LDS read.
constexpr int JL = 128;                  // keys per LDS block
constexpr int VL_PITCH = JL * 2 + 16;    // bytes per V^T row (bfloat16), skewed: 68 dwords

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

template <int DH>
constexpr int pv_long_lds() { return 2 * (DH * VL_PITCH + (DH / 16) * 16); }

template <int DH>
__global__ __launch_bounds__(512) void pv_long_kernel(const PvParams p, const int wgs_per_group) {
  constexpr int TC = DH / 32;
  constexpr int CP = DH / 16;            // 16-byte pieces per key row
  constexpr int VBUF = DH * VL_PITCH + CP * 16;
  constexpr int NIDS = (JL / 4) * CP;    // (4 keys, 16 channels) pieces per block: at most 256
  extern __shared__ __align__(16) int8_t lds[];      // two V^T buffers: channel r at r * VL_PITCH + (r / 16) * 16
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;

  const int T = p.tiles_i;
  const int lowT = (T + 1) / 2;                      // tiles taken from the front; T - lowT from the back
  const int64_t g = blockIdx.x / wgs_per_group;
  const int wb = (int)(blockIdx.x - g * wgs_per_group);
  const int kq = 4 * wb + (wave & 3);
  const bool active = wave < 4 ? kq < lowT : kq < T - lowT;
  const int it = !active ? 0 : (wave < 4 ? kq : T - 1 - kq);
  const int it_max = 4 * wb < T - lowT ? T - 1 - 4 * wb : (4 * wb + 3 < lowT ? 4 * wb + 3 : lowT - 1);
  auto keys_of = [&](int tile) {                     // keys the rows of query tile `tile` can see
    int rows_end = (tile + 1) * 32;
    rows_end = rows_end < p.Nq ? rows_end : p.Nq;
    return p.causal ? (rows_end < p.Nk ? rows_end : p.Nk) : p.Nk;
  };
  const int nk_wg = keys_of(it_max);                 // workgroup-uniform
  const int nk_wave = active ? keys_of(it) : 0;
  const int nblk = (nk_wg + JL - 1) / JL;

  const int64_t b = g / p.H;
  const int h = (int)(g - b * p.H);
  const int8_t* const Vg = p.V + b * p.Nk * p.ldv + h * DH;
  const int qi = it * 32 + l32;
  const int qi_ld = qi < p.Nq ? qi : p.Nq - 1;
  const uint8_t* const crow = p.codes + (g * p.Nq + qi_ld) * p.ld;
  const int limit = p.causal ? (qi_ld + 1 < p.Nk ? qi_ld + 1 : p.Nk) : p.Nk;        // valid keys of this row: j < limit
  const int min_limit = p.causal ? (it * 32 + 1 < p.Nk ? it * 32 + 1 : p.Nk) : p.Nk;  // the smallest limit in this wavefront

  // ---- V: 4 keys x 16 channels per thread, requested one block ahead ----
  const int c16 = tid % CP, j4 = tid / CP;
  v4i vreg[4];
  auto request = [&](int blk) {
    if (tid < NIDS) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = blk * JL + j4 * 4 + e;
        vreg[e] = j < p.Nk ? *reinterpret_cast<const v4i*>(Vg + (int64_t)j * p.ldv + c16 * 16) : v4i{0, 0, 0, 0};
      }
    }
  };
  const float dvf = (float)(p.dv - 128);
  auto deposit = [&](int blk) {
    if (tid < NIDS) {
      int8_t* const dst = lds + (blk & 1) * VBUF + (c16 * 16) * VL_PITCH + c16 * 16 + j4 * 8;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        unsigned u[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) u[e] = (unsigned)vreg[e][d] ^ 0x80808080u;      // stored code + 128, unsigned
#pragma unroll
        for (int bb = 0; bb < 4; ++bb) {
          unsigned f[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) f[e] = __float_as_uint((float)((u[e] >> (8 * bb)) & 0xFFu) + dvf);   // code - z_v, exact
          uint2 w;          // the upper halves are the bfloat16 values (exact: at most 8 significant bits)
          w.x = __builtin_amdgcn_perm(f[1], f[0], 0x07060302u);
          w.y = __builtin_amdgcn_perm(f[3], f[2], 0x07060302u);
          *reinterpret_cast<uint2*>(dst + (4 * d + bb) * VL_PITCH) = w;
        }
      }
    }
  };

  v16f E[TC], O[TC];
#pragma unroll
  for (int c = 0; c < TC; ++c)
#pragma unroll
    for (int e = 0; e < 16; ++e) { E[c][e] = 0.f; O[c][e] = 0.f; }

  request(0);
  deposit(0);
  if (nblk > 1) request(1);
  for (int blk = 0; blk < nblk; ++blk) {
    const int jb = blk * JL;
    // this lane's codes of the block (16 per key tile), requested before the barrier
    v4i cw[JL / 32];
#pragma unroll
    for (int t = 0; t < JL / 32; ++t) {
      const int j0 = jb + t * 32 + half * 16;
      cw[t] = (jb + t * 32 < nk_wave && j0 < p.ld) ? *reinterpret_cast<const v4i*>(crow + j0) : v4i{0, 0, 0, 0};
    }
    __syncthreads();        // block blk is in place; every wavefront has finished with the buffer block blk + 1 goes into
    if (blk + 1 < nblk) {
      deposit(blk + 1);
      if (blk + 2 < nblk) request(blk + 2);
    }
    const int8_t* const buf = lds + (blk & 1) * VBUF;
#pragma unroll
    for (int t = 0; t < JL / 32; ++t) {
      if (jb + t * 32 < nk_wave) {          // wavefront-uniform
        const int j0 = jb + t * 32 + half * 16;
        const bool partial = jb + t * 32 + 32 > min_limit;
        v4i pe[2], po[2];
#pragma unroll
        for (int d4 = 0; d4 < 4; ++d4) {
          unsigned c = (unsigned)cw[t][d4];
          if (partial) {      // masked and padding keys read as code 255, whose power of two is stored as zero
            int nv = limit - (j0 + d4 * 4);
            nv = nv < 0 ? 0 : (nv > 4 ? 4 : nv);
            c |= nv == 4 ? 0u : ~((1u << (8 * nv)) - 1u);
          }
          if (p.zero_max) c |= rq_byte_eq_mask(c, p.qmax4);      // the largest code reads as 255 as well (uniform branch)
#pragma unroll
          for (int pr = 0; pr < 2; ++pr) {
            // two codes as halfwords; bfloat16 bits of 2^-k are (127 - k) << 7 = 0x3F80 - ((code & 0xFE) << 6)
            const unsigned cx = __builtin_amdgcn_perm(0u, c, pr ? 0x0C030C02u : 0x0C010C00u);
            const unsigned bits = 0x3F803F80u - ((cx & 0x00FE00FEu) << 6);
            const unsigned odd = (cx & 0x00010001u) * 0xFFFFu;       // 0xFFFF in the halfwords that hold odd codes
            const unsigned vo = bits & odd;
            po[d4 >> 1][(d4 & 1) * 2 + pr] = (int)vo;
            pe[d4 >> 1][(d4 & 1) * 2 + pr] = (int)(bits ^ vo);
          }
        }
#pragma unroll
        for (int c = 0; c < TC; ++c) {
          const int r = c * 32 + l32;
#pragma unroll
          for (int s = 0; s < 2; ++s) {
            const v4i fv = *reinterpret_cast<const v4i*>(buf + r * VL_PITCH + (r >> 4) * 16 + (t * 32 + half * 16 + s * 8) * 2);
            E[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, fv), __builtin_bit_cast(v8bf, pe[s]), E[c], 0, 0, 0);
            O[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, fv), __builtin_bit_cast(v8bf, po[s]), O[c], 0, 0, 0);
          }
        }
      }
    }
  }
  if (!active || qi >= p.Nq) return;
  const int64_t tok = b * p.Nq + qi;
  // the parity scales of the int8 scheme carry its -1/128; here the probabilities are the powers of two themselves
  const double ae = -128.0 * p.a_even, ao = -128.0 * p.a_odd;
#pragma unroll
  for (int c = 0; c < TC; ++c) {
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const int col = h * DH + c * 32 + 8 * gq + half * 4;
      double y[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) y[e] = ae * (double)E[c][4 * gq + e] + ao * (double)O[c][4 * gq + e];
      if (p.out_f32)
        *reinterpret_cast<float4*>(p.out_f32 + tok * p.ldf + col) = make_float4((float)y[0], (float)y[1], (float)y[2], (float)y[3]);
      if (p.out_q) {
        int k[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          int q = (int)rint(y[e] * p.inv_so) + p.zo;
          k[e] = q < p.lo ? p.lo : (q > p.hi ? p.hi : q);
        }
        *reinterpret_cast<int*>(p.out_q + tok * p.ldq + col) = rq_pack4(k[0], k[1], k[2], k[3]);
      }
    }
  }
}

template <int DH>
rq_status launch_long(rq_ctx* ctx, const PvParams& p, int64_t groups) {
  const int wgs_per_group = ((p.tiles_i + 1) / 2 + 3) / 4;
  const int64_t blocks = groups * wgs_per_group;
  if (blocks > (int64_t)1 << 30) return rq_fail(ctx, RQ_ERR_SHAPE, "rq_attn_pv: %lld workgroups exceed 2^30", (long long)blocks);
  constexpr int lds = pv_long_lds<DH>();
  static rq_once_per_device lds_attr;
  RQ_HIP(rq_allow_dynamic_lds(ctx, lds_attr, reinterpret_cast<const void*>(&pv_long_kernel<DH>), lds));
  hipLaunchKernelGGL((pv_long_kernel<DH>), dim3((unsigned)blocks), dim3(512), lds, ctx->stream, p, wgs_per_group);
  return RQ_OK;
}

template <int DH>
void launch(rq_ctx* ctx, const PvParams& p, int64_t groups, bool wide) {
  const int blocks_per_group = (p.tiles_i + 3) / 4;
  const dim3 grid((unsigned)(groups * blocks_per_group));
  if (wide) hipLaunchKernelGGL((pv_kernel<DH, true, 256>), grid, dim3(256), 0, ctx->stream, p);
  else if (p.Nk > 256 && p.Nk <= 288) hipLaunchKernelGGL((pv_kernel<DH, false, 288>), grid, dim3(256), 0, ctx->stream, p);
  else hipLaunchKernelGGL((pv_kernel<DH, false, 256>), grid, dim3(256), 0, ctx->stream, p);
}

}  // namespace

rq_status rq_launch_pv(rq_ctx* ctx, const rq_pv_desc* d) {
  PvParams p;
  p.codes = d->codes; p.V = d->V; p.ld = d->ld; p.ldv = d->ldv;
  p.H = d->H; p.Nq = d->Nq; p.Nk = d->Nk;
  p.causal = d->mask == RQ_MASK_CAUSAL;
  p.wmax = ((1 << d->bits_p) - 1) >> 4;
  const double ss = (double)d->s_log * (double)d->s_v;
  p.a_even = -ss / 128.0;
  p.a_odd = -ss / (128.0 * 1.4142135623730951);
  p.dv = d->v_off - d->z_v;
  p.out_f32 = d->out_f32; p.ldf = d->ldf; p.out_q = d->out_q; p.ldq = d->ldq;
  p.inv_so = d->out_q ? 1.0 / (double)d->s_o : 0.0;
  p.zo = d->z_o - d->off_o; p.lo = -d->off_o; p.hi = (1 << d->bits_o) - 1 - d->off_o;
  p.tiles_i = (d->Nq + 31) / 32;
  p.num_cu = ctx->num_cu > 0 ? ctx->num_cu : 256;
  p.zero_max = (d->flags & RQ_LOG_ZERO_AT_MAX_CODE) != 0;
  p.qmax4 = (unsigned)((1 << d->bits_p) - 1) * 0x01010101u;
  const bool wide = d->bits_p > 4;
  const int64_t groups = d->batch * d->H;
  if (wide && d->Nk > JB) {
    rq_status st = RQ_ERR_SHAPE;
    switch (d->d_head) {
      case 32: st = launch_long<32>(ctx, p, groups); break;
      case 64: st = launch_long<64>(ctx, p, groups); break;
      case 128: st = launch_long<128>(ctx, p, groups); break;
      default: return rq_fail(ctx, RQ_ERR_SHAPE, "rq_attn_pv: d_head = %d must be 32, 64 or 128", d->d_head);
    }
    if (st != RQ_OK) return st;
    RQ_HIP(hipGetLastError());
    return RQ_OK;
  }
  switch (d->d_head) {
    case 32: launch<32>(ctx, p, groups, wide); break;
    case 64: launch<64>(ctx, p, groups, wide); break;
    case 128: launch<128>(ctx, p, groups, wide); break;
    default: return rq_fail(ctx, RQ_ERR_SHAPE, "rq_attn_pv: d_head = %d must be 32, 64 or 128", d->d_head);
  }
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}
