// One-kernel attention for rows whose key-tile count does not fit the register-resident kernel well (257 .. 288 keys:
// nine tiles on eight wavefronts), without an additive bias or mask and with codes of at most 4 bits
// (attention Eq. of Section "Transformer blocks"; Eq. (3.3-1), second line; shift de-quantization of the log sqrt 2 codes).
// Same integers and the same float32 code formula as the register-resident kernel:
//   acc[i, j] = sum_c q'[i, c] k'[j, c] + dq colsum(k'[j, :])                 exact, int32, int8 matrix cores
//   M_i = max_j acc,  S_i = sum_j 2^(c1 (acc - M_i)),  code = clip(round(2 (log2 S_i + log2 s) - 2 c1 (acc - M_i)), 0, qmax)
//   out[i, :] = s s_v (sum_{even codes} 2^-(code/2) v[j, :] + 2^-1/2 sum_{odd codes} 2^-((code-1)/2) v[j, :])
// but the Q.K^T tile of a (query tile, key tile) pair is formed THREE times -- once for the maximum, once for the sum,
// once for the codes, which go straight into their P.V products -- so a wavefront never holds more than one tile of
// logits (16 registers) next to the P.V accumulators.  That keeps a wavefront under 170 registers, three wavefronts
// share a SIMD, and the two extra sets of matrix-core products (which the vector ALU work outweighs anyway) run in
// the shadow of the other wavefronts' conversions.
//
// A workgroup of 12 wavefronts is persistent over passes of GPB (batch item, head) groups, whose GPB * NT
// (group, query tile) tasks make R = GPB * NT / 12 full rounds.  The groups' keys (chunk-rotated rows) and transposed
// values live in GPB LDS slots; the slots are refilled by halves while the rounds that do not read them run: the
// second half of a pass during its first round, the first half of the next pass during the last round (global loads
// into registers before the round's task, LDS writes after it, one barrier per round).
#include <type_traits>

#include "qk_softmax.h"

namespace {

using rqks::QksParams;
using rqks::QKS_TAB_HI;
using rqks::QKS_TAB_LO;
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int W = 12;      // wavefronts per workgroup
constexpr int NTHR = W * 64;

constexpr int slot_bytes(int ksteps, int nt) { return nt * 32 * ksteps * 32 + ksteps * 32 * (nt * 32 + 16); }

template <int KSTEPS, int NT, int GPB, bool DQ, bool ZM>
__global__ __launch_bounds__(NTHR) void attn_stream_kernel(const QksParams p) {
  constexpr int DH = KSTEPS * 32;
  constexpr int TC = DH / 32;
  constexpr int VTP = NT * 32 + 16;     // bytes per V^T row (skewed)
  constexpr int CPR = DH / 16;          // 16-byte chunks per key row
  constexpr int RPL = 16 / CPR;         // key rows per 256 bytes
  constexpr int NTASK = GPB * NT, R = NTASK / W, HG = GPB / 2;
  static_assert(NTASK % W == 0 && GPB % 2 == 0, "the tasks of a pass make full rounds; slots are refilled by halves");
  static_assert(W <= HG * NT, "the first round reads first-half slots only");
  static_assert(HG * NT <= (R - 1) * W, "the last round reads second-half slots only");
  constexpr int NCHUNK = NT * 32 * CPR;                     // 16-byte key chunks per group
  constexpr int NPIECE = NT * 8 * (DH / 4);                 // (4 keys x 4 channels) pieces of V per group
  constexpr int KS_BYTES = NT * 32 * DH, SLOT_BYTES = KS_BYTES + DH * VTP;
  static_assert(NCHUNK % 64 == 0 && (CPR & (CPR - 1)) == 0, "whole 1 KiB blocks; the chunk rotation is a mask");
  constexpr int LU = (NCHUNK / 64 + W - 1) / W;             // 1 KiB blocks of a slot per wavefront
  constexpr int VU = (NPIECE + NTHR - 1) / NTHR;            // value pieces per thread and slot
  extern __shared__ __align__(16) int8_t lds[];   // per slot: keys [NT * 32][DH] (chunk c of row r at position (c + r / RPL) % CPR), then V^T [DH][VTP]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int Gi = (int)p.G;
  const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};

  const unsigned ldk32 = (unsigned)p.ldk;      // the launcher checks that a group's rows span less than 2^31 bytes
  auto group_base = [&](int g, const int8_t* base) {       // first byte of the group's slice of a token-major tensor
    g = g < Gi ? g : Gi - 1;
    const int b = g / p.H, h = g - b * p.H;
    return base + (int64_t)b * p.so + (int64_t)h * p.si;
  };
  // Refill of HG slots (first slot slot0) with groups g0 ..: asynchronous loads straight into LDS, 16 bytes per lane, a
  // wavefront's 64 lanes at 64 consecutive 16-byte places; no register holds the data while it travels.  The lane that
  // serves place q of the key array fetches the chunk that belongs there (row q / CPR, chunk rotated back); the values
  // land in token-major order [key][DH] at the start of the slot's V^T region and are transposed later (transpose_v).
  // Groups past the end re-read the last one (their tasks are skipped); rows past the end re-read the last row (masked).
  // (The lane index passes through an empty asm statement: what is derived from it is then formed where it is used, a few
  // instructions, instead of being kept in registers -- or spilled -- across the rounds.)
  auto request = [&](int g0, int slot0) {
    int ln = lane;
    asm volatile("" : "+v"(ln));
#pragma unroll
    for (int sl = 0; sl < HG; ++sl) {
      const int8_t* const Kg = group_base(g0 + sl, p.K);
      const int8_t* const Vg = group_base(g0 + sl, p.V);
      int8_t* const slot = lds + (slot0 + sl) * SLOT_BYTES;
#pragma unroll
      for (int u = 0; u < LU; ++u) {
        const int i = wave + u * W;                  // 1 KiB block of the slot's key (and value) array
        if (i < NCHUNK / 64) {                       // wavefront-uniform
          const int q = i * 64 + ln;
          const int row = q / CPR, place = q % CPR;
          const int c = (place - row / RPL) & (CPR - 1);
          const unsigned ro = (unsigned)(row < p.N ? row : p.N - 1) * ldk32;
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Kg + (ro + (unsigned)c * 16u)),
                                           (__attribute__((address_space(3))) void*)(slot + i * 1024), 16, 0, 0);
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Vg + (ro + (unsigned)place * 16u)),
                                           (__attribute__((address_space(3))) void*)(slot + KS_BYTES + i * 1024), 16, 0, 0);
        }
      }
    }
  };
  // V [key][DH] -> V^T [DH][VTP] in place, through registers: every (4 keys x 4 channels) piece of the HG slots is read,
  // the workgroup meets at a barrier (the two layouts overlap), the byte-transposed pieces are written.  The caller has
  // waited for the loads and passed a barrier before, and passes one after.
  auto transpose_v = [&](int slot0) {
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    unsigned vreg[HG][VU][4];
#pragma unroll
    for (int sl = 0; sl < HG; ++sl)
#pragma unroll
      for (int u = 0; u < VU; ++u) {
        const int local = t + u * NTHR;
        const int c4 = local % (DH / 4), j4 = local / (DH / 4);
        const int8_t* src = lds + (slot0 + sl) * SLOT_BYTES + KS_BYTES + (j4 * 4) * DH + c4 * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) vreg[sl][u][e] = local < NPIECE ? *reinterpret_cast<const unsigned*>(src + e * DH) : 0u;
      }
    __syncthreads();
#pragma unroll
    for (int sl = 0; sl < HG; ++sl)
#pragma unroll
      for (int u = 0; u < VU; ++u) {
        const int local = t + u * NTHR;
        const int c4 = local % (DH / 4), j4 = local / (DH / 4);
        if (local < NPIECE) {
          const unsigned r0 = vreg[sl][u][0], r1 = vreg[sl][u][1], r2 = vreg[sl][u][2], r3 = vreg[sl][u][3];
          const unsigned lo01 = __builtin_amdgcn_perm(r1, r0, 0x05010400u);   // r0.b0 r1.b0 r0.b1 r1.b1
          const unsigned hi01 = __builtin_amdgcn_perm(r1, r0, 0x07030602u);   // r0.b2 r1.b2 r0.b3 r1.b3
          const unsigned lo23 = __builtin_amdgcn_perm(r3, r2, 0x05010400u);
          const unsigned hi23 = __builtin_amdgcn_perm(r3, r2, 0x07030602u);
          int8_t* dst = lds + (slot0 + sl) * SLOT_BYTES + KS_BYTES + (c4 * 4) * VTP + j4 * 4;
          *reinterpret_cast<unsigned*>(dst) = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);            // channel 0 of keys 0..3
          *reinterpret_cast<unsigned*>(dst + VTP) = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
          *reinterpret_cast<unsigned*>(dst + 2 * VTP) = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
          *reinterpret_cast<unsigned*>(dst + 3 * VTP) = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
        }
      }
  };
  auto wait_loads = [&]() { __builtin_amdgcn_s_waitcnt(0x0F70); };      // vmcnt(0): every load of this wavefront has landed

  const int stride = (int)gridDim.x * GPB;
  int gq = (int)blockIdx.x * GPB;
  // query fragments of task t of the pass that starts at group g0 (requested one task ahead; skipped tasks re-read valid rows)
  v4i fq_next[KSTEPS];
  auto request_q = [&](int g0, int t) {
    const int ws = t / NT, it = t - ws * NT;
    const int qi = it * 32 + l32;
    const int8_t* Qg = group_base(g0 + ws, p.Q);
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s)
      fq_next[s] = *reinterpret_cast<const v4i*>(Qg + (int64_t)(qi < p.N ? qi : p.N - 1) * p.ldq + s * 32 + half * 16);
  };
  if (gq < Gi) {      // workgroup-uniform
    request_q(gq, wave);
    request(gq, 0);
    wait_loads();
    __syncthreads();
    transpose_v(0);
  }
  __syncthreads();
  const float c1f = (float)p.c1, qmaxf = (float)p.qmax;
  const float m2cf = (float)(-2.0 * p.c1);
  const int rem_last = p.N - (NT - 1) * 32;      // keys of a row in the last key tile (1 .. 32)
  const unsigned qmax4 = (unsigned)p.qmax * 0x01010101u;

  for (; gq < Gi; gq += stride) {
    for (int r = 0; r < R; ++r) {
      const bool fill_second = r == 0 && gq + HG < Gi;            // workgroup-uniform
      const bool fill_next = r == R - 1 && gq + stride < Gi;
      if (fill_second) request(gq + HG, HG);
      if (fill_next) request(gq + stride, 0);

      const int task = r * W + wave;
      const int ws = task / NT, it = task - ws * NT;
      const int64_t g = gq + ws;
      const bool live = g < p.G;                                  // wavefront-uniform
      const int64_t b = g / p.H;
      const int h = (int)(g - b * p.H);
      const int8_t* const ks = lds + ws * SLOT_BYTES;
      const int8_t* const vt = ks + KS_BYTES;
      const int qi = it * 32 + l32;
      v4i fq[KSTEPS];
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) fq[s] = fq_next[s];
      int amax = INT32_MIN;
      float C0f = 0.f;
      // The terms dk rowsum(q') + d_head dq dk of the zero-point expansion are the same for every key of a row and cancel
      // in the softmax; dq colsum(k') is kept (DQ).  A tile's accumulators start from cinit (0, or minus the row's maximum:
      // the matrix core then delivers acc - max itself).  This lane ends up with keys jt*32 + 8*(e/4) + 4*half + e%4 of row qi.
      auto qk_tile = [&](int jt, const v16i& cinit) {
        v4i fk[KSTEPS];
        const int kr = jt * 32 + l32;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s)
          fk[s] = *reinterpret_cast<const v4i*>(ks + kr * DH + ((((s * 2 + half) + kr / RPL) % CPR) * 16));
        v16i a = cinit;
        if (DQ) {
          v16i ck;
#pragma unroll
          for (int e = 0; e < 16; ++e) ck[e] = 0;
#pragma unroll
          for (int s = 0; s < KSTEPS; ++s) ck = __builtin_amdgcn_mfma_i32_32x32x32_i8(fk[s], ones, ck, 0, 0, 0);
#pragma unroll
          for (int e = 0; e < 16; ++e) a[e] += p.dq * ck[e];
        }
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) a = __builtin_amdgcn_mfma_i32_32x32x32_i8(fk[s], fq[s], a, 0, 0, 0);
        return a;
      };
      v16i cneg;      // minus the row's maximum in every element
      // ---- sweep 1: the row's largest accumulator ----
      if (live) {
        v16i zero;
#pragma unroll
        for (int e = 0; e < 16; ++e) zero[e] = 0;
        // (the key-tile loops are kept rolled, two tiles per trip so that one tile's operand reads and matrix products
        // overlap the other's conversions: fully unrolled, the reads of later tiles pile up in registers; the last tile,
        // the one with keys past the row's end, has its own copy of each body)
        auto max_tile = [&](const v16i& a) {
#pragma unroll
          for (int e = 0; e < 16; ++e) amax = max(amax, a[e]);
        };
        int jt = 0;
#pragma unroll 1
        for (; jt + 1 < NT - 1; jt += 2) {
          const v16i a0 = qk_tile(jt, zero), a1 = qk_tile(jt + 1, zero);
          max_tile(a0);
          max_tile(a1);
        }
        if ((NT - 1) & 1) max_tile(qk_tile(NT - 2, zero));
        {
          const v16i a = qk_tile(NT - 1, zero);
#pragma unroll
          for (int gk = 0; gk < 4; ++gk) {
            if (gk * 8 >= rem_last) continue;      // groups of 8 keys wholly past the row's end (uniform)
#pragma unroll
            for (int e = 4 * gk; e < 4 * gk + 4; ++e) {
              const int j = (NT - 1) * 32 + 8 * gk + 4 * half + (e & 3);
              amax = j < p.N ? max(amax, a[e]) : amax;
            }
          }
        }
        amax = max(amax, __shfl_xor(amax, 32, 64));
#pragma unroll
        for (int e = 0; e < 16; ++e) cneg[e] = -amax;
        // ---- sweep 2: the sum of 2^(c1 (acc - max)) ----
        float ssum = 0.f;
        auto sum_tile = [&](const v16i& d) {
#pragma unroll
          for (int e = 0; e < 16; ++e) ssum += __builtin_amdgcn_exp2f((float)d[e] * c1f);
        };
#pragma unroll 1
        for (jt = 0; jt + 1 < NT - 1; jt += 2) {
          const v16i d0 = qk_tile(jt, cneg), d1 = qk_tile(jt + 1, cneg);
          sum_tile(d0);
          sum_tile(d1);
        }
        if ((NT - 1) & 1) sum_tile(qk_tile(NT - 2, cneg));
        {
          const v16i d = qk_tile(NT - 1, cneg);
#pragma unroll
          for (int gk = 0; gk < 4; ++gk) {
            if (gk * 8 >= rem_last) continue;
#pragma unroll
            for (int e = 4 * gk; e < 4 * gk + 4; ++e) {
              const int j = (NT - 1) * 32 + 8 * gk + 4 * half + (e & 3);
              // padding keys get a fixed huge negative distance: exp2(-huge) = 0
              ssum += __builtin_amdgcn_exp2f((float)(j < p.N ? d[e] : -0x40000000) * c1f);
            }
          }
        }
        ssum += __shfl_xor(ssum, 32, 64);
        C0f = (float)(2.0 * ((double)__builtin_amdgcn_logf(ssum) + p.log2s));
        // ---- sweep 3: codes, and their products with V ----
        uint8_t* crow = p.codes ? p.codes + (g * p.N + (qi < p.N ? qi : 0)) * p.ld : nullptr;
        v16i E[TC], O[TC];
#pragma unroll
        for (int c = 0; c < TC; ++c)
#pragma unroll
          for (int e = 0; e < 16; ++e) { E[c][e] = 0; O[c][e] = 0; }
        int sa = 0, so = 0;
        auto code_tile = [&](int jt, auto last) {
          const v16i d16 = qk_tile(jt, cneg);
          unsigned pk[4];
#pragma unroll
          for (int gk = 0; gk < 4; ++gk) {
            if (last.value && gk * 8 >= rem_last) { pk[gk] = qmax4; continue; }      // keys past the row's end
            unsigned w = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int j = jt * 32 + 8 * gk + 4 * half + e;
              const int d = (!last.value || j < p.N) ? d16[4 * gk + e] : -0x40000000;
              const float vf = fminf(fmaf((float)d, m2cf, C0f), qmaxf);
              if (e == 0) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 0, w);
              if (e == 1) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 1, w);
              if (e == 2) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 2, w);
              if (e == 3) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 3, w);
            }
            pk[gk] = w;
          }
          // lane l holds key groups {0,8,16,24}+{0..3}, lane l+32 {4,12,20,28}+{0..3}: after the swaps lane l owns keys
          // 0..15 and lane l+32 keys 16..31 of this tile, which is the column operand layout of the P.V product
          auto s02 = __builtin_amdgcn_permlane32_swap(pk[0], pk[2], false, false);
          auto s13 = __builtin_amdgcn_permlane32_swap(pk[1], pk[3], false, false);
          const int j0 = jt * 32 + half * 16;
          const v4i tv = {(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
          if (crow && qi < p.N && j0 < p.ld) *reinterpret_cast<v4i*>(crow + j0) = tv;
          // A accumulates -(128 >> (code / 2)) v of ALL keys, O that of the keys with odd codes only (the even-code sum is
          // their difference, taken in the epilogue): one byte mask per four codes instead of two
          v4i pa, po;
#pragma unroll
          for (int d4 = 0; d4 < 4; ++d4) {
            const unsigned c = (unsigned)tv[d4];
            unsigned pall = __builtin_amdgcn_perm(QKS_TAB_HI, QKS_TAB_LO, (c >> 1) & 0x07070707u);      // -(128 >> (code / 2))
            if (last.value) {      // padding keys contribute nothing, whatever their code
              int nv = p.N - (j0 + d4 * 4);
              nv = nv < 0 ? 0 : (nv > 4 ? 4 : nv);
              pall &= nv == 4 ? 0xFFFFFFFFu : ((1u << (8 * nv)) - 1u);
            }
            if (ZM) pall &= ~rq_byte_eq_mask(c, qmax4);
            // byte selectors 0x0C / 0x0D of a byte permute read as the constants 0x00 / 0xFF: 0xFF in the bytes that hold odd codes
            const unsigned odd = __builtin_amdgcn_perm(0u, 0u, (c & 0x01010101u) | 0x0C0C0C0Cu);
            pa[d4] = (int)pall;
            po[d4] = (int)(pall & odd);
          }
          if (p.dv != 0) {
#pragma unroll
            for (int d4 = 0; d4 < 4; ++d4) {
              sa = __builtin_amdgcn_sdot4(pa[d4], 0x01010101, sa, false);
              so = __builtin_amdgcn_sdot4(po[d4], 0x01010101, so, false);
            }
          }
#pragma unroll
          for (int c = 0; c < TC; ++c) {
            const v4i fv = *reinterpret_cast<const v4i*>(vt + (c * 32 + l32) * VTP + j0);
            E[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fv, pa, E[c], 0, 0, 0);
            O[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fv, po, O[c], 0, 0, 0);
          }
        };
#pragma unroll 1
        for (int jt = 0; jt < NT - 1; ++jt) code_tile(jt, std::false_type{});
        code_tile(NT - 1, std::true_type{});
        // the refill has had three sweeps to land; waiting here, before this round's last loads and stores are
        // issued, keeps those out of the wait
        if (fill_second || fill_next) wait_loads();
        // the next task's query fragments travel while this one's output is formed
        if (r + 1 < R) request_q(gq, (r + 1) * W + wave);
        else if (gq + stride < Gi) request_q(gq + stride, wave);
        // ---- output: lane holds channels c*32 + 8*(e/4) + 4*half + e%4 of row qi ----
        // from here on E holds the even-code sums
#pragma unroll
        for (int c = 0; c < TC; ++c) E[c] -= O[c];
        double psE = (double)(sa - so), psO = (double)so;
        if (p.dv != 0) {   // the two halves of the wavefront saw different keys of the same row
          psE += __shfl_xor(psE, 32, 64);
          psO += __shfl_xor(psO, 32, 64);
        }
        if (qi < p.N) {
          const int64_t tok = b * p.N + qi;
          // |E|, |O| <= 288 * 128 * 255 < 2^24: the integer sums convert to float32 exactly
          const float ae = (float)p.a_even, ao = (float)p.a_odd, iso = (float)p.inv_so;
          const float zof = (float)p.zo, lof = (float)p.lo, hif = (float)p.hi;
#pragma unroll
          for (int c = 0; c < TC; ++c)
#pragma unroll
            for (int gk = 0; gk < 4; ++gk) {
              const int col = h * DH + c * 32 + 8 * gk + half * 4;
              float y[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                if (p.dv == 0) y[e] = fmaf(ao, (float)O[c][4 * gk + e], ae * (float)E[c][4 * gk + e]);
                else   // the zero-point term cancels most of the sum: form it in float64
                  y[e] = (float)(p.a_even * ((double)E[c][4 * gk + e] + (double)p.dv * psE) +
                                 p.a_odd * ((double)O[c][4 * gk + e] + (double)p.dv * psO));
              }
              if (p.out_f32) *reinterpret_cast<float4*>(p.out_f32 + tok * p.ldf + col) = make_float4(y[0], y[1], y[2], y[3]);
              if (p.out_q) {
                int k[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const float v = fmaf(y[e], iso, zof);
                  k[e] = (int)fminf(fmaxf(rintf(v), lof), hif);
                  // 8-bit output codes next to a rounding tie: decided again in float64 from the exact integer sums
                  if (p.hi - p.lo > 127 && fabsf(v - rintf(v)) > 0.5f - 1.0f / 4096.0f) {
                    const double y64 = p.a_even * ((double)E[c][4 * gk + e] + (double)p.dv * psE) +
                                       p.a_odd * ((double)O[c][4 * gk + e] + (double)p.dv * psO);
                    const int q = (int)rint(y64 * p.inv_so) + p.zo;
                    k[e] = q < p.lo ? p.lo : (q > p.hi ? p.hi : q);
                  }
                }
                *reinterpret_cast<int*>(p.out_q + tok * p.ldo + col) = rq_pack4(k[0], k[1], k[2], k[3]);
              }
            }
        }
      } else if (fill_second || fill_next) {
        wait_loads();
      }
      __syncthreads();      // every wavefront is done with the slots of this round, and the refill is in LDS
      if (fill_second || fill_next) {
        transpose_v(fill_second ? HG : 0);
        __syncthreads();
      }
    }
  }
}

template <int KSTEPS, int NT, int GPB, bool DQ, bool ZM>
rq_status launch(rq_ctx* ctx, const QksParams& p) {
  if (p.G > (int64_t)1 << 30) return rq_fail(ctx, RQ_ERR_SHAPE, "fused attention: %lld groups exceed 2^30", (long long)p.G);
  if (p.ldk <= 0 || p.ldk * (int64_t)(NT * 32) >= (int64_t)1 << 31)
    return rq_fail(ctx, RQ_ERR_SHAPE, "streamed attention: token pitch %lld too large", (long long)p.ldk);
  constexpr int lds = GPB * slot_bytes(KSTEPS, NT);
  static_assert(lds <= 160 * 1024, "slots exceed the LDS of a compute unit");
  const int64_t cap = (int64_t)(ctx->num_cu > 0 ? ctx->num_cu : 256);      // one workgroup per CU
  const int64_t passes = (p.G + GPB - 1) / GPB;
  const dim3 grid((unsigned)(passes < cap ? passes : cap));
  static rq_once_per_device lds_attr;
  RQ_HIP(rq_allow_dynamic_lds(ctx, lds_attr, reinterpret_cast<const void*>(&attn_stream_kernel<KSTEPS, NT, GPB, DQ, ZM>), lds));
  hipLaunchKernelGGL((attn_stream_kernel<KSTEPS, NT, GPB, DQ, ZM>), grid, dim3(NTHR), lds, ctx->stream, p);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

}  // namespace

// Shapes this kernel serves (and where it is the fastest one-kernel attention): nine key tiles, d_head 32 or 64, no bias,
// codes of at most 4 bits.
bool rq_attn_stream_supported(int N, int d_head, int bits_p, bool has_bias) {
  return !has_bias && bits_p >= 2 && bits_p <= 4 && N > 256 && N <= 288 && (d_head == 32 || d_head == 64);
}

rq_status rq_launch_attn_stream(rq_ctx* ctx, const rqks::QksParams& p, int d_head) {
  // variants: with the dq colsum(k') term (DQ), with RQ_LOG_ZERO_AT_MAX_CODE (ZM)
#define RQ_STREAM_PICK(KS)                                                                       \
  do {                                                                                           \
    if (p.dq && p.zero_max) return launch<KS, 9, 4, true, true>(ctx, p);                         \
    if (p.dq) return launch<KS, 9, 4, true, false>(ctx, p);                                      \
    if (p.zero_max) return launch<KS, 9, 4, false, true>(ctx, p);                                \
    return launch<KS, 9, 4, false, false>(ctx, p);                                               \
  } while (0)
  if (p.tiles == 9 && d_head == 64) RQ_STREAM_PICK(2);
  if (p.tiles == 9 && d_head == 32) RQ_STREAM_PICK(1);
#undef RQ_STREAM_PICK
  return rq_fail(ctx, RQ_ERR_SHAPE, "streamed attention: %d key tiles at d_head = %d not supported", p.tiles, d_head);
}
