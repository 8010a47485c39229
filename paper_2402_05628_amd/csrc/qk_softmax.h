// Fused Q.K^T + Softmax-log2 quantizer for short rows (up to 288 keys): the exact int32 accumulators of one query
// tile against ALL keys stay in registers, so the [G, N, N] logits never travel through memory
// (attention Eq. of Section "Transformer blocks"; Eq. (3.3-1), second line).  Same arithmetic as rq_qgemm in
// activation mode followed by rq_softmax_log2_quant:
//   acc[i, j] = sum_c (q[i, c] - z_q)(k[j, c] - z_k)                         exact, int32, on the int8 matrix cores
//   code[i, j] = clip(round(2 (log2 sum_k 2^(t_k - t_max) - (t_j - t_max) + log2 s)), 0, 2^b - 1),  t = scale * acc * log2 e (+ bias)
// One workgroup of 8 wavefronts serves one (batch item, head): the keys are staged once in LDS (chunk-rotated rows, so
// the 32-row MFMA operand reads are conflict-free), each wavefront owns 32 query rows.  Keys are the ROW operand and
// queries the COLUMN operand, so a lane holds 4 consecutive keys of one query row per MFMA tile; the two lanes l and
// l+32 together hold a whole row: the row maximum / sum need one lane exchange, and after two v_permlane32_swap each
// lane owns 16 consecutive codes and issues one 16-byte store.
#pragma once
#include "rq_internal.h"

namespace rqks {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

struct QksParams {
  const int8_t* Q;
  const int8_t* K;
  int64_t ldq, ldk;            // row pitch (bytes) of the token-major tensors
  int64_t so, si;              // strides between batch items / heads
  int H, N;                    // heads, tokens per group (Nq == Nk)
  int dq, dk;                  // storage offset minus zero-point of Q and of K
  const float* bias;           // [H, N, N] or NULL
  int bias_lds;                // the bias planes of this workgroup's group slots are kept in LDS (set by the launcher)
  int causal;
  double c1, log2s;            // logit_scale * log2(e), log2(s_log)
  int qmax;
  uint8_t* codes;
  int64_t ld;                  // row pitch of the codes
  int tiles;                   // ceil(N / 32)
  int64_t G;                   // batch * H groups
  // fused P.V (PV variants only): shift de-quantized probabilities times the stored values, re-quantized output
  const int8_t* V;
  int dv;                      // storage offset minus zero-point of V
  double a_even, a_odd;        // s_log * s_v * (-1/128), the same divided by sqrt 2
  float* out_f32;
  int64_t ldf;
  int8_t* out_q;
  int64_t ldo;
  double inv_so;
  int zo, lo, hi;              // z_o - off_o and the clamp bounds of the stored code
  int zero_max;                // RQ_LOG_ZERO_AT_MAX_CODE: keys whose code is the largest one contribute nothing to P.V
};

// table of -(128 >> k), k = 0..7, as the two dwords of a byte permute: 2^-k = -(entry) / 128
constexpr unsigned QKS_TAB_LO = 0xF0E0C080u, QKS_TAB_HI = 0xFFFEFCF8u;

// NT = ceil(N / 32) exactly: tiles 0 .. NT-2 hold valid keys only, so only the last tile (or, with MASKALL = causal mask,
// every tile) pays for per-element masking.
// PV: the codes of a key tile go straight on as the column operand of the P.V product (after the two lane swaps a lane
// owns 16 consecutive keys of its query row, which is that operand's layout); V^T is staged in LDS next to the keys;
// even and odd codes accumulate separately and exactly in int32, as in rq_attn_pv (codes of at most 4 bits: one window).
// Registers per lane: the accumulators of Q.K^T (16 per key tile) and the even and odd accumulators of P.V (32 per 32
// channels) are never live together: the codes of all key tiles are packed first (4 registers per tile, the Q.K^T
// accumulators die as they are converted) and P.V runs afterwards from the packed codes.  (Feeding every tile's codes
// straight into its P.V products, where both sets fit, measured slower at every shape: 42 against 36 us at ViT-B.)
constexpr bool fused_pv_supported(int ksteps, int nt) { return nt * 16 <= 176 && nt * 4 + ksteps * 32 <= 176; }
// the one-kernel attention with a bias and / or codes of 5 or 6 bits exists for rows of up to this many key tiles
constexpr int FUSED_EXT_TILES = 5;

// LDS per group: keys [nt * 32][dh], then (fused P.V) V^T [dh][nt * 32 + 16]
constexpr int slot_bytes(int ksteps, int nt, bool pv) { return nt * 32 * ksteps * 32 + (pv ? ksteps * 32 * (nt * 32 + 16) : 0); }
// Groups per workgroup pass: short rows share a pass so that every wavefront has a tile (1 .. 4 tiles: 8, 4, 2, 2 groups).
// (Longer rows whose tile count does not divide 8 -- 5, 6, 9 tiles -- measured no faster with 3 or 4 groups per pass: the
// staging of a pass is not overlapped with its arithmetic, and it grows with the groups.)
constexpr int groups_per_pass(int ksteps, int nt, bool pv) {
  int want = nt <= 4 ? 8 / nt : 1;
  while (want > 1 && want * slot_bytes(ksteps, nt, pv) > 160 * 1024) --want;
  return want;
}

// PVM: 0 = codes only; 1 = fused P.V on the int8 matrix cores (codes of at most 4 bits: one shift window); 2 = fused P.V
// for wider codes on the bfloat16 matrix cores: a power of two 2^-k is exact in bfloat16 whatever k is, and so is
// code - z_v, so there are no windows and no zero-point sum; the products are exact, the sums round in float32.
template <int KSTEPS, int NT, bool HAS_BIAS, bool F64CODE, bool MASKALL, int PVM>
__global__ __launch_bounds__(512) void qk_softmax_kernel(const QksParams p) {
  constexpr bool PV = PVM != 0, WIDE = PVM == 2;
  constexpr int DH = KSTEPS * 32;
  constexpr int TC = DH / 32;
  constexpr int VTP = NT * 32 + 16;     // bytes per V^T row (skewed)
  constexpr int CPR = DH / 16;          // 16-byte chunks per key row
  constexpr int RPL = 16 / CPR;         // key rows per 256 bytes
  // A workgroup serves GPB groups per pass; their GPB * NT (group slot, query tile) tasks are dealt to the 8 wavefronts in
  // turn (task t: slot t / NT, tile t % NT), so that rows whose tile count does not divide 8 leave few wavefronts idle.
  constexpr int GPB = groups_per_pass(KSTEPS, NT, PV);
  constexpr int NTASK = GPB * NT;
  constexpr int NCHUNK = NT * 32 * CPR;                     // 16-byte key chunks per group
  constexpr int NPIECE = NT * 8 * (DH / 4);                 // (4 keys x 4 channels) pieces of V per group
  constexpr int KS_BYTES = NT * 32 * DH, SLOT_BYTES = KS_BYTES + (PV ? DH * VTP : 0);
  constexpr int KCH = (GPB * NCHUNK + 511) / 512;           // key chunks per thread and pass
  constexpr int VCH = PV ? (GPB * NPIECE + 511) / 512 : 1;
  extern __shared__ __align__(16) int8_t lds[];   // per slot: keys [NT * 32][DH] (chunk c of row r at position (c + r / RPL) % CPR), then V^T [DH][VTP]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  constexpr int nt = NT;
  const int ws0 = wave / NT;                                // this wavefront's first task: group slot
  const int it0 = wave - ws0 * NT;                          // and query tile
  const int Gi = (int)p.G;
  const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
  // Workgroups are persistent over the (batch item, head) groups.  The keys (and values) and this wavefront's first query
  // fragments of the NEXT pass are requested into registers before the current pass's arithmetic, so their latency hides.
  v4i kreg[KCH], qreg[KSTEPS];
  unsigned vreg[VCH][4];
  auto group_base = [&](int g, const int8_t* base) {       // first byte of the group's slice of a token-major tensor
    g = g < Gi ? g : Gi - 1;
    const int b = g / p.H, h = g - b * p.H;
    return base + (int64_t)b * p.so + (int64_t)h * p.si;
  };
  auto request = [&](int gq) {
    if (PV) {
#pragma unroll
      for (int u = 0; u < VCH; ++u) {
        const int id = tid + u * 512;
        const int slot = id / NPIECE, local = id - slot * NPIECE;
        const int c4 = local % (DH / 4), j4 = local / (DH / 4);
        const int8_t* Vg = group_base(gq + slot, p.V);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = j4 * 4 + e;
          vreg[u][e] = (slot < GPB && j < p.N) ? *reinterpret_cast<const unsigned*>(Vg + (int64_t)j * p.ldk + c4 * 4) : 0u;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < KCH; ++u) {
      const int id = tid + u * 512;
      const int slot = id / NCHUNK, local = id - slot * NCHUNK;
      const int r = local / CPR, c = local - r * CPR;
      const int rr = r < p.N ? r : p.N - 1;
      if (slot < GPB) kreg[u] = *reinterpret_cast<const v4i*>(group_base(gq + slot, p.K) + (int64_t)rr * p.ldk + c * 16);
    }
    const int qi = it0 * 32 + l32;
    const int qi_ld = qi < p.N ? qi : p.N - 1;
    const int8_t* Qg = group_base(gq + ws0, p.Q);
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) qreg[s] = *reinterpret_cast<const v4i*>(Qg + (int64_t)qi_ld * p.ldq + s * 32 + half * 16);
  };
  // Which groups a workgroup starts with.  Consecutive groups are consecutive heads of one batch item, whose 64- (or
  // 32-) byte slices of a token row share 128-byte lines.  Workgroup b runs on XCD b % 8, each XCD with its own L2: with one
  // group per pass, neighbouring heads are dealt to the two workgroups b and b + 8 of the same XCD (same round), so that
  // XCD fetches the shared lines once instead of two XCDs fetching them each.  (A permutation of the workgroups of the
  // first whole multiple of 16; the rest keep their index.)
  unsigned wg = blockIdx.x;
  if (GPB == 1 && wg < (gridDim.x & ~15u)) {
    const unsigned xcd = wg & 7u, slot = wg >> 3;
    wg = (slot & 1u) + 2u * (xcd + 8u * (slot >> 1));
  }
  int gq = (int)wg * GPB;
  if (gq < Gi) request(gq);
  // Bias planes in LDS: a workgroup's group slot s always meets head (blockIdx.x * GPB + s) % H (the launcher checks that
  // the stride between passes is a multiple of H), so its GPB planes are copied once and every bias read of every pass is
  // an LDS read instead of a 4-byte gather from the L2.
  float* const bias_lds = reinterpret_cast<float*>(lds + GPB * SLOT_BYTES);
  if (HAS_BIAS && p.bias_lds) {
    const int nn = p.N * p.N;
    for (int s2 = 0; s2 < GPB; ++s2) {
      const float* src = p.bias + (int64_t)((gq + s2) % p.H) * nn;
      for (int i = tid; i < nn; i += 512) bias_lds[s2 * nn + i] = src[i];
    }
  }
  for (; gq < Gi; gq += (int)gridDim.x * GPB) {
  // ---- stage the keys of this pass in LDS (every wavefront has finished with the previous pass) ----
#pragma unroll
  for (int u = 0; u < KCH; ++u) {
    const int id = tid + u * 512;
    const int slot = id / NCHUNK, local = id - slot * NCHUNK;
    const int r = local / CPR, c = local - r * CPR;
    if (slot < GPB) *reinterpret_cast<v4i*>(lds + slot * SLOT_BYTES + r * DH + (((c + r / RPL) % CPR) * 16)) = kreg[u];
  }
  if (PV) {      // 4 keys x 4 channels per piece, bytes transposed in registers: V^T[channel][key]
#pragma unroll
    for (int u = 0; u < VCH; ++u) {
      const int id = tid + u * 512;
      const int slot = id / NPIECE, local = id - slot * NPIECE;
      const int c4 = local % (DH / 4), j4 = local / (DH / 4);
      if (slot < GPB) {
        const unsigned r0 = vreg[u][0], r1 = vreg[u][1], r2 = vreg[u][2], r3 = vreg[u][3];
        const unsigned lo01 = __builtin_amdgcn_perm(r1, r0, 0x05010400u);   // r0.b0 r1.b0 r0.b1 r1.b1
        const unsigned hi01 = __builtin_amdgcn_perm(r1, r0, 0x07030602u);   // r0.b2 r1.b2 r0.b3 r1.b3
        const unsigned lo23 = __builtin_amdgcn_perm(r3, r2, 0x05010400u);
        const unsigned hi23 = __builtin_amdgcn_perm(r3, r2, 0x07030602u);
        const unsigned o0 = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);  // channel 0 of keys 0..3
        const unsigned o1 = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
        const unsigned o2 = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
        const unsigned o3 = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
        int8_t* dst = lds + slot * SLOT_BYTES + KS_BYTES + (c4 * 4) * VTP + j4 * 4;
        *reinterpret_cast<unsigned*>(dst) = o0;
        *reinterpret_cast<unsigned*>(dst + VTP) = o1;
        *reinterpret_cast<unsigned*>(dst + 2 * VTP) = o2;
        *reinterpret_cast<unsigned*>(dst + 3 * VTP) = o3;
      }
    }
  }
  v4i fq0[KSTEPS];
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) fq0[s] = qreg[s];
  __syncthreads();
  // The next pass's operands are requested into registers ahead of time.  With P.V fused (LATE) the request waits until
  // this wavefront's last query tile has turned its accumulators into packed codes, so that its registers are not live
  // while the accumulators are.
  constexpr bool LATE = PV;
  const bool more = gq + (int)gridDim.x * GPB < Gi;
  bool requested = false;
  if (!LATE && more) { request(gq + (int)gridDim.x * GPB); requested = true; }

  for (int task = wave; task < NTASK; task += 8) {       // wavefront-uniform
    const int ws = task / NT, it = task - ws * NT;
    const int64_t g = gq + ws;
    if (g >= p.G) break;
    const int64_t b = g / p.H;
    const int h = (int)(g - b * p.H);
    const int8_t* const Qg = p.Q + b * p.so + (int64_t)h * p.si;
    const int8_t* const ks = lds + ws * SLOT_BYTES;
    const int8_t* const vt = ks + KS_BYTES;
    const int qi = it * 32 + l32;
    const int qi_ld = qi < p.N ? qi : p.N - 1;
    v4i fq[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s)
      fq[s] = task == wave ? fq0[s] : *reinterpret_cast<const v4i*>(Qg + (int64_t)qi_ld * p.ldq + s * 32 + half * 16);
    // Zero-point corrections: sum (q' + dq)(k' + dk) = sum q'k' + dq colsum(k'[j, :]) + dk rowsum(q'[i, :]) + d_head dq dk.  The last
    // two terms are the same for every key of a row and cancel in the softmax (only differences to the row's maximum enter
    // the codes), so they are left out; the accumulators start at zero (the first MFMA of a tile takes the constant 0 as C).
    v16i acc[NT];
#pragma unroll
    for (int jt = 0; jt < NT; ++jt) {
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[jt][e] = 0;
      if (jt < nt) {
        v4i fk[KSTEPS];
        const int r = jt * 32 + l32;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s)
          fk[s] = *reinterpret_cast<const v4i*>(ks + r * DH + ((((s * 2 + half) + r / RPL) % CPR) * 16));
        if (p.dq != 0) {
          v16i ck;
#pragma unroll
          for (int e = 0; e < 16; ++e) ck[e] = 0;
#pragma unroll
          for (int s = 0; s < KSTEPS; ++s) ck = __builtin_amdgcn_mfma_i32_32x32x32_i8(fk[s], ones, ck, 0, 0, 0);
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[jt][e] = p.dq * ck[e];
        }
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) acc[jt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fk[s], fq[s], acc[jt], 0, 0, 0);
      }
      if (NT >= 7) __builtin_amdgcn_sched_barrier(0);     // keep the operand reads of later tiles from piling up in registers
    }
    // ---- softmax statistics of row qi: this lane holds keys jt*32 + 8*(e/4) + 4*half + e%4 ----
    const int limit = MASKALL ? (qi_ld + 1 < p.N ? qi_ld + 1 : p.N) : p.N;     // valid keys: j < limit
    const int rem_last = p.N - (NT - 1) * 32;                                  // keys of the row in the last key tile (1 .. 32)
    const float c1f = (float)p.c1;
    const float qmaxf = (float)p.qmax;
    float ssum = 0.f;
    double C0;
    double tmax = -1e300;
    int amax = INT32_MIN;
    const float* brow = !HAS_BIAS ? nullptr
                        : (p.bias_lds ? static_cast<const float*>(bias_lds) + ((int64_t)ws * p.N + qi_ld) * p.N
                                      : p.bias + ((int64_t)h * p.N + qi_ld) * p.N);
    if (HAS_BIAS && !F64CODE) {
      // Codes of at most 6 bits: t = acc * c1 + bias * log2(e) in float32 (c1 split into two floats, so the product is
      // as good as exact), every bias read once; the accumulator registers then hold t, later t - t_max.
      const float c1lo = (float)(p.c1 - (double)c1f);
      float tmf = -INFINITY;
#pragma unroll
      for (int jt = 0; jt < NT; ++jt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = jt * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
          const bool ok = jt < nt && j < limit;
          const float af = (float)acc[jt][e];
          const float t = ok ? fmaf(af, c1f, fmaf(af, c1lo, brow[ok ? j : 0] * 1.4426950408889634f)) : -INFINITY;
          acc[jt][e] = __float_as_int(t);
          tmf = fmaxf(tmf, t);
        }
      tmf = fmaxf(tmf, __shfl_xor(tmf, 32, 64));
#pragma unroll
      for (int jt = 0; jt < NT; ++jt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float d = __int_as_float(acc[jt][e]) - tmf;      // masked and padding keys: -inf
          acc[jt][e] = __float_as_int(d);
          ssum += __builtin_amdgcn_exp2f(d);
        }
    } else if (HAS_BIAS) {
      // t = acc * c1 + bias * log2(e), kept as the float64 bit pattern is too costly in registers: recomputed below
#pragma unroll
      for (int jt = 0; jt < NT; ++jt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = jt * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
          if (jt < nt && j < limit) tmax = fmax(tmax, fma((double)acc[jt][e], p.c1, (double)brow[j] * 1.4426950408889634));
        }
      tmax = fmax(tmax, __shfl_xor(tmax, 32, 64));
#pragma unroll
      for (int jt = 0; jt < NT; ++jt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = jt * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
          if (jt < nt && j < limit)
            ssum += __builtin_amdgcn_exp2f((float)(fma((double)acc[jt][e], p.c1, (double)brow[j] * 1.4426950408889634) - tmax));
        }
    } else {
      // only the tile that holds the row's last valid key (and, with a causal mask, every tile) needs per-element masking;
      // in that last tile the groups of 8 keys that lie wholly beyond the row's end are skipped altogether (197 keys:
      // three of the four groups of the seventh tile)
#pragma unroll
      for (int jt = 0; jt < NT; ++jt) {
        const bool partial = MASKALL || jt == NT - 1;      // a constant once the loop is unrolled
        if (partial) {
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            if (jt == NT - 1 && gq * 8 >= rem_last) continue;      // wavefront-uniform
#pragma unroll
            for (int e = 4 * gq; e < 4 * gq + 4; ++e) {
              const int j = jt * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
              acc[jt][e] = j < limit ? acc[jt][e] : INT32_MIN;        // masked and padding keys
              amax = max(amax, acc[jt][e]);
            }
          }
        } else {
#pragma unroll
          for (int e = 0; e < 16; ++e) amax = max(amax, acc[jt][e]);
        }
      }
      amax = max(amax, __shfl_xor(amax, 32, 64));
#pragma unroll
      for (int jt = 0; jt < NT; ++jt) {
        const bool partial = MASKALL || jt == NT - 1;      // a constant once the loop is unrolled
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          if (jt == NT - 1 && gq * 8 >= rem_last) continue;
#pragma unroll
          for (int e = 4 * gq; e < 4 * gq + 4; ++e) {
            // acc - amax <= 0; INT32_MIN - amax would wrap, so masked keys get a fixed huge negative distance
            const int d = (partial && acc[jt][e] == INT32_MIN) ? -0x40000000 : acc[jt][e] - amax;
            if (F64CODE) {
              acc[jt][e] = d;
              ssum += __builtin_amdgcn_exp2f((float)d * c1f);     // exp2(-huge) = 0
            } else {
              const float df = (float)d;                          // kept as float bits: the code below needs no second convert
              acc[jt][e] = __float_as_int(df);
              ssum += __builtin_amdgcn_exp2f(df * c1f);
            }
          }
        }
      }
    }
    ssum += __shfl_xor(ssum, 32, 64);
    C0 = 2.0 * ((double)__builtin_amdgcn_logf(ssum) + p.log2s);
    const double m2c = -2.0 * p.c1;
    const float C0f = (float)C0, m2cf = (float)m2c;
    // ---- codes (and, fused, their product with V) ----
    uint8_t* crow = p.codes ? p.codes + (g * p.N + (qi < p.N ? qi : 0)) * p.ld : nullptr;
    v16i E[PV && !WIDE ? TC : 1], O[PV && !WIDE ? TC : 1];
    v16f Ef[WIDE ? TC : 1], Of[WIDE ? TC : 1];
    v4i tvs[PV ? NT : 1];         // the packed codes of every key tile: P.V runs after all of them
    int se = 0, so = 0;
    // the P.V products of one key tile from its 16 codes per lane
    auto pv_tile = [&](int jt, const v4i& tv) {
      const int j0 = jt * 32 + half * 16;
      v4i pe, po;
#pragma unroll
      for (int d4 = 0; d4 < 4; ++d4) {
        const unsigned c = (unsigned)tv[d4];
        unsigned pall = __builtin_amdgcn_perm(QKS_TAB_HI, QKS_TAB_LO, (c >> 1) & 0x07070707u);
        if (MASKALL || jt == NT - 1) {      // masked and padding keys contribute nothing, whatever their code
          int nv = limit - (j0 + d4 * 4);
          nv = nv < 0 ? 0 : (nv > 4 ? 4 : nv);
          pall &= nv == 4 ? 0xFFFFFFFFu : ((1u << (8 * nv)) - 1u);
        }
        if (p.zero_max) pall &= ~rq_byte_eq_mask(c, (unsigned)p.qmax * 0x01010101u);      // uniform branch
        const unsigned lsb = c & 0x01010101u;
        const unsigned odd = (lsb << 8) - lsb;        // 0xFF in the bytes that hold odd codes
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
        const v4i fv = *reinterpret_cast<const v4i*>(vt + (c * 32 + l32) * VTP + j0);
        constexpr int ci = 0;      // (dead code in the wide variants, whose int accumulator arrays have one element)
        E[WIDE ? ci : c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fv, pe, E[WIDE ? ci : c], 0, 0, 0);
        O[WIDE ? ci : c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fv, po, O[WIDE ? ci : c], 0, 0, 0);
      }
    };
    // the same for wide codes: probabilities and values as bfloat16 (contraction index of k-step s: key 8 s + e of the
    // lane's 16 keys, for both operands)
    auto pv_tile_wide = [&](int jt, const v4i& tv) {
      const int j0 = jt * 32 + half * 16;
      v4i pe[2], po[2];
#pragma unroll
      for (int d4 = 0; d4 < 4; ++d4) {
        unsigned c = (unsigned)tv[d4];
        if (MASKALL || jt == NT - 1) {      // masked and padding keys read as code 255, whose power of two is stored as zero
          int nv = limit - (j0 + d4 * 4);
          nv = nv < 0 ? 0 : (nv > 4 ? 4 : nv);
          c |= nv == 4 ? 0u : ~((1u << (8 * nv)) - 1u);
        }
        if (p.zero_max) c |= rq_byte_eq_mask(c, (unsigned)p.qmax * 0x01010101u);      // reads as 255 as well (uniform branch)
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
      const float dvf = (float)(p.dv - 128);
#pragma unroll
      for (int c = 0; c < TC; ++c) {
        const v4i fv = *reinterpret_cast<const v4i*>(vt + (c * 32 + l32) * VTP + j0);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          v4i a;      // 8 values code - z_v of this channel as bfloat16 (exact: at most 8 significant bits)
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const unsigned u = (unsigned)fv[2 * s + q] ^ 0x80808080u;      // stored code + 128, unsigned
            const unsigned f0 = __float_as_uint((float)(u & 0xFFu) + dvf), f1 = __float_as_uint((float)((u >> 8) & 0xFFu) + dvf);
            const unsigned f2 = __float_as_uint((float)((u >> 16) & 0xFFu) + dvf), f3 = __float_as_uint((float)(u >> 24) + dvf);
            a[2 * q] = (int)__builtin_amdgcn_perm(f1, f0, 0x07060302u);
            a[2 * q + 1] = (int)__builtin_amdgcn_perm(f3, f2, 0x07060302u);
          }
          v16f& ef = Ef[WIDE ? c : 0];
          v16f& of = Of[WIDE ? c : 0];
          ef = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, pe[s]), ef, 0, 0, 0);
          of = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, po[s]), of, 0, 0, 0);
        }
      }
    };
#pragma unroll
    for (int jt = 0; jt < NT; ++jt) {
      if (jt < nt) {
        unsigned pk[4];
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          if (!HAS_BIAS && jt == NT - 1 && gq * 8 >= rem_last) { pk[gq] = (unsigned)p.qmax * 0x01010101u; continue; }   // keys past the row's end
          unsigned w = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int j = jt * 32 + 8 * gq + 4 * half + e;
            float vf;
            if (HAS_BIAS && !F64CODE) {
              vf = fmaf(__int_as_float(acc[jt][4 * gq + e]), -2.f, C0f);     // masked keys: +inf -> saturates at qmax
            } else if (HAS_BIAS) {
              const double t = j < limit ? fma((double)acc[jt][4 * gq + e], p.c1, (double)brow[j < p.N ? j : 0] * 1.4426950408889634) : -1e300;
              vf = j < limit ? (float)rint(fma(t - tmax, -2.0, C0)) : qmaxf;
            } else if (F64CODE) {
              vf = (float)rint(fma((double)acc[jt][4 * gq + e], m2c, C0));    // masked keys: huge -> saturates at qmax
            } else {
              vf = fmaf(__int_as_float(acc[jt][4 * gq + e]), m2cf, C0f);
            }
            vf = fminf(vf, qmaxf);
            if (e == 0) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 0, w);
            if (e == 1) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 1, w);
            if (e == 2) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 2, w);
            if (e == 3) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 3, w);
          }
          pk[gq] = w;
        }
        // lane l holds key groups {0,8,16,24}+{0..3}, lane l+32 {4,12,20,28}+{0..3}: after the swaps lane l owns keys
        // 0..15 and lane l+32 keys 16..31 of this tile
        auto s02 = __builtin_amdgcn_permlane32_swap(pk[0], pk[2], false, false);
        auto s13 = __builtin_amdgcn_permlane32_swap(pk[1], pk[3], false, false);
        const int j0 = jt * 32 + half * 16;
        const v4i tv = {(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
        if (crow && qi < p.N && j0 < p.ld) *reinterpret_cast<v4i*>(crow + j0) = tv;
        if (PV) tvs[jt] = tv;
      }
    }
    if (PV) {
      if (more && !requested && task + 8 >= NTASK) { request(gq + (int)gridDim.x * GPB); requested = true; }
      if (WIDE) {
#pragma unroll
        for (int c = 0; c < TC; ++c)
#pragma unroll
          for (int e = 0; e < 16; ++e) { Ef[WIDE ? c : 0][e] = 0.f; Of[WIDE ? c : 0][e] = 0.f; }
#pragma unroll
        for (int jt = 0; jt < NT; ++jt)
          if (jt < nt) pv_tile_wide(jt, tvs[jt]);
      } else {
#pragma unroll
        for (int c = 0; c < TC; ++c)
#pragma unroll
          for (int e = 0; e < 16; ++e) { E[WIDE ? 0 : c][e] = 0; O[WIDE ? 0 : c][e] = 0; }
#pragma unroll
        for (int jt = 0; jt < NT; ++jt)
          if (jt < nt) pv_tile(jt, tvs[jt]);
      }
    }
    if (PV) {
      double psE = (double)se, psO = (double)so;
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
          for (int gq = 0; gq < 4; ++gq) {
            const int col = h * DH + c * 32 + 8 * gq + half * 4;
            float y[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              // (wide codes: the probabilities were the powers of two themselves, not -128 times them, and V carried its zero-point)
              if (WIDE) y[e] = -128.f * fmaf(ao, Of[WIDE ? c : 0][4 * gq + e], ae * Ef[WIDE ? c : 0][4 * gq + e]);
              else if (p.dv == 0) y[e] = fmaf(ao, (float)O[WIDE ? 0 : c][4 * gq + e], ae * (float)E[WIDE ? 0 : c][4 * gq + e]);
              else   // the zero-point term cancels most of the sum: form it in float64
                y[e] = (float)(p.a_even * ((double)E[WIDE ? 0 : c][4 * gq + e] + (double)p.dv * psE) +
                               p.a_odd * ((double)O[WIDE ? 0 : c][4 * gq + e] + (double)p.dv * psO));
            }
            if (p.out_f32)
              *reinterpret_cast<float4*>(p.out_f32 + tok * p.ldf + col) = make_float4(y[0], y[1], y[2], y[3]);
            if (p.out_q) {
              int k[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const float v = fmaf(y[e], iso, zof);
                k[e] = (int)fminf(fmaxf(rintf(v), lof), hif);
                // 8-bit output codes next to a rounding tie: decided again in float64 from the exact integer sums
                if (!WIDE && p.hi - p.lo > 127 && fabsf(v - rintf(v)) > 0.5f - 1.0f / 4096.0f) {
                  const double y64 = p.a_even * ((double)E[WIDE ? 0 : c][4 * gq + e] + (double)p.dv * psE) +
                                     p.a_odd * ((double)O[WIDE ? 0 : c][4 * gq + e] + (double)p.dv * psO);
                  const int q = (int)rint(y64 * p.inv_so) + p.zo;
                  k[e] = q < p.lo ? p.lo : (q > p.hi ? p.hi : q);
                }
              }
              *reinterpret_cast<int*>(p.out_q + tok * p.ldo + col) = rq_pack4(k[0], k[1], k[2], k[3]);
            }
          }
      }
    }
  }
  if (more && !requested) request(gq + (int)gridDim.x * GPB);      // wavefronts without a query tile in this pass
  __syncthreads();      // every wavefront is done with this group's keys
  }
}

template <int KSTEPS, int NT>
rq_status launch(rq_ctx* ctx, const QksParams& p, int64_t groups) {
  if (groups > (int64_t)1 << 30) return rq_fail(ctx, RQ_ERR_SHAPE, "fused attention: %lld groups exceed 2^30", (long long)groups);
  const bool pv = p.V != nullptr;
  const int GPB = groups_per_pass(KSTEPS, NT, pv);      // groups per workgroup pass (as in the kernel)
  const int lds_kv = GPB * slot_bytes(KSTEPS, NT, pv);
  const int64_t cap = (int64_t)(ctx->num_cu > 0 ? ctx->num_cu : 256);      // one 8-wavefront workgroup per CU
  const int64_t passes = (groups + GPB - 1) / GPB;
  const dim3 grid((unsigned)(passes < cap ? passes : cap));
  const bool f64 = p.qmax > 63;
  // float32 bias path: the workgroup's GPB bias planes go to LDS where they fit and every pass of a workgroup meets the
  // same heads (stride between passes a multiple of H, or a single pass)
  QksParams pp = p;
  const int64_t bias_bytes = (int64_t)GPB * p.N * p.N * 4;
  pp.bias_lds = p.bias && !f64 && !p.causal && lds_kv + bias_bytes <= 160 * 1024 &&
                (passes <= cap || ((int64_t)grid.x * GPB) % p.H == 0);
  const int lds = lds_kv + (pp.bias_lds ? (int)bias_bytes : 0);
  constexpr int lds_max = 160 * 1024;
#define RQ_QKS_LAUNCH(B, F, C, P)                                                                                        \
  do {                                                                                                                \
    static rq_once_per_device lds_attr;                                                                               \
    RQ_HIP(rq_allow_dynamic_lds(ctx, lds_attr, reinterpret_cast<const void*>(&qk_softmax_kernel<KSTEPS, NT, B, F, C, P>), \
                                lds_max));                                                                            \
    hipLaunchKernelGGL((qk_softmax_kernel<KSTEPS, NT, B, F, C, P>), grid, dim3(512), lds, ctx->stream, pp);           \
  } while (0)
  // the float64 code path also serves every masked or biased case; the lean variant is the common one
  if (pv) {
    const bool wide = p.qmax > 15;      // more than one window of 8 shifts
    if constexpr (fused_pv_supported(KSTEPS, NT)) {
      if (!p.bias && !wide) RQ_QKS_LAUNCH(false, false, false, 1);
      else if constexpr (NT <= FUSED_EXT_TILES) {      // with a bias and / or wide codes: windows of up to 160 keys
        if (p.bias && wide) RQ_QKS_LAUNCH(true, false, false, 2);
        else if (wide) RQ_QKS_LAUNCH(false, false, false, 2);
        else RQ_QKS_LAUNCH(true, false, false, 1);
      } else return rq_fail(ctx, RQ_ERR_SHAPE, "fused attention with a bias or wide codes: %d key tiles not supported", NT);
    } else return rq_fail(ctx, RQ_ERR_SHAPE, "fused attention: %d key tiles at d_head = %d do not fit the registers", NT, KSTEPS * 32);
  } else if (p.bias && p.causal) RQ_QKS_LAUNCH(true, true, true, 0);
  else if (p.bias && f64) RQ_QKS_LAUNCH(true, true, false, 0);
  else if (p.bias) RQ_QKS_LAUNCH(true, false, false, 0);
  else if (p.causal) RQ_QKS_LAUNCH(false, true, true, 0);
  else if (f64) RQ_QKS_LAUNCH(false, true, false, 0);
  else RQ_QKS_LAUNCH(false, false, false, 0);
#undef RQ_QKS_LAUNCH
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

template <int KSTEPS>
rq_status launch_nt(rq_ctx* ctx, const QksParams& p, int64_t groups) {
  switch (p.tiles) {
    case 1: return launch<KSTEPS, 1>(ctx, p, groups);
    case 2: return launch<KSTEPS, 2>(ctx, p, groups);
    case 3: return launch<KSTEPS, 3>(ctx, p, groups);
    case 4: return launch<KSTEPS, 4>(ctx, p, groups);
    case 5: return launch<KSTEPS, 5>(ctx, p, groups);
    case 6: return launch<KSTEPS, 6>(ctx, p, groups);
    case 7: return launch<KSTEPS, 7>(ctx, p, groups);
    case 8: return launch<KSTEPS, 8>(ctx, p, groups);
    case 9: return launch<KSTEPS, 9>(ctx, p, groups);
  }
  return rq_fail(ctx, RQ_ERR_SHAPE, "fused Q.K^T + softmax: %d key tiles not supported", p.tiles);
}

}  // namespace rqks
