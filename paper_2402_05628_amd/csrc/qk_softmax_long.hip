// Fused Q.K^T + Softmax-log2 quantizer for LONG rows (more than 288 keys, no additive bias): the logits of a row no
// longer fit in registers, so they are formed twice and never stored
// (attention Eq. of Section "Transformer blocks"; Eq. (3.3-1), second line):
//   sweep 1 over the keys: exact int32 Q.K^T tiles on the int8 matrix cores, a running integer maximum M and a running
//           sum S = sum_j 2^(c (acc_j - M)) per query row (rescaled whenever the maximum moves);
//   sweep 2 over the keys: the same tiles again, code_j = clip(round(2 (log2 S + log2 s) - 2 c (acc_j - M)), 0, 2^b - 1).
// Same integers and the same code formula as rq_qgemm (activation mode) + rq_softmax_log2_quant; only the order in
// which the float32 sum is accumulated differs.  Against those two calls this saves writing and reading 4 bytes per
// (query, key) pair; the second set of MFMAs costs far less than that traffic.
//
// One workgroup of 8 wavefronts serves 8 query tiles (32 rows each) of one (batch item, head).  The keys stream through
// a double-buffered LDS ring in chunks of 128 (chunk-rotated rows: conflict-free 32-row operand reads), one barrier per
// chunk, the chunk after next requested into registers meanwhile.  Wavefronts w and w + 4 take query tiles from the two
// ends of the group (k and T-1-k): with a causal mask tile t needs t + 1 key tiles, so every pair carries the same work.
// Codes of a chunk (32 rows x 128 keys per wavefront) pass through the wavefront's own LDS patch and leave as whole
// 128-byte row segments.
#include <type_traits>

#include "qk_softmax.h"

namespace {

using rqks::QksParams;
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int CT = 4;             // key tiles per chunk
constexpr int CK = CT * 32;       // keys per chunk
constexpr int SP = CK + 16;       // row pitch of the code patch (bytes): 36 dwords, conflict-free both ways

constexpr int lds_bytes(int dh) { return 2 * CK * dh + 8 * 32 * SP + 2 * CK * 4; }

template <int KSTEPS, bool F64CODE>
__global__ __launch_bounds__(512) void qk_softmax_long_kernel(const QksParams p, const int wgs_per_group) {
  constexpr int DH = KSTEPS * 32;
  constexpr int CPR = DH / 16;          // 16-byte pieces per key row
  constexpr int RPL = 16 / CPR;         // key rows per 256 bytes
  constexpr int NPIECE = CK * CPR;      // pieces per chunk
  constexpr int PCH = (NPIECE + 511) / 512;
  constexpr int KBUF = CK * DH;
  extern __shared__ __align__(16) int8_t lds[];     // two key buffers, one code patch per wavefront, two sets of key sums
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  uint8_t* const patch = reinterpret_cast<uint8_t*>(lds) + 2 * KBUF + wave * (32 * SP);
  int* const ksum = reinterpret_cast<int*>(lds + 2 * KBUF + 8 * 32 * SP);      // [2][CK]: dq * sum_c k'[j, c] of the chunk's keys

  const int T = p.tiles;
  const int lowT = (T + 1) / 2;                      // tiles taken from the front; T - lowT from the back
  const int64_t g = blockIdx.x / wgs_per_group;
  const int wb = (int)(blockIdx.x - g * wgs_per_group);
  const int kq = 4 * wb + (wave & 3);
  const bool active = wave < 4 ? kq < lowT : kq < T - lowT;
  const int it = !active ? 0 : (wave < 4 ? kq : T - 1 - kq);
  // key tiles the workgroup walks: up to its longest wavefront's diagonal tile (workgroup-uniform)
  const int it_max = 4 * wb < T - lowT ? T - 1 - 4 * wb : (4 * wb + 3 < lowT ? 4 * wb + 3 : lowT - 1);
  const int kt_end = p.causal ? it_max + 1 : T;
  const int nch = (kt_end + CT - 1) / CT;
  const int my_end = p.causal ? (it + 1 < T ? it + 1 : T) : T;     // key tiles this wavefront's rows can see

  const int64_t bi = g / p.H;
  const int h = (int)(g - bi * p.H);
  const int8_t* const Qg = p.Q + bi * p.so + (int64_t)h * p.si;
  const int8_t* const Kg = p.K + bi * p.so + (int64_t)h * p.si;

  v4i kreg[PCH];
  auto request = [&](int c) {
    const int kc = c < nch ? c : c - nch;
#pragma unroll
    for (int u = 0; u < PCH; ++u) {
      const int id = tid + u * 512;
      const int r = id / CPR, cc = id - r * CPR;
      int key = kc * CK + r;
      key = key < p.N ? key : p.N - 1;
      if (NPIECE >= 512 || id < NPIECE) kreg[u] = *reinterpret_cast<const v4i*>(Kg + (int64_t)key * p.ldk + cc * 16);
    }
  };
  // The zero-point term dq * sum_c k'[j, c] depends on the key alone: the CPR neighbouring lanes that hold a key's
  // pieces add them up as the chunk is deposited, instead of a second MFMA per tile against an all-ones operand.
  auto deposit = [&](int c) {
    int8_t* const buf = lds + (c & 1) * KBUF;
#pragma unroll
    for (int u = 0; u < PCH; ++u) {
      const int id = tid + u * 512;
      const int r = id / CPR, cc = id - r * CPR;
      if (NPIECE >= 512 || id < NPIECE) *reinterpret_cast<v4i*>(buf + r * DH + (((cc + r / RPL) % CPR) * 16)) = kreg[u];
      if (p.dq != 0) {
        int sk = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) sk = __builtin_amdgcn_sdot4(kreg[u][e], 0x01010101, sk, false);
        sk += __builtin_amdgcn_update_dpp(0, sk, 0xB1, 0xF, 0xF, true);                    // lane ^ 1
        if (CPR >= 4) sk += __builtin_amdgcn_update_dpp(0, sk, 0x4E, 0xF, 0xF, true);      // lane ^ 2
        if (CPR >= 8) sk += __builtin_amdgcn_update_dpp(0, sk, 0x141, 0xF, 0xF, true);     // the other quad of the 8 lanes
        if (cc == 0 && (NPIECE >= 512 || id < NPIECE)) ksum[(c & 1) * CK + r] = p.dq * sk;
      }
    }
  };

  const int qi = it * 32 + l32;
  const int qi_ld = qi < p.N ? qi : p.N - 1;
  v4i fq[KSTEPS];
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) fq[s] = *reinterpret_cast<const v4i*>(Qg + (int64_t)qi_ld * p.ldq + s * 32 + half * 16);
  const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
  int base = 0;
  if (p.dq != 0 || p.dk != 0) {
    v16i rq;
#pragma unroll
    for (int e = 0; e < 16; ++e) rq[e] = 0;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) rq = __builtin_amdgcn_mfma_i32_32x32x32_i8(ones, fq[s], rq, 0, 0, 0);
    base = p.dk * rq[0] + DH * p.dq * p.dk;     // every element holds the sum over this lane's query row
  }
  const int limit = p.causal ? (qi_ld + 1 < p.N ? qi_ld + 1 : p.N) : p.N;      // valid keys of this row: j < limit
  const int min_limit = p.causal ? (it * 32 + 1 < p.N ? it * 32 + 1 : p.N) : p.N;   // the smallest limit in this wavefront
  const float c1f = (float)p.c1;
  const float qmaxf = (float)p.qmax;
  const int qfill = p.qmax * 0x01010101;

  // exact accumulators of key tile t of chunk c, minus `ref`; returns whether the tile holds masked or padding keys for
  // some row of this wavefront (wavefront-uniform) -- those come back as INT32_MIN
  auto tile = [&](auto may_mask, int c, int t, int jt, int ref, v16i& acc) -> bool {
    const int8_t* const buf = lds + (c & 1) * KBUF;
    v4i fk[KSTEPS];
    const int r = t * 32 + l32;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) fk[s] = *reinterpret_cast<const v4i*>(buf + r * DH + ((((s * 2 + half) + r / RPL) % CPR) * 16));
    const int b0 = base - ref;
    if (p.dq != 0) {
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        const v4i ks = *reinterpret_cast<const v4i*>(ksum + (c & 1) * CK + t * 32 + 8 * gq + 4 * half);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[4 * gq + e] = b0 + ks[e];
      }
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = b0;
    }
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fk[s], fq[s], acc, 0, 0, 0);
    const bool partial = decltype(may_mask)::value && (jt + 1) * 32 > min_limit;      // only the diagonal / last tile pays for masking
    if (partial) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int j = jt * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
        acc[e] = j < limit ? acc[e] : INT32_MIN;
      }
    }
    return partial;
  };

  int m = INT32_MIN;        // running maximum and sum over this LANE's keys of its row (the two halves meet after sweep 1)
  float ssum = 0.f;
  int M = 0;
  double C0 = 0.0;
  float C0f = 0.f;
  const double m2c = -2.0 * p.c1;
  const float m2cf = (float)m2c;

  // the 16 codes a lane ends up owning, from the distances acc - M of one tile
  auto encode = [&](const v16i& acc) -> v4i {
    unsigned pk[4];
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      unsigned w = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int d = acc[4 * gq + e];
        float vf;
        if (F64CODE) vf = (float)rint(fma((double)d, m2c, C0));
        else vf = fmaf((float)d, m2cf, C0f);
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
    return v4i{(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
  };

  request(0);
  deposit(0);
  if (2 * nch > 1) request(1);
  for (int c = 0; c < 2 * nch; ++c) {
    __syncthreads();        // chunk c is in place; every wavefront has finished with the buffer chunk c + 1 goes into
    if (c + 1 < 2 * nch) {
      deposit(c + 1);
      if (c + 2 < 2 * nch) request(c + 2);
    }
    if (!active) continue;
    const int kc0 = c < nch ? c : c - nch;
    const bool interior = (kc0 * CT + CT) * 32 <= min_limit;      // four tiles of valid keys for every row of the wavefront
    if (c < nch && interior) {
      // ---- sweep 1, four full tiles at once: one move of the running sum, 64 independent terms ----
      v16i acc[CT];
#pragma unroll
      for (int t = 0; t < CT; ++t) tile(std::false_type{}, c, t, c * CT + t, 0, acc[t]);
      int tmax = acc[0][0];
#pragma unroll
      for (int t = 0; t < CT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) tmax = max(tmax, acc[t][e]);
      const int newm = max(m, tmax);
      ssum *= m == INT32_MIN ? 0.f : __builtin_amdgcn_exp2f((float)(m - newm) * c1f);
      m = newm;
      float part[CT];
#pragma unroll
      for (int t = 0; t < CT; ++t) {
        part[t] = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) part[t] += __builtin_amdgcn_exp2f((float)(acc[t][e] - m) * c1f);
      }
      ssum += (part[0] + part[1]) + (part[2] + part[3]);
    } else if (c < nch) {
      // ---- sweep 1: row statistics ----
#pragma unroll
      for (int t = 0; t < CT; ++t) {
        const int jt = c * CT + t;
        if (jt < my_end) {
          v16i acc;
          const bool partial = tile(std::true_type{}, c, t, jt, 0, acc);
          int tmax = acc[0];
#pragma unroll
          for (int e = 1; e < 16; ++e) tmax = max(tmax, acc[e]);
          const int newm = max(m, tmax);
          // a lane that has seen no valid key yet holds an empty sum; otherwise move the sum to the new maximum
          ssum *= m == INT32_MIN ? 0.f : __builtin_amdgcn_exp2f((float)(m - newm) * c1f);
          m = newm;
          if (partial) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const int d = acc[e] == INT32_MIN ? -0x40000000 : acc[e] - m;      // exp2(-huge) = 0
              ssum += __builtin_amdgcn_exp2f((float)d * c1f);
            }
          } else {
#pragma unroll
            for (int e = 0; e < 16; ++e) ssum += __builtin_amdgcn_exp2f((float)(acc[e] - m) * c1f);
          }
        }
      }
    } else {
      const int kc = c - nch;
      if (kc == 0) {
        // ---- the two lanes of a row combine their halves (the same expression on both sides) ----
        const int m2 = __shfl_xor(m, 32, 64);
        const float s2 = __shfl_xor(ssum, 32, 64);
        M = max(m, m2);
        const float f_own = m == INT32_MIN ? 0.f : __builtin_amdgcn_exp2f((float)(m - M) * c1f);
        const float f_oth = m2 == INT32_MIN ? 0.f : __builtin_amdgcn_exp2f((float)(m2 - M) * c1f);
        const float S = m >= m2 ? fmaf(s2, f_oth, ssum) : fmaf(ssum, f_own, s2);
        C0 = 2.0 * ((double)__builtin_amdgcn_logf(S) + p.log2s);
        C0f = (float)C0;
      }
      // ---- sweep 2: codes; the accumulators start at -M, so they come out as the distance to the row maximum ----
      if (interior) {
#pragma unroll
        for (int t = 0; t < CT; ++t) {
          v16i acc;
          tile(std::false_type{}, c, t, kc * CT + t, M, acc);
          *reinterpret_cast<v4i*>(patch + l32 * SP + t * 32 + half * 16) = encode(acc);
        }
      } else {
#pragma unroll
        for (int t = 0; t < CT; ++t) {
          const int jt = kc * CT + t;
          v4i tv = {qfill, qfill, qfill, qfill};      // tiles past the row's last key: the largest code
          if (jt < my_end) {
            v16i acc;
            const bool partial = tile(std::true_type{}, c, t, jt, M, acc);
            if (partial) {
#pragma unroll
              for (int e = 0; e < 16; ++e) acc[e] = acc[e] == INT32_MIN ? -0x40000000 : acc[e];   // masked keys: huge -> saturates at qmax
            }
            tv = encode(acc);
          }
          *reinterpret_cast<v4i*>(patch + l32 * SP + t * 32 + half * 16) = tv;
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // this wavefront's own writes; no other wavefront touches `patch`
      const int col = kc * CK + (lane & 7) * 16;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = r * 8 + (lane >> 3);
        const v4i tv = *reinterpret_cast<const v4i*>(patch + row * SP + (lane & 7) * 16);
        const int q = it * 32 + row;
        if (q < p.N && col < p.ld) *reinterpret_cast<v4i*>(p.codes + ((int64_t)g * p.N + q) * p.ld + col) = tv;
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // reads done before the next chunk overwrites the patch
    }
  }
  // columns beyond the chunks this workgroup walked (keys above the diagonal, row padding): the largest code
  if (active) {
    const v4i fill = {qfill, qfill, qfill, qfill};
    for (int64_t col0 = (int64_t)nch * CK; col0 < p.ld; col0 += CK) {
      const int64_t col = col0 + (lane & 7) * 16;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int q = it * 32 + r * 8 + (lane >> 3);
        if (q < p.N && col < p.ld) *reinterpret_cast<v4i*>(p.codes + ((int64_t)g * p.N + q) * p.ld + col) = fill;
      }
    }
  }
}

template <int KSTEPS>
rq_status launch(rq_ctx* ctx, const QksParams& p) {
  const int T = p.tiles;
  const int wgs_per_group = ((T + 1) / 2 + 3) / 4;
  const int64_t blocks = p.G * wgs_per_group;
  if (blocks > (int64_t)1 << 30)
    return rq_fail(ctx, RQ_ERR_SHAPE, "fused Q.K^T + softmax: %lld workgroups exceed 2^30", (long long)blocks);
  constexpr int lds = lds_bytes(KSTEPS * 32);
#define RQ_QKL_LAUNCH(F)                                                                                                  \
  do {                                                                                                                    \
    static rq_once_per_device lds_attr;                                                                                   \
    RQ_HIP(rq_allow_dynamic_lds(ctx, lds_attr, reinterpret_cast<const void*>(&qk_softmax_long_kernel<KSTEPS, F>), lds));  \
    hipLaunchKernelGGL((qk_softmax_long_kernel<KSTEPS, F>), dim3((unsigned)blocks), dim3(512), lds, ctx->stream, p, wgs_per_group); \
  } while (0)
  // float64 code arithmetic beyond 6 bits (as in rq_softmax_log2_quant)
  if (p.qmax > 63) RQ_QKL_LAUNCH(true);
  else RQ_QKL_LAUNCH(false);
#undef RQ_QKL_LAUNCH
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

}  // namespace

rq_status rq_launch_qk_softmax_long(rq_ctx* ctx, const rqks::QksParams& p, int d_head) {
  switch (d_head) {
    case 32: return launch<1>(ctx, p);
    case 64: return launch<2>(ctx, p);
    case 128: return launch<4>(ctx, p);
  }
  return rq_fail(ctx, RQ_ERR_SHAPE, "fused Q.K^T + softmax: d_head = %d not supported", d_head);
}
