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

struct QksParams {
  const int8_t* Q;
  const int8_t* K;
  int64_t ldq, ldk;            // row pitch (bytes) of the token-major tensors
  int64_t so, si;              // strides between batch items / heads
  int H, N;                    // heads, tokens per group (Nq == Nk)
  int dq, dk;                  // storage offset minus zero-point of Q and of K
  const float* bias;           // [H, N, N] or NULL
  int causal;
  double c1, log2s;            // logit_scale * log2(e), log2(s_log)
  int qmax;
  uint8_t* codes;
  int64_t ld;                  // row pitch of the codes
  int tiles;                   // ceil(N / 32)
  int64_t G;                   // batch * H groups
};

// NT = ceil(N / 32) exactly: tiles 0 .. NT-2 hold valid keys only, so only the last tile (or, with MASKALL = causal mask,
// every tile) pays for per-element masking.
template <int KSTEPS, int NT, bool HAS_BIAS, bool F64CODE, bool MASKALL>
__global__ __launch_bounds__(512) void qk_softmax_kernel(const QksParams p) {
  constexpr int DH = KSTEPS * 32;
  constexpr int CPR = DH / 16;          // 16-byte chunks per key row
  constexpr int RPL = 16 / CPR;         // key rows per 256 bytes
  extern __shared__ __align__(16) int8_t ks[];   // [NT * 32][DH], chunk c of row r stored at position (c + r / RPL) % CPR
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  constexpr int nt = NT;
  const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
  const bool corr = p.dq != 0 || p.dk != 0;
  constexpr int KCH = (NT * 32 * CPR + 511) / 512;      // 16-byte key chunks per thread
  const int nchunks = nt * 32 * CPR;
  // Workgroups are persistent over the (batch item, head) groups.  The keys and this wavefront's first query fragments of
  // the NEXT group are requested into registers before the current group's arithmetic, so their latency hides behind it.
  v4i kreg[KCH], qreg[KSTEPS];
  auto request = [&](int64_t g) {
    const int64_t b = g / p.H;
    const int h = (int)(g - b * p.H);
    const int8_t* Kg = p.K + b * p.so + (int64_t)h * p.si;
    const int8_t* Qg = p.Q + b * p.so + (int64_t)h * p.si;
#pragma unroll
    for (int u = 0; u < KCH; ++u) {
      const int id = tid + u * 512;
      const int r = id / CPR, c = id - r * CPR;
      const int rr = r < p.N ? r : p.N - 1;
      if (id < nchunks) kreg[u] = *reinterpret_cast<const v4i*>(Kg + (int64_t)rr * p.ldk + c * 16);
    }
    const int qi = wave * 32 + l32;
    const int qi_ld = qi < p.N ? qi : p.N - 1;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) qreg[s] = *reinterpret_cast<const v4i*>(Qg + (int64_t)qi_ld * p.ldq + s * 32 + half * 16);
  };
  int64_t g = blockIdx.x;
  if (g < p.G) request(g);
  for (; g < p.G; g += gridDim.x) {
  const int64_t b = g / p.H;
  const int h = (int)(g - b * p.H);
  const int8_t* Qg = p.Q + b * p.so + (int64_t)h * p.si;
  // ---- stage the keys of this group in LDS (every wavefront has finished with the previous group's keys) ----
#pragma unroll
  for (int u = 0; u < KCH; ++u) {
    const int id = tid + u * 512;
    const int r = id / CPR, c = id - r * CPR;
    if (id < nchunks) *reinterpret_cast<v4i*>(ks + r * DH + (((c + r / RPL) % CPR) * 16)) = kreg[u];
  }
  v4i fq0[KSTEPS];
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) fq0[s] = qreg[s];
  __syncthreads();
  if (g + gridDim.x < p.G) request(g + gridDim.x);

  for (int it = wave; it < nt; it += 8) {       // wavefront-uniform
    const int qi = it * 32 + l32;
    const int qi_ld = qi < p.N ? qi : p.N - 1;
    v4i fq[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s)
      fq[s] = it == wave ? fq0[s] : *reinterpret_cast<const v4i*>(Qg + (int64_t)qi_ld * p.ldq + s * 32 + half * 16);
    int base = 0;
    if (corr) {
      v16i rq;
#pragma unroll
      for (int e = 0; e < 16; ++e) rq[e] = 0;
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) rq = __builtin_amdgcn_mfma_i32_32x32x32_i8(ones, fq[s], rq, 0, 0, 0);
      base = p.dk * rq[0] + DH * p.dq * p.dk;   // every element of rq holds rowsum(q'[i, :]) of this lane's query row
    }
    v16i acc[NT];
#pragma unroll
    for (int jt = 0; jt < NT; ++jt) {
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[jt][e] = base;
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
          for (int e = 0; e < 16; ++e) acc[jt][e] += p.dq * ck[e];
        }
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) acc[jt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fk[s], fq[s], acc[jt], 0, 0, 0);
      }
    }
    // ---- softmax statistics of row qi: this lane holds keys jt*32 + 8*(e/4) + 4*half + e%4 ----
    const int limit = MASKALL ? (qi_ld + 1 < p.N ? qi_ld + 1 : p.N) : p.N;     // valid keys: j < limit
    const float c1f = (float)p.c1;
    const float qmaxf = (float)p.qmax;
    float ssum = 0.f;
    double C0;
    double tmax = -1e300;
    int amax = INT32_MIN;
    const float* brow = HAS_BIAS ? p.bias + ((int64_t)h * p.N + qi_ld) * p.N : nullptr;
    if (HAS_BIAS) {
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
      // only the tile that holds the row's last valid key (and, with a causal mask, every tile) needs per-element masking
#pragma unroll
      for (int jt = 0; jt < NT; ++jt) {
        const bool partial = MASKALL || jt == NT - 1;      // a constant once the loop is unrolled
        if (partial) {
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int j = jt * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
            acc[jt][e] = j < limit ? acc[jt][e] : INT32_MIN;        // masked and padding keys
            amax = max(amax, acc[jt][e]);
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
        for (int e = 0; e < 16; ++e) {
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
    ssum += __shfl_xor(ssum, 32, 64);
    C0 = 2.0 * ((double)__builtin_amdgcn_logf(ssum) + p.log2s);
    const double m2c = -2.0 * p.c1;
    const float C0f = (float)C0, m2cf = (float)m2c;
    // ---- codes ----
    uint8_t* crow = p.codes + (g * p.N + (qi < p.N ? qi : 0)) * p.ld;
#pragma unroll
    for (int jt = 0; jt < NT; ++jt) {
      if (jt < nt) {
        unsigned pk[4];
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          unsigned w = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int j = jt * 32 + 8 * gq + 4 * half + e;
            float vf;
            if (HAS_BIAS) {
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
        if (qi < p.N && j0 < p.ld) {
          v4i tv = {(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
          *reinterpret_cast<v4i*>(crow + j0) = tv;
        }
      }
    }
  }
  __syncthreads();      // every wavefront is done with this group's keys
  }
}

template <int KSTEPS, int NT>
rq_status launch(rq_ctx* ctx, const QksParams& p, int64_t groups) {
  const int lds = NT * 32 * KSTEPS * 32;
  const int64_t cap = (int64_t)(ctx->num_cu > 0 ? ctx->num_cu : 256);      // one 8-wavefront workgroup per CU
  const dim3 grid((unsigned)(groups < cap ? groups : cap));
  const bool f64 = p.qmax > 63;
#define RQ_QKS_LAUNCH(B, F, C)                                                                                        \
  do {                                                                                                                \
    static bool attr_set = false;                                                                                     \
    if (!attr_set) {                                                                                                  \
      RQ_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&qk_softmax_kernel<KSTEPS, NT, B, F, C>),              \
                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds));                                   \
      attr_set = true;                                                                                                \
    }                                                                                                                 \
    hipLaunchKernelGGL((qk_softmax_kernel<KSTEPS, NT, B, F, C>), grid, dim3(512), lds, ctx->stream, p);               \
  } while (0)
  // the float64 code path also serves every masked or biased case; the lean variant is the common one
  if (p.bias && p.causal) RQ_QKS_LAUNCH(true, true, true);
  else if (p.bias) RQ_QKS_LAUNCH(true, true, false);
  else if (p.causal) RQ_QKS_LAUNCH(false, true, true);
  else if (f64) RQ_QKS_LAUNCH(false, true, false);
  else RQ_QKS_LAUNCH(false, false, false);
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
