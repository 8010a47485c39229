// rq_qgemm_ln_quant: a weight-mode GEMM whose workgroup owns WHOLE output rows (64 tokens x all N <= 768 channels), so that
// the residual add, the next LayerNorm / RMSNorm and its layer-wise quantizer run in the epilogue:
//   xbar = s_a s_w (acc + corrections) + b + residual                      (proj + residual, block equations)
//   q    = clip(rne(norm(xbar) * gamma~ / s~ + beta~ / s~ + z~), 0, 2^b - 1)   (rq_ln_quant's arithmetic)
// xbar still goes to memory (the second residual needs it) but is never read back for the normalization.
// Same pipeline as the tiled kernel (asynchronous global->LDS ring, packed 4-bit weights unpacked behind the MFMAs, fenced
// issue order); one workgroup per CU, wavefront w owns channels [w N/4, (w+1) N/4) of all 64 tokens.  Epilogue: 32 x 64
// output pieces pass through LDS into a row layout (16 lanes per row, 256-byte segments) in which the residual is added,
// xbar is stored and the row statistics are taken; the values stay in registers (they replace the accumulators), the
// statistics of the four wavefronts meet in LDS, and the codes leave as one dword (4 codes) per lane.
#include <cstring>

#include "qgemm_pipe.h"

namespace {

using rqg::GemmParams;
using rqg::v16i;
using rqg::v4i;
using rqg::wait_vm;
using rqg::static_for_down;
using std::integral_constant;

struct RowLnParams {
  GemmParams g;
  const float* gamma_t;
  const float* beta_t;
  double inv_s, zcode, eps;
  float qmaxf;
  unsigned off4;
  int norm_kind;
  int8_t* q;
  int64_t ldq2;
  int32_t* rowsum;
};

__device__ __forceinline__ int sum16_i(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);
  return v;
}

template <int TN, int S>
__global__ __launch_bounds__(256, 1) void qgemm_rowln_kernel(const RowLnParams P) {
  const GemmParams& p = P.g;
  constexpr int TM = 2, BM = 64, BN = 128 * TN;
  constexpr int A_BYTES = BM * 64, B_BYTES = BN * 32, STAGE = A_BYTES + B_BYTES;
  constexpr int LPS = 1 + TN;                               // loads per thread and stage
  constexpr int Q = TM * TN;                                // MFMAs per sub-step
  constexpr int NCH = TN / 2;                               // 64-column pieces per wavefront
  constexpr int PITCH = 68;
  static_assert(TN % 2 == 0 && (S - 1) * LPS <= 63, "even number of 32-column tiles per wavefront; the load counter holds 63");
  extern __shared__ __align__(16) int8_t ring[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int wn0 = wave * 32 * TN;
  const int m0 = blockIdx.x * BM;
  const int nk = p.K / 64;
  const int Mi = (int)p.M;

  // ---- asynchronous loads (same chunk rotation as the tiled kernel) ----
  unsigned aofs, bofs[TN];
  {
    const int dl_row = lane >> 2;
    const int dl_c = ((lane & 3) - (dl_row >> 2)) & 3;
    int m = m0 + wave * 16 + dl_row;
    m = m < Mi ? m : Mi - 1;
    aofs = (unsigned)m * (unsigned)p.lda + (unsigned)(dl_c * 16);
#pragma unroll
    for (int t = 0; t < TN; ++t) {
      const int row = t * 128 + (tid >> 1);
      bofs[t] = (unsigned)row * (unsigned)p.ldb + (unsigned)(((tid & 1) ^ ((row >> 3) & 1)) * 16);
    }
  }
  const int8_t* const gA = p.A;
  const uint8_t* const gB = p.B;
  auto issue = [&](int slot, int kt) {
    int8_t* la = ring + slot * STAGE;
    int8_t* lb = la + A_BYTES;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gA + (aofs + (unsigned)kt * 64u)),
                                     (__attribute__((address_space(3))) void*)(la + wave * 1024), 16, 0, 0);
#pragma unroll
    for (int t = 0; t < TN; ++t)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gB + (bofs[t] + (unsigned)kt * 32u)),
                                       (__attribute__((address_space(3))) void*)(lb + (t * 4 + wave) * 1024), 16, 0, 0);
  };
  int zraw[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) zraw[j] = p.z_b[wn0 + j * 32 + l32];
  __builtin_amdgcn_sched_barrier(0);
  const bool ramp = nk > S && S > 2;
#pragma unroll
  for (int s = 0; s < S; ++s)
    if (s < nk && (s < 2 || !ramp)) issue(s, s);
  __builtin_amdgcn_sched_barrier(0);

  // ---- MFMA operand fragments ----
  int a_off[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) a_off[s] = l32 * 64 + (((2 * half + s + (l32 >> 2)) & 3) * 16);
  int b_off[TN], zb4[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = wn0 + j * 32 + l32;
    b_off[j] = A_BYTES + n * 32 + ((half ^ ((n >> 3) & 1)) * 16);
    zb4[j] = (int)((unsigned)(zraw[j] * 0x01010101) - 0x80808080u);
  }
  v4i fa[TM], fb[TN], fbn[TN], bpk[TN];
  auto load_a = [&](int slot, int s, int i) { fa[i] = *reinterpret_cast<const v4i*>(ring + slot * STAGE + a_off[s] + i * 2048); };
  auto unpack_dword = [&](v4i (&dst)[TN], int s, int idx) {
    const int j = idx >> 2, c = idx & 3;
    const int d = bpk[j][2 * s + (c >> 1)];
    dst[j][c] = (int)((unsigned)(((c & 1) ? (d >> 4) : d) & 0x0F0F0F0F) - (unsigned)zb4[j]) ^ 0x80808080;
  };
  auto fetch_b = [&](int slot) {
#pragma unroll
    for (int j = 0; j < TN; ++j) bpk[j] = *reinterpret_cast<const v4i*>(ring + slot * STAGE + b_off[j]);
  };
  v16i acc[TN][TM];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[j][i][e] = 0;

  {
    const int later = ramp ? 1 : (nk - 1 < S - 1 ? nk - 1 : S - 1);
    static_for_down<S - 1>([&](auto RC) {
      constexpr int r = decltype(RC)::value;
      if (later == r) wait_vm<r * LPS>();
    });
  }
  asm volatile("s_barrier" ::: "memory");
  fetch_b(0);
#pragma unroll
  for (int i = 0; i < TM; ++i) load_a(0, 0, i);
#pragma unroll
  for (int idx = 0; idx < 4 * TN; ++idx) unpack_dword(fb, 0, idx);
  int slot = 0;
  auto step = [&](auto WAITC, auto ISSUEC, auto MOREC, auto RAMPC, int kt) {
    constexpr int WAIT = decltype(WAITC)::value;
    constexpr bool ISSUE = decltype(ISSUEC)::value, MORE = decltype(MOREC)::value, RAMP = decltype(RAMPC)::value;
    const int nslot = slot + 1 == S ? 0 : slot + 1;
    // sub-step 0: multiply with fb; behind each MFMA two dwords of the sub-step 1 weights are unpacked
#pragma unroll
    for (int q = 0; q < Q; ++q) {
      const int i = q / TN, j = q % TN;
      acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[j], fa[i], acc[j][i], 0, 0, 0);
      unpack_dword(fbn, 1, 2 * q);
      unpack_dword(fbn, 1, 2 * q + 1);
      if (j == TN - 1) load_a(slot, 1, i);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (MORE) {
      wait_vm<WAIT * LPS>();
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
      fetch_b(nslot);
      if (RAMP) {
#pragma unroll
        for (int s = 2; s < S; ++s) issue(s, s);
      }
      if (ISSUE) issue(slot, kt + S);
      __builtin_amdgcn_sched_barrier(0);
    }
    // sub-step 1: multiply with fbn; the next k-step's packets were requested above and are unpacked behind the later MFMAs
    constexpr int Q0 = Q > 4 ? 2 : Q - 1;                                   // first MFMA slot that unpacks
    constexpr int PER = (4 * TN + (Q - Q0) - 1) / (Q - Q0);                 // dwords per slot
#pragma unroll
    for (int q = 0; q < Q; ++q) {
      const int i = q / TN, j = q % TN;
      acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fbn[j], fa[i], acc[j][i], 0, 0, 0);
      if (MORE) {
        if (q >= Q0) {
#pragma unroll
          for (int u = 0; u < PER; ++u)
            if ((q - Q0) * PER + u < 4 * TN) unpack_dword(fb, 0, (q - Q0) * PER + u);
        }
        if (j == TN - 1) load_a(nslot, 0, i);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    slot = nslot;
  };
  using T_ = integral_constant<bool, true>;
  using F_ = integral_constant<bool, false>;
  int kt = 0;
  if (ramp) {
    step(integral_constant<int, 0>{}, T_{}, T_{}, T_{}, 0);
    kt = 1;
  }
  for (; kt + S < nk; ++kt) step(integral_constant<int, S - 2>{}, T_{}, T_{}, F_{}, kt);
  static_for_down<S - 1>([&](auto RC) {
    constexpr int r = decltype(RC)::value;
    if (r < nk) {
      step(integral_constant<int, (r > 0 ? r - 1 : 0)>{}, F_{}, integral_constant<bool, (r > 0)>{}, F_{}, kt);
      ++kt;
    }
  });

  // ================= epilogue: the ring is idle =================
  float* const c_scale = reinterpret_cast<float*>(ring);              // [BN] s_a * s_w
  float* const c_bias = c_scale + BN;                                  // [BN]
  float* const c_g = c_bias + BN;                                      // [BN] gamma~ / s~
  float* const c_h = c_g + BN;                                         // [BN] beta~ / s~ + z~
  int* const c_cs = reinterpret_cast<int*>(c_h + BN);                  // [BN] (a_off - z_a) * colsum_w
  float* const stats = reinterpret_cast<float*>(c_cs + BN);            // row statistics: partial sums, then rstd and -mean * rstd
  float* const stage = stats + 4 * 64 * 2 + 64 * 2 + wave * (32 * PITCH);
  static_assert(5 * BN * 4 + (4 * 64 * 2 + 64 * 2) * 4 + 4 * 32 * PITCH * 4 <= S * STAGE, "epilogue scratch fits the idle ring");
  __syncthreads();
  for (int n = tid; n < BN; n += 256) {
    c_scale[n] = p.s_a * p.s_b[n];
    c_bias[n] = p.bias ? p.bias[n] : 0.f;
    c_g[n] = (float)((double)P.gamma_t[n] * P.inv_s);
    c_h[n] = (float)((P.beta_t ? (double)P.beta_t[n] * P.inv_s : 0.0) + P.zcode);
    c_cs[n] = (p.da != 0 && p.colsum_b) ? p.da * p.colsum_b[n] : 0;
  }
  __syncthreads();

  const int rrow = lane >> 4, rcol = (lane & 15) * 4;       // row layout: 4 rows x 16 float4 per pass
  const bool corr = p.da != 0;
  float4 val[TM][NCH][8];                                   // the tile in row layout: token i*32 + r*4 + rrow, channels wn0 + c*64 + rcol .. +3
  float s1[TM][8], s2[TM][8];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int r = 0; r < 8; ++r) { s1[i][r] = 0.f; s2[i][r] = 0.f; }
  // residual segments of a piece are requested one piece ahead, so that only the first request's latency is exposed
  auto request_residual = [&](int pc, float4 (&res)[8]) {
    const int i = pc / NCH, c = pc % NCH;
    const int ncol = wn0 + c * 64 + rcol;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int m = m0 + i * 32 + r * 4 + rrow;
      res[r] = m < Mi ? *reinterpret_cast<const float4*>(p.residual + (int64_t)m * p.ldr + ncol) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  float4 res_cur[8], res_nxt[8];
  request_residual(0, res_cur);
#pragma unroll
  for (int pc = 0; pc < TM * NCH; ++pc) {
    const int i = pc / NCH, c = pc % NCH;
    const int ncol = wn0 + c * 64 + rcol;
    if (pc + 1 < TM * NCH) request_residual(pc + 1, res_nxt);
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int j = c * 2 + jj;
        const int nl = wn0 + j * 32 + 8 * g + half * 4;
        const float4 sc = *reinterpret_cast<const float4*>(&c_scale[nl]);
        const float4 bi = *reinterpret_cast<const float4*>(&c_bias[nl]);
        int t[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = acc[j][i][4 * g + e];
        if (corr) {
          const v4i cs = *reinterpret_cast<const v4i*>(&c_cs[nl]);
#pragma unroll
          for (int e = 0; e < 4; ++e) t[e] += cs[e];
        }
        *reinterpret_cast<float4*>(stage + l32 * PITCH + jj * 32 + 8 * g + half * 4) =
            make_float4(fmaf((float)t[0], sc.x, bi.x), fmaf((float)t[1], sc.y, bi.y), fmaf((float)t[2], sc.z, bi.z), fmaf((float)t[3], sc.w, bi.w));
      }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // this wavefront's own writes; nobody else touches `stage`
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int m = m0 + i * 32 + r * 4 + rrow;
      const float4 y = *reinterpret_cast<const float4*>(stage + (r * 4 + rrow) * PITCH + rcol);
      const float4 v = make_float4(y.x + res_cur[r].x, y.y + res_cur[r].y, y.z + res_cur[r].z, y.w + res_cur[r].w);
      val[i][c][r] = v;
      s1[i][r] += (v.x + v.y) + (v.z + v.w);
      s2[i][r] = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, s2[i][r]))));
      if (m < Mi) *reinterpret_cast<float4*>(p.out_f32 + (int64_t)m * p.ldf + ncol) = v;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // reads done before the next piece overwrites the region
#pragma unroll
    for (int r = 0; r < 8; ++r) res_cur[r] = res_nxt[r];
  }
  // ---- row statistics: the 16 lanes of a DPP row share a token (float32 partial sums of 12 .. 48 values each), the four
  //      wavefronts meet in LDS, and wavefront 0 finishes one token per lane in float64 ----
  auto sum16f = [](float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
    return v;
  };
  float* const part = reinterpret_cast<float*>(stats);                 // [4 wavefronts][64 rows][2]
  float* const rowc = part + 4 * 64 * 2;                               // [64 rows][2]: rstd, -mean * rstd
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const float a = sum16f(s1[i][r]), b = sum16f(s2[i][r]);
      if ((lane & 15) == 0) {
        const int row = i * 32 + r * 4 + rrow;
        *reinterpret_cast<float2*>(&part[(wave * 64 + row) * 2]) = make_float2(a, b);
      }
    }
  __syncthreads();
  if (wave == 0) {
    double a = 0.0, b = 0.0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float2 t2 = *reinterpret_cast<const float2*>(&part[(w * 64 + lane) * 2]);
      a += (double)t2.x; b += (double)t2.y;
    }
    const double invD = 1.0 / (double)BN;
    double mean = 0.0, var = b * invD;
    if (P.norm_kind == RQ_NORM_LAYERNORM) {
      mean = a * invD;
      var = fma(-mean, mean, var);
      var = var < 0.0 ? 0.0 : var;
    }
    double rstd = (double)__builtin_amdgcn_rsqf((float)(var + P.eps));
    rstd = rstd * fma(-0.5 * (var + P.eps), rstd * rstd, 1.5);
    rstd = rstd * fma(-0.5 * (var + P.eps), rstd * rstd, 1.5);
    *reinterpret_cast<float2*>(&rowc[lane * 2]) = make_float2((float)rstd, (float)(-mean * rstd));
  }
  __syncthreads();
  float4 gq[NCH], hq[NCH];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    gq[c] = *reinterpret_cast<const float4*>(&c_g[wn0 + c * 64 + rcol]);
    hq[c] = *reinterpret_cast<const float4*>(&c_h[wn0 + c * 64 + rcol]);
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int row = i * 32 + r * 4 + rrow;
      const int m = m0 + row;
      const float2 rc = *reinterpret_cast<const float2*>(&rowc[row * 2]);
      const float rf = rc.x, nf = rc.y;
      int rsum = 0;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const float4 v = val[i][c][r];
        unsigned w = 0;
        w = __builtin_amdgcn_cvt_pk_u8_f32(fminf(fmaf(fmaf(v.x, rf, nf), gq[c].x, hq[c].x), P.qmaxf), 0, w);
        w = __builtin_amdgcn_cvt_pk_u8_f32(fminf(fmaf(fmaf(v.y, rf, nf), gq[c].y, hq[c].y), P.qmaxf), 1, w);
        w = __builtin_amdgcn_cvt_pk_u8_f32(fminf(fmaf(fmaf(v.z, rf, nf), gq[c].z, hq[c].z), P.qmaxf), 2, w);
        w = __builtin_amdgcn_cvt_pk_u8_f32(fminf(fmaf(fmaf(v.w, rf, nf), gq[c].w, hq[c].w), P.qmaxf), 3, w);
        w = ((w | 0x80808080u) - (P.off4 & 0x7F7F7F7Fu)) ^ ((w ^ ~P.off4) & 0x80808080u);     // stored = code - off per byte
        if (P.rowsum) rsum = __builtin_amdgcn_sdot4((int)w, 0x01010101, rsum, false);
        if (m < Mi) *reinterpret_cast<unsigned*>(P.q + (int64_t)m * P.ldq2 + wn0 + c * 64 + rcol) = w;
      }
      if (P.rowsum) {
        rsum = sum16_i(rsum);
        if ((lane & 15) == 0 && m < Mi) atomicAdd(P.rowsum + m, rsum);       // four wavefronts per token; the caller zeroes rowsum
      }
    }
}

template <int TN>
rq_status launch(rq_ctx* ctx, const RowLnParams& P) {
  constexpr int S = TN <= 2 ? 6 : (TN <= 4 ? 5 : 4);
  constexpr int lds_bytes = S * (64 * 64 + 128 * TN * 32);
  static_assert(lds_bytes <= 160 * 1024, "one workgroup per CU");
  static rq_once_per_device lds_attr;
  RQ_HIP(rq_allow_dynamic_lds(ctx, lds_attr, reinterpret_cast<const void*>(&qgemm_rowln_kernel<TN, S>), lds_bytes));
  const unsigned blocks = (unsigned)((P.g.M + 63) / 64);
  hipLaunchKernelGGL((qgemm_rowln_kernel<TN, S>), dim3(blocks), dim3(256), lds_bytes, ctx->stream, P);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

}  // namespace

bool rq_qgemm_rowln_applies(const rq_gemm_desc* g, const rq_ln_desc* ln) {
  return g->b_format == RQ_W_U4 && g->N % 256 == 0 && g->N <= 768 && g->K % 64 == 0 && g->act == RQ_ACT_NONE && g->residual &&
         g->out_f32 && !g->out_q && !g->out_acc && g->batch_outer <= 1 && g->batch_inner <= 1 && ln->bits <= 6 && !ln->rowsum &&
         (double)g->M * (double)g->lda < 4.0e9 && (double)g->N * (double)g->ldb < 4.0e9;
}

rq_status rq_launch_qgemm_rowln(rq_ctx* ctx, const rq_gemm_desc* d, const rq_ln_desc* ln) {
  RowLnParams P;
  GemmParams& p = P.g;
  std::memset(&P, 0, sizeof P);
  p.M = d->M; p.N = d->N; p.K = d->K;
  p.A = d->A; p.lda = d->lda;
  p.B = static_cast<const uint8_t*>(d->B); p.ldb = d->ldb;
  p.s_b = d->s_b; p.z_b = d->z_b; p.colsum_b = d->colsum_b; p.bias = d->bias;
  p.s_a = d->s_a; p.da = d->a_off - d->z_a;
  p.residual = d->residual; p.ldr = d->ldr; p.out_f32 = d->out_f32; p.ldf = d->ldf;
  P.gamma_t = ln->gamma_t; P.beta_t = ln->beta_t;
  P.inv_s = 1.0 / (double)ln->s_tilde; P.zcode = (double)ln->z_tilde; P.eps = ln->eps;
  P.qmaxf = (float)((1 << ln->bits) - 1);
  P.off4 = (unsigned)(ln->store_off & 0xFF) * 0x01010101u;
  P.norm_kind = ln->norm_kind;
  P.q = ln->q; P.ldq2 = ln->ldq; P.rowsum = ln->rowsum;
  switch (d->N / 128) {
    case 2: return launch<2>(ctx, P);
    case 4: return launch<4>(ctx, P);
    case 6: return launch<6>(ctx, P);
  }
  return rq_fail(ctx, RQ_ERR_SHAPE, "rq_qgemm_ln_quant: N = %d is not 256, 512 or 768", d->N);
}
