// Weight-mode rq_qgemm for a handful of tokens (decode-style, M <= 12) with packed 4-bit weights: a matrix-vector
// product bound by the weight bytes (0.5 B per multiply-add), so the matrix cores are not used.
//   acc[m, n] = sum_k (a[m, k] - z_a) (w[n, k] - z_w[n])      exact int32, same contract as the MFMA kernels
// Each wavefront owns whole weight rows: a lane fetches 16 packed bytes (32 codes) per 2048-wide slice of K, splits the
// nibbles with one `and` / `shift+and` per 4 codes (raw codes: the zero-point goes into the rank-1 correction
// z_w[n] * rowsum_a[m], the row sums come from the activation registers), multiplies with v_dot4 against the activation
// slice it keeps in registers, and the 64 partial sums meet in a DPP reduction.  Several rows are in flight per wavefront.
#include "qgemm_common.h"

namespace {

using rqg::GemmParams;
typedef int v4i __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int wave_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);    // lane ^ 1
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);    // lane ^ 2
  v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);   // row_half_mirror
  v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);   // row_mirror
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}

// NCH = ceil(K / 2048) slices, MP tokens per pass (NCH * MP * 8 activation registers), R rows in flight per wavefront
template <int NCH, int MP, int R, bool GATED>
__global__ __launch_bounds__(256) void qgemv_kernel(const GemmParams p, int m_base) {
  const int lane = threadIdx.x & 63;
  const int wave_g = blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = gridDim.x * 4;
  constexpr bool gated = GATED;                            // SiLU(gate) * up: a unit is a gate row and its up row
  constexpr int RPU = GATED ? 2 : 1;                       // weight rows per output column
  const int units = gated ? p.N / 2 : p.N;                 // output columns
  const int mcount = (int)p.M - m_base < MP ? (int)p.M - m_base : MP;
  // ---- this lane's slices of the activations: codes k = c * 2048 + lane * 32 .. + 31 ----
  v4i a[NCH][MP][2];
  int rowsum[MP];
#pragma unroll
  for (int m = 0; m < MP; ++m) {
    int rs = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int k = c * 2048 + lane * 32;
      const bool ok = k < p.K && m < mcount;
      const int8_t* src = p.A + (int64_t)(m_base + (m < mcount ? m : 0)) * p.lda + (ok ? k : 0);
      a[c][m][0] = ok ? *reinterpret_cast<const v4i*>(src) : v4i{0, 0, 0, 0};
      a[c][m][1] = ok ? *reinterpret_cast<const v4i*>(src + 16) : v4i{0, 0, 0, 0};
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        rs = __builtin_amdgcn_sdot4(a[c][m][0][d], 0x01010101, rs, false);
        rs = __builtin_amdgcn_sdot4(a[c][m][1][d], 0x01010101, rs, false);
      }
    }
    rowsum[m] = wave_sum(rs);
  }
  for (int u0 = wave_g * R; u0 < units; u0 += nwaves * R) {
    int dot[R][RPU][MP];
    v4i w[R][RPU][NCH];
    // ---- request every packed slice of these rows first ----
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int g = 0; g < RPU; ++g)
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
          const int u = u0 + r < units ? u0 + r : units - 1;
          const int n = gated ? (u / 32) * 64 + (u % 32) + 32 * g : u;
          const int k = c * 2048 + lane * 32;
          w[r][g][c] = k < p.K ? *reinterpret_cast<const v4i*>(p.B + (int64_t)n * p.ldb + (k >> 1)) : v4i{0, 0, 0, 0};
        }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int g = 0; g < RPU; ++g) {
#pragma unroll
        for (int m = 0; m < MP; ++m) dot[r][g][m] = 0;
        {
#pragma unroll
          for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int d = 0; d < 4; ++d) {
              // packed dword d holds codes 8d .. 8d+3 in the low nibbles and 8d+4 .. 8d+7 in the high nibbles
              const int lo = w[r][g][c][d] & 0x0F0F0F0F, hi = (w[r][g][c][d] >> 4) & 0x0F0F0F0F;
#pragma unroll
              for (int m = 0; m < MP; ++m) {
                const int a_lo = d < 2 ? a[c][m][0][2 * d] : a[c][m][1][2 * d - 4];
                const int a_hi = d < 2 ? a[c][m][0][2 * d + 1] : a[c][m][1][2 * d - 3];
                dot[r][g][m] = __builtin_amdgcn_sdot4(a_lo, lo, dot[r][g][m], false);
                dot[r][g][m] = __builtin_amdgcn_sdot4(a_hi, hi, dot[r][g][m], false);
              }
            }
#pragma unroll
          for (int m = 0; m < MP; ++m) dot[r][g][m] = wave_sum(dot[r][g][m]);
        }
      }
    // ---- lane (r * MP + m) finishes output (unit u0 + r, token m_base + m) ----
    const int r_l = lane / MP, m_l = lane % MP;
    if (r_l < R && u0 + r_l < units && m_l < mcount) {
      int d0 = 0, d1 = 0, rs = 0;
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < MP; ++m)
          if (r == r_l && m == m_l) { d0 = dot[r][0][m]; d1 = dot[r][RPU - 1][m]; rs = rowsum[m]; }
      const int u = u0 + r_l;
      const int64_t mt = m_base + m_l;
      const int n = gated ? (u / 32) * 64 + (u % 32) : u;
      // true = sum (a' + da)(w - z) = sum a'w - z rowsum(a') + da colsum(w - z)
      auto true_acc = [&](int dotv, int nn) { return dotv - p.z_b[nn] * rs + ((p.da != 0 && p.colsum_b) ? p.da * p.colsum_b[nn] : 0); };
      const int t0 = true_acc(d0, n);
      if (p.out_acc) {
        p.out_acc[mt * p.ldacc + n] = t0;
        if (gated) p.out_acc[mt * p.ldacc + n + 32] = true_acc(d1, n + 32);
      }
      float y = fmaf((float)t0, p.s_a * p.s_b[n], p.bias ? p.bias[n] : 0.f);
      if (p.act == RQ_ACT_GELU) y = rqg::gelu_f(y);
      else if (gated) {
        const float up = fmaf((float)true_acc(d1, n + 32), p.s_a * p.s_b[n + 32], p.bias ? p.bias[n + 32] : 0.f);
        y = rqg::silu_f(y) * up;
      }
      if (p.residual) y += p.residual[mt * p.ldr + u];
      if (p.out_f32) p.out_f32[mt * p.ldf + u] = y;
      if (p.out_q) {
        int sg = p.n_seg > 1 ? u / p.seg_len : 0;
        sg = sg < p.n_seg ? sg : p.n_seg - 1;
        const float vf = fmaf(y, p.inv_so[sg], p.zcode[sg]);
        float v = fminf(fmaxf(rintf(vf), 0.f), p.qmaxf);
        if (p.act == RQ_ACT_NONE && p.qmaxf > 127.f && fabsf(vf - rintf(vf)) > 0.5f - rqg::TIE_GUARD) {   // 8-bit codes near a tie: float64
          const float r = p.residual ? p.residual[mt * p.ldr + u] : 0.f;
          v = (float)(rqg::requant_exact4(p, t0, t0, t0, t0, n, r, r, r, r, sg) & 0xFFu);
        }
        p.out_q[mt * p.ldq + u] = (int8_t)((int)v - (p.off4[sg] & 0xFF));
      }
    }
  }
}

template <int NCH, int MP>
void launch(rq_ctx* ctx, const GemmParams& p) {
  constexpr int R = NCH >= 4 ? 2 : 4;            // rows in flight per wavefront, bounded by the registers their slices take
  const bool gated = p.act == RQ_ACT_SILU_GATED;
  const int units = gated ? p.N / 2 : p.N;
  int64_t blocks = ((int64_t)units + 4 * R - 1) / (4 * R);
  const int64_t cap = (int64_t)ctx->num_cu * 4;
  if (blocks > cap) blocks = cap;
  for (int m_base = 0; m_base < (int)p.M; m_base += MP) {
    if (gated) hipLaunchKernelGGL((qgemv_kernel<NCH, MP, R, true>), dim3((unsigned)blocks), dim3(256), 0, ctx->stream, p, m_base);
    else hipLaunchKernelGGL((qgemv_kernel<NCH, MP, R, false>), dim3((unsigned)blocks), dim3(256), 0, ctx->stream, p, m_base);
  }
}

}  // namespace

bool rq_qgemv_applies(const rqg::GemmParams& p, bool w4) {
  return w4 && p.M <= 12 && p.K <= 16384 && !p.centered && p.lda % 16 == 0 && (reinterpret_cast<uintptr_t>(p.A) & 15) == 0 &&
         (reinterpret_cast<uintptr_t>(p.B) & 15) == 0 && (p.ldb % 16) == 0 && p.K % 64 == 0;
}

rq_status rq_launch_qgemv_w4(rq_ctx* ctx, const rqg::GemmParams& p) {
  const int nch = (p.K + 2047) / 2048;
  if (nch <= 1) { if (p.M >= 4) launch<1, 4>(ctx, p); else launch<1, 1>(ctx, p); }
  else if (nch <= 2) { if (p.M >= 4) launch<2, 4>(ctx, p); else launch<2, 1>(ctx, p); }
  else if (nch <= 4) { if (p.M >= 2) launch<4, 2>(ctx, p); else launch<4, 1>(ctx, p); }
  else if (nch <= 6) { if (p.M >= 2) launch<6, 2>(ctx, p); else launch<6, 1>(ctx, p); }
  else launch<8, 1>(ctx, p);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}
