// Fused Q.K^T + Softmax-log2 quantizer: entry point; the kernels are instantiated per head width in their own files.
#include "qk_softmax.h"

using rqks::QksParams;
rq_status rq_launch_qk_softmax_d32(rq_ctx* ctx, const rqks::QksParams& p, int64_t groups);
rq_status rq_launch_qk_softmax_d64(rq_ctx* ctx, const rqks::QksParams& p, int64_t groups);
rq_status rq_launch_qk_softmax_d128(rq_ctx* ctx, const rqks::QksParams& p, int64_t groups);
rq_status rq_launch_qk_softmax_long(rq_ctx* ctx, const rqks::QksParams& p, int d_head);
bool rq_attn_stream_supported(int N, int d_head, int bits_p, bool has_bias);
rq_status rq_launch_attn_stream(rq_ctx* ctx, const rqks::QksParams& p, int d_head);


extern "C" int32_t rq_attn_fused_supported(int32_t N, int32_t d_head, int32_t bits_p, int32_t has_bias) {
  if (N <= 0 || N > 288 || bits_p < 2 || !(d_head == 32 || d_head == 64 || d_head == 128)) return 0;
  const int nt = (N + 31) / 32;
  if (!rqks::fused_pv_supported(d_head / 32, nt)) return 0;
  if (bits_p <= 4 && !has_bias) return 1;
  return bits_p <= 6 && nt <= rqks::FUSED_EXT_TILES ? 1 : 0;      // with a bias and / or codes of 5 or 6 bits
}

// Where the one-kernel attention is also the faster choice: up to 8 key tiles, and nine where the streamed kernel
// serves them.  (Nine tiles on the 8 wavefronts of the register-resident kernel take two rounds per group;
// rq_qk_softmax_log2_quant + rq_attn_pv are then as fast or faster: 257 keys, d_head 64, 1024 groups: 117 us against
// 53 + 51 us.)
bool rq_attn_fused_preferred(int N, int d_head, int bits_p, bool has_bias) {
  if (!rq_attn_fused_supported(N, d_head, bits_p, has_bias)) return false;
  return (N + 31) / 32 <= 8 || rq_attn_stream_supported(N, d_head, bits_p, has_bias);
}

rq_status rq_launch_attn_fused(rq_ctx* ctx, const rq_attn_fused_desc* d) {
  QksParams p;
  p.Q = d->Q; p.K = d->K; p.V = d->V; p.ldq = d->ld_tok; p.ldk = d->ld_tok; p.so = (int64_t)d->N * d->ld_tok; p.si = d->d_head;
  p.H = d->H; p.N = d->N; p.dq = d->q_off - d->z_q; p.dk = d->k_off - d->z_k; p.dv = d->v_off - d->z_v;
  p.bias = d->bias; p.causal = 0;
  p.c1 = d->logit_scale * 1.4426950408889634; p.log2s = log2((double)d->s_log); p.qmax = (1 << d->bits_p) - 1;
  p.codes = d->codes; p.ld = d->ld; p.tiles = (d->N + 31) / 32;
  const double ss = (double)d->s_log * (double)d->s_v;
  p.a_even = -ss / 128.0;
  p.a_odd = -ss / (128.0 * 1.4142135623730951);
  p.out_f32 = d->out_f32; p.ldf = d->ldf; p.out_q = d->out_q; p.ldo = d->ldq;
  p.inv_so = d->out_q ? 1.0 / (double)d->s_o : 0.0;
  p.zo = d->z_o - d->off_o; p.lo = -d->off_o; p.hi = (1 << d->bits_o) - 1 - d->off_o;
  p.G = d->batch * d->H;
  p.zero_max = (d->flags & RQ_LOG_ZERO_AT_MAX_CODE) != 0;
  if (rq_attn_stream_supported(d->N, d->d_head, d->bits_p, d->bias != nullptr)) return rq_launch_attn_stream(ctx, p, d->d_head);
  const int ks = d->d_head / 32;
  if (ks == 1) return rq_launch_qk_softmax_d32(ctx, p, p.G);
  if (ks == 2) return rq_launch_qk_softmax_d64(ctx, p, p.G);
  return rq_launch_qk_softmax_d128(ctx, p, p.G);
}

// Rows of up to 288 keys keep their logits in registers; longer rows form them twice, which is implemented without an
// additive bias only.
bool rq_qk_softmax_supported(int N, int d_head, bool has_bias) {
  return (N <= 288 || (!has_bias && N <= 65536)) && (d_head == 32 || d_head == 64 || d_head == 128);
}

// Q, K: token-major int8 (row b*N + i, column h*d_head + c), stored code - off.  codes: [batch*H, N, ld].
rq_status rq_launch_qk_softmax(rq_ctx* ctx, const int8_t* Q, const int8_t* K, int64_t ld_tok, int64_t batch, int H, int N,
                               int d_head, int q_off, int z_q, int k_off, int z_k, double logit_scale, const float* bias,
                               int mask, float s_log, int bits, uint8_t* codes, int64_t ld) {
  QksParams p;
  p.V = nullptr; p.dv = 0; p.out_f32 = nullptr; p.out_q = nullptr; p.zero_max = 0;
  p.Q = Q; p.K = K; p.ldq = ld_tok; p.ldk = ld_tok; p.so = (int64_t)N * ld_tok; p.si = d_head;
  p.H = H; p.N = N; p.dq = q_off - z_q; p.dk = k_off - z_k; p.bias = bias; p.causal = mask == RQ_MASK_CAUSAL;
  p.c1 = logit_scale * 1.4426950408889634; p.log2s = log2((double)s_log); p.qmax = (1 << bits) - 1;
  p.codes = codes; p.ld = ld; p.tiles = (N + 31) / 32;
  const int64_t groups = batch * H;
  p.G = groups;
  const int ks = d_head / 32;
  if (N > 288) {
    if (bias) return rq_fail(ctx, RQ_ERR_SHAPE, "fused Q.K^T + softmax: rows of %d keys with a bias are not supported", N);
    return rq_launch_qk_softmax_long(ctx, p, d_head);
  }
  if (ks == 1) return rq_launch_qk_softmax_d32(ctx, p, groups);
  if (ks == 2) return rq_launch_qk_softmax_d64(ctx, p, groups);
  if (ks == 4) return rq_launch_qk_softmax_d128(ctx, p, groups);
  return rq_fail(ctx, RQ_ERR_SHAPE, "fused Q.K^T + softmax: N = %d, d_head = %d not supported", N, d_head);
}
