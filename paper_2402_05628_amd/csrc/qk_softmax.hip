// Fused Q.K^T + Softmax-log2 quantizer: entry point; the kernels are instantiated per head width in their own files.
#include "qk_softmax.h"

using rqks::QksParams;
rq_status rq_launch_qk_softmax_d32(rq_ctx* ctx, const rqks::QksParams& p, int64_t groups);
rq_status rq_launch_qk_softmax_d64(rq_ctx* ctx, const rqks::QksParams& p, int64_t groups);
rq_status rq_launch_qk_softmax_d128(rq_ctx* ctx, const rqks::QksParams& p, int64_t groups);


bool rq_qk_softmax_supported(int N, int d_head) { return N <= 288 && (d_head == 32 || d_head == 64 || d_head == 128); }

// Q, K: token-major int8 (row b*N + i, column h*d_head + c), stored code - off.  codes: [batch*H, N, ld].
rq_status rq_launch_qk_softmax(rq_ctx* ctx, const int8_t* Q, const int8_t* K, int64_t ld_tok, int64_t batch, int H, int N,
                               int d_head, int q_off, int z_q, int k_off, int z_k, double logit_scale, const float* bias,
                               int mask, float s_log, int bits, uint8_t* codes, int64_t ld) {
  QksParams p;
  p.Q = Q; p.K = K; p.ldq = ld_tok; p.ldk = ld_tok; p.so = (int64_t)N * ld_tok; p.si = d_head;
  p.H = H; p.N = N; p.dq = q_off - z_q; p.dk = k_off - z_k; p.bias = bias; p.causal = mask == RQ_MASK_CAUSAL;
  p.c1 = logit_scale * 1.4426950408889634; p.log2s = log2((double)s_log); p.qmax = (1 << bits) - 1;
  p.codes = codes; p.ld = ld; p.tiles = (N + 31) / 32;
  const int64_t groups = batch * H;
  p.G = groups;
  const int ks = d_head / 32;
  if (ks == 1) return rq_launch_qk_softmax_d32(ctx, p, groups);
  if (ks == 2) return rq_launch_qk_softmax_d64(ctx, p, groups);
  if (ks == 4) return rq_launch_qk_softmax_d128(ctx, p, groups);
  return rq_fail(ctx, RQ_ERR_SHAPE, "fused Q.K^T + softmax: N = %d, d_head = %d not supported", N, d_head);
}
