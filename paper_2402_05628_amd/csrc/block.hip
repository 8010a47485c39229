// rq_block_forward: host-side sequencing of the block's kernels on one stream, no host synchronization
// (Eqs. for X-bar and Y and the attention Eq. of Section "Transformer blocks").
// Attention is processed in chunks of batch items sized so that the int32 logits and the codes of one chunk
// stay resident in the 256 MB last-level cache between Q.K^T, Softmax-log2 and P.V.
#include <cmath>
#include <cstring>

#include "rq_internal.h"

namespace {

constexpr size_t ALIGN = 256;
size_t up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

struct Plan {
  int64_t T, batch, seq, ld, bchunk;
  size_t o_a, o_rowsum, o_qkv, o_acc, o_codes, o_o, o_xbar, o_hid, total;
};

int64_t g_attn_chunk_bytes = 64ll << 20;

Plan make_plan(const rq_block_params* p, int64_t batch, int64_t seq) {
  Plan pl;
  pl.batch = batch; pl.seq = seq; pl.T = batch * seq;
  pl.ld = (seq + 15) / 16 * 16;
  const int64_t per_item = (int64_t)p->H * seq * pl.ld * 5;
  pl.bchunk = g_attn_chunk_bytes / (per_item > 0 ? per_item : 1);
  if (pl.bchunk < 1) pl.bchunk = 1;
  if (pl.bchunk > batch) pl.bchunk = batch;
  const int64_t gch = pl.bchunk * p->H;
  size_t o = 0;
  pl.o_a = o; o += up((size_t)pl.T * p->D);
  pl.o_rowsum = o; o += up((size_t)pl.T * 4);
  pl.o_qkv = o; o += up((size_t)pl.T * 3 * p->D);
  pl.o_acc = o; o += up((size_t)gch * seq * pl.ld * 4);
  pl.o_codes = o; o += up((size_t)gch * seq * pl.ld);
  pl.o_o = o; o += up((size_t)pl.T * p->D);
  pl.o_xbar = o; o += up((size_t)pl.T * p->D * 4);
  pl.o_hid = o; o += up((size_t)pl.T * p->Dm);
  pl.total = o;
  return pl;
}

void fill_linear(rq_gemm_desc& g, const rq_qlinear& l, const int8_t* A, int64_t M, int64_t lda, float s_a, int z_a, int a_off,
                 const int32_t* rowsum) {
  std::memset(&g, 0, sizeof g);
  g.M = M; g.N = l.N; g.K = l.K;
  g.A = A; g.lda = lda; g.a_off = a_off; g.z_a = z_a; g.s_a = s_a;
  g.B = l.w; g.ldb = l.format == RQ_W_U4 ? l.K / 2 : l.K; g.b_format = l.format;
  g.s_b = l.s_w; g.z_b = l.z_w; g.colsum_b = l.colsum_w; g.rowsum_a = rowsum; g.bias = l.bias;
  g.batch_outer = 1; g.batch_inner = 1; g.n_seg = 1;
}

rq_status check_linear(rq_ctx* ctx, const char* name, const rq_qlinear& l, int N, int K) {
  RQ_REQUIRE(l.N == N && l.K == K, RQ_ERR_SHAPE, "rq_block_forward: %s is %d x %d, expected %d x %d", name, l.N, l.K, N, K);
  RQ_REQUIRE(l.w && l.s_w && l.z_w && l.colsum_w, RQ_ERR_INVALID_ARG, "rq_block_forward: %s has NULL arrays", name);
  RQ_REQUIRE(l.format == RQ_W_I8_BAKED || l.format == RQ_W_I8_CENTERED || l.format == RQ_W_U4, RQ_ERR_INVALID_ARG,
             "rq_block_forward: %s format %d", name, l.format);
  return RQ_OK;
}

}  // namespace

extern "C" {

rq_status rq_set_attn_chunk_bytes(int64_t bytes) {
  if (bytes < (1 << 20)) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_set_attn_chunk_bytes: at least 1 MiB");
  g_attn_chunk_bytes = bytes;
  return RQ_OK;
}

size_t rq_block_workspace_bytes(const rq_block_params* p, int64_t batch, int64_t seq) {
  if (!p || batch <= 0 || seq <= 0 || p->D <= 0 || p->H <= 0 || p->Dm <= 0) return 0;
  return make_plan(p, batch, seq).total;
}

rq_status rq_block_forward(rq_ctx* ctx, const rq_block_params* p, const float* x, float* y, int64_t batch, int64_t seq,
                           void* workspace, size_t workspace_bytes) {
  if (!ctx) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_block_forward: ctx is NULL");
  RQ_REQUIRE(p && x && y && workspace, RQ_ERR_INVALID_ARG, "rq_block_forward: params, x, y, workspace must be non-NULL");
  RQ_REQUIRE(batch > 0 && seq > 0, RQ_ERR_SHAPE, "rq_block_forward: batch = %lld, seq = %lld", (long long)batch, (long long)seq);
  RQ_REQUIRE(p->D > 0 && p->H > 0 && p->Dm > 0 && p->D % p->H == 0, RQ_ERR_SHAPE, "rq_block_forward: D = %d, H = %d, Dm = %d", p->D,
             p->H, p->Dm);
  const int D = p->D, H = p->H, dh = D / H, Dm = p->Dm;
  RQ_REQUIRE(dh == 32 || dh == 64 || dh == 128, RQ_ERR_SHAPE, "rq_block_forward: d_head = %d must be 32, 64 or 128", dh);
  RQ_REQUIRE(D % 64 == 0 && Dm % 64 == 0, RQ_ERR_SHAPE, "rq_block_forward: D and Dm must be multiples of 64");
  RQ_REQUIRE(seq <= 4096, RQ_ERR_SHAPE, "rq_block_forward: seq = %lld exceeds 4096", (long long)seq);
  RQ_REQUIRE(p->act == RQ_ACT_GELU || p->act == RQ_ACT_SILU_GATED, RQ_ERR_INVALID_ARG, "rq_block_forward: act %d", p->act);
  RQ_REQUIRE(p->bits_a >= 2 && p->bits_a <= 8 && p->bits_p >= 2 && p->bits_p <= 8, RQ_ERR_INVALID_ARG,
             "rq_block_forward: bits_a = %d, bits_p = %d", p->bits_a, p->bits_p);
  RQ_REQUIRE(p->ln1_gamma_t && p->ln2_gamma_t, RQ_ERR_INVALID_ARG, "rq_block_forward: LayerNorm gammas must be non-NULL");
  const bool gated = p->act == RQ_ACT_SILU_GATED;
  rq_status st;
  if ((st = check_linear(ctx, "qkv", p->qkv, 3 * D, D)) != RQ_OK) return st;
  if ((st = check_linear(ctx, "proj", p->proj, D, D)) != RQ_OK) return st;
  if ((st = check_linear(ctx, "fc1", p->fc1, gated ? 2 * Dm : Dm, D)) != RQ_OK) return st;
  if ((st = check_linear(ctx, "fc2", p->fc2, D, Dm)) != RQ_OK) return st;
  RQ_REQUIRE(rq_aligned(x, 16) && rq_aligned(y, 16) && rq_aligned(workspace, ALIGN), RQ_ERR_INVALID_ARG,
             "rq_block_forward: x, y need 16-byte and workspace 256-byte alignment");
  const Plan pl = make_plan(p, batch, seq);
  RQ_REQUIRE(workspace_bytes >= pl.total, RQ_ERR_WORKSPACE, "rq_block_forward: workspace has %zu bytes, %zu needed", workspace_bytes,
             pl.total);
  RQ_NEED_DEVICE();

  char* ws = static_cast<char*>(workspace);
  int8_t* a = reinterpret_cast<int8_t*>(ws + pl.o_a);
  int32_t* rowsum = reinterpret_cast<int32_t*>(ws + pl.o_rowsum);
  int8_t* qkv = reinterpret_cast<int8_t*>(ws + pl.o_qkv);
  int32_t* acc = reinterpret_cast<int32_t*>(ws + pl.o_acc);
  uint8_t* codes = reinterpret_cast<uint8_t*>(ws + pl.o_codes);
  int8_t* o = reinterpret_cast<int8_t*>(ws + pl.o_o);
  float* xbar = reinterpret_cast<float*>(ws + pl.o_xbar);
  int8_t* hid = reinterpret_cast<int8_t*>(ws + pl.o_hid);
  const int64_t T = pl.T;
  const int ba = p->bits_a;

  auto need_rowsum = [](const rq_qlinear& l) { return l.format == RQ_W_I8_CENTERED; };

  // ---- LN1 + layer-wise quant -------------------------------------------------------------------------
  const int off1 = rq_store_offset(ba, p->ln1_z);
  {
    rq_ln_desc d;
    std::memset(&d, 0, sizeof d);
    d.T = T; d.D = D; d.norm_kind = p->norm_kind; d.eps = p->eps; d.x = x; d.ldx = D;
    d.gamma_t = p->ln1_gamma_t; d.beta_t = p->ln1_beta_t; d.s_tilde = p->ln1_s; d.z_tilde = p->ln1_z; d.bits = ba;
    d.store_off = off1; d.q = a; d.ldq = D; d.rowsum = need_rowsum(p->qkv) ? rowsum : nullptr;
    rq_prof_begin(ctx, RQ_STEP_LN1);
    st = rq_ln_quant(ctx, &d);
    rq_prof_end(ctx);
    if (st != RQ_OK) return st;
  }
  // ---- QKV projection, re-quantized to the three static activation quantizers ---------------------------
  const int offq = rq_store_offset(ba, p->z_q), offk = rq_store_offset(ba, p->z_k), offv = rq_store_offset(ba, p->z_v);
  {
    rq_gemm_desc g;
    fill_linear(g, p->qkv, a, T, D, p->ln1_s, p->ln1_z, off1, rowsum);
    g.out_q = qkv; g.ldq = 3 * D; g.bits_o = ba; g.n_seg = 3; g.seg_len = D;
    g.s_o[0] = p->s_q; g.s_o[1] = p->s_k; g.s_o[2] = p->s_v;
    g.z_o[0] = p->z_q; g.z_o[1] = p->z_k; g.z_o[2] = p->z_v;
    g.off_o[0] = offq; g.off_o[1] = offk; g.off_o[2] = offv;
    rq_prof_begin(ctx, RQ_STEP_QKV);
    st = rq_qgemm(ctx, &g);
    rq_prof_end(ctx);
    if (st != RQ_OK) return st;
  }
  // ---- attention, chunked over batch items -----------------------------------------------------------------
  const int offo = rq_store_offset(ba, p->z_o);
  for (int64_t b0 = 0; b0 < batch; b0 += pl.bchunk) {
    const int64_t nb = (batch - b0) < pl.bchunk ? (batch - b0) : pl.bchunk;
    const int8_t* qkv_c = qkv + b0 * seq * 3 * D;
    {
      rq_gemm_desc g;
      std::memset(&g, 0, sizeof g);
      g.M = seq; g.N = (int)seq; g.K = dh;
      g.A = qkv_c; g.lda = 3 * D; g.a_off = offq; g.z_a = p->z_q; g.s_a = p->s_q;
      g.B = qkv_c + D; g.ldb = 3 * D; g.b_format = RQ_B_ACT_I8; g.b_off = offk; g.z_b_scalar = p->z_k;
      g.out_acc = acc; g.ldacc = pl.ld; g.acc_stride_group = seq * pl.ld;
      g.batch_outer = nb; g.batch_inner = H;
      g.a_stride_outer = seq * 3 * D; g.a_stride_inner = dh; g.b_stride_outer = seq * 3 * D; g.b_stride_inner = dh;
      g.causal = p->mask == RQ_MASK_CAUSAL;
      rq_prof_begin(ctx, RQ_STEP_QK);
      st = rq_qgemm(ctx, &g);
      rq_prof_end(ctx);
      if (st != RQ_OK) return st;
    }
    {
      rq_softmax_desc d;
      std::memset(&d, 0, sizeof d);
      d.G = nb * H; d.H = H; d.Nq = (int)seq; d.Nk = (int)seq; d.ld = pl.ld; d.acc = acc;
      d.logit_scale = (double)p->s_q * (double)p->s_k / std::sqrt((double)dh);
      d.bias = p->rel_bias; d.mask = p->mask; d.s_log = p->s_log; d.bits = p->bits_p; d.codes = codes;
      rq_prof_begin(ctx, RQ_STEP_SOFTMAX);
      st = rq_softmax_log2_quant(ctx, &d);
      rq_prof_end(ctx);
      if (st != RQ_OK) return st;
    }
    {
      rq_pv_desc d;
      std::memset(&d, 0, sizeof d);
      d.batch = nb; d.H = H; d.Nq = (int)seq; d.Nk = (int)seq; d.d_head = dh; d.ld = pl.ld; d.codes = codes;
      d.V = qkv_c + 2 * D; d.ldv = 3 * D; d.s_log = p->s_log; d.s_v = p->s_v; d.z_v = p->z_v; d.v_off = offv;
      d.bits_p = p->bits_p; d.mask = p->mask;
      d.out_q = o + b0 * seq * D; d.ldq = D; d.s_o = p->s_o; d.z_o = p->z_o; d.off_o = offo; d.bits_o = ba;
      rq_prof_begin(ctx, RQ_STEP_PV);
      st = rq_attn_pv(ctx, &d);
      rq_prof_end(ctx);
      if (st != RQ_OK) return st;
    }
  }
  // ---- output projection + residual ------------------------------------------------------------------------
  if (need_rowsum(p->proj)) {
    rq_prof_begin(ctx, RQ_STEP_AUX);
    st = rq_rowsum_i8(ctx, o, T, D, D, rowsum);
    rq_prof_end(ctx);
    if (st != RQ_OK) return st;
  }
  {
    rq_gemm_desc g;
    fill_linear(g, p->proj, o, T, D, p->s_o, p->z_o, offo, rowsum);
    g.residual = x; g.ldr = D; g.out_f32 = xbar; g.ldf = D;
    rq_prof_begin(ctx, RQ_STEP_PROJ);
    st = rq_qgemm(ctx, &g);
    rq_prof_end(ctx);
    if (st != RQ_OK) return st;
  }
  // ---- LN2 + layer-wise quant ----------------------------------------------------------------------------------
  const int off2 = rq_store_offset(ba, p->ln2_z);
  {
    rq_ln_desc d;
    std::memset(&d, 0, sizeof d);
    d.T = T; d.D = D; d.norm_kind = p->norm_kind; d.eps = p->eps; d.x = xbar; d.ldx = D;
    d.gamma_t = p->ln2_gamma_t; d.beta_t = p->ln2_beta_t; d.s_tilde = p->ln2_s; d.z_tilde = p->ln2_z; d.bits = ba;
    d.store_off = off2; d.q = a; d.ldq = D; d.rowsum = need_rowsum(p->fc1) ? rowsum : nullptr;
    rq_prof_begin(ctx, RQ_STEP_LN2);
    st = rq_ln_quant(ctx, &d);
    rq_prof_end(ctx);
    if (st != RQ_OK) return st;
  }
  // ---- FC1 + activation, re-quantized ------------------------------------------------------------------------------
  const int offh = rq_store_offset(ba, p->z_h);
  {
    rq_gemm_desc g;
    fill_linear(g, p->fc1, a, T, D, p->ln2_s, p->ln2_z, off2, rowsum);
    g.act = p->act; g.out_q = hid; g.ldq = Dm; g.bits_o = ba; g.n_seg = 1; g.seg_len = Dm;
    g.s_o[0] = p->s_h; g.z_o[0] = p->z_h; g.off_o[0] = offh;
    rq_prof_begin(ctx, RQ_STEP_FC1);
    st = rq_qgemm(ctx, &g);
    rq_prof_end(ctx);
    if (st != RQ_OK) return st;
  }
  // ---- FC2 + residual ------------------------------------------------------------------------------------------------
  if (need_rowsum(p->fc2)) {
    rq_prof_begin(ctx, RQ_STEP_AUX);
    st = rq_rowsum_i8(ctx, hid, T, Dm, Dm, rowsum);
    rq_prof_end(ctx);
    if (st != RQ_OK) return st;
  }
  {
    rq_gemm_desc g;
    fill_linear(g, p->fc2, hid, T, Dm, p->s_h, p->z_h, offh, rowsum);
    g.residual = xbar; g.ldr = D; g.out_f32 = y; g.ldf = D;
    rq_prof_begin(ctx, RQ_STEP_FC2);
    st = rq_qgemm(ctx, &g);
    rq_prof_end(ctx);
    if (st != RQ_OK) return st;
  }
  return RQ_OK;
}

}  // extern "C"
