// rq_block_forward: host-side sequencing of the block's kernels on one stream, no host synchronization
// (Eqs. for X-bar and Y and the attention Eq. of Section "Transformer blocks").
// Attention is processed in chunks of batch items sized so that the int32 logits and the codes of one chunk
// stay resident in the 256 MB last-level cache between Q.K^T, Softmax-log2 and P.V.
#include <cmath>
#include <cstring>
#include <mutex>

#include "rq_internal.h"

namespace {

constexpr size_t ALIGN = 256;
size_t up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

struct Plan {
  int64_t T, batch, seq, ld, bchunk;
  size_t o_a, o_rowsum, o_qkv, o_acc, o_codes, o_o, o_xbar, o_hid, total;
  size_t acc_bytes, codes_bytes;
};

void export_layout(const Plan& pl, rq_block_layout* out) {
  out->batch_chunk = pl.bchunk; out->ld = pl.ld;
  out->a = pl.o_a; out->rowsum = pl.o_rowsum; out->qkv = pl.o_qkv; out->logits = pl.o_acc; out->logits_bytes = pl.acc_bytes;
  out->codes = pl.o_codes; out->codes_bytes = pl.codes_bytes; out->o = pl.o_o; out->xbar = pl.o_xbar; out->hidden = pl.o_hid;
  out->total = pl.total;
}

constexpr int64_t DEFAULT_CHUNK_BYTES = 64ll << 20;

// Q.K^T + Softmax-log2 in one kernel (no int32 logits in memory)
bool use_fused(const rq_block_params* p, int64_t seq) {
  return p->attn_path != RQ_ATTN_THREE_KERNELS && p->H > 0 && p->D % p->H == 0 &&
         rq_qk_softmax_supported((int)seq, p->D / p->H, p->rel_bias != nullptr);
}

// the whole attention in one kernel: neither logits nor codes reach memory
bool use_whole(const rq_block_params* p, int64_t seq) {
  return p->attn_path == RQ_ATTN_AUTO && p->H > 0 && p->D % p->H == 0 && p->mask == RQ_MASK_NONE &&
         rq_attn_fused_preferred((int)seq, p->D / p->H, p->bits_p, p->rel_bias != nullptr);
}

// The workspace layout follows the attention path the parameters select; the forward pass and the workspace query
// read the same fields, so the two cannot disagree.
Plan make_plan(const rq_block_params* p, int64_t batch, int64_t seq) {
  Plan pl;
  pl.batch = batch; pl.seq = seq; pl.T = batch * seq;
  pl.ld = (seq + 15) / 16 * 16;
  const bool fused = use_fused(p, seq);       // no int32 logits in memory: only the codes count
  const bool whole = use_whole(p, seq);      // nothing to keep cache-resident between kernels: one chunk
  const int64_t per_item = (int64_t)p->H * seq * pl.ld * (fused ? 1 : 5);
  const int64_t chunk_bytes = p->attn_chunk_bytes > 0 ? p->attn_chunk_bytes : DEFAULT_CHUNK_BYTES;
  pl.bchunk = whole ? batch : chunk_bytes / (per_item > 0 ? per_item : 1);
  if (pl.bchunk < 1) pl.bchunk = 1;
  if (pl.bchunk > batch) pl.bchunk = batch;
  if (batch > 0) {      // equal chunks: a small last chunk would run its kernels on a nearly empty chip
    const int64_t chunks = (batch + pl.bchunk - 1) / pl.bchunk;
    pl.bchunk = (batch + chunks - 1) / chunks;
  }
  const int64_t gch = pl.bchunk * p->H;
  size_t o = 0;
  pl.o_a = o; o += up((size_t)pl.T * p->D);
  pl.o_rowsum = o; o += up((size_t)pl.T * 4);
  pl.o_qkv = o; o += up((size_t)pl.T * 3 * p->D);
  pl.acc_bytes = fused ? 0 : up((size_t)gch * seq * pl.ld * 4);
  pl.codes_bytes = whole ? 0 : up((size_t)gch * seq * pl.ld);
  pl.o_acc = o; o += pl.acc_bytes;
  pl.o_codes = o; o += pl.codes_bytes;
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

size_t rq_block_workspace_bytes(const rq_block_params* p, int64_t batch, int64_t seq) {
  if (!p || batch <= 0 || seq <= 0 || p->D <= 0 || p->H <= 0 || p->Dm <= 0) return 0;
  return make_plan(p, batch, seq).total;
}

rq_status rq_block_workspace_layout(const rq_block_params* p, int64_t batch, int64_t seq, rq_block_layout* out) {
  if (!p || !out || batch <= 0 || seq <= 0 || p->D <= 0 || p->H <= 0 || p->Dm <= 0)
    return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_block_workspace_layout: NULL argument or non-positive size");
  export_layout(make_plan(p, batch, seq), out);
  return RQ_OK;
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
  RQ_REQUIRE(p->attn_path >= RQ_ATTN_AUTO && p->attn_path <= RQ_ATTN_THREE_KERNELS, RQ_ERR_INVALID_ARG,
             "rq_block_forward: attn_path = %d", p->attn_path);
  RQ_REQUIRE(p->attn_chunk_bytes == 0 || p->attn_chunk_bytes >= (1 << 20), RQ_ERR_INVALID_ARG,
             "rq_block_forward: attn_chunk_bytes must be 0 (default) or at least 1 MiB");
  RQ_REQUIRE((p->flags & ~RQ_LOG_ZERO_AT_MAX_CODE) == 0, RQ_ERR_INVALID_ARG, "rq_block_forward: flags = %d", p->flags);
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
  const float* const x_all = x;
  float* const y_all = y;
  // the pass over the batch items [first, first + nbatch): every intermediate is token-major, so a part of the batch works in
  // its own rows of the same workspace arrays
  auto run_part = [&](int64_t first, int64_t nbatch) -> rq_status {
  rq_status st;
  const int64_t t0 = first * seq;
  int8_t* a = reinterpret_cast<int8_t*>(ws + pl.o_a) + t0 * D;
  int32_t* rowsum = reinterpret_cast<int32_t*>(ws + pl.o_rowsum) + t0;
  int8_t* qkv = reinterpret_cast<int8_t*>(ws + pl.o_qkv) + t0 * 3 * D;
  int32_t* acc = reinterpret_cast<int32_t*>(ws + pl.o_acc);
  uint8_t* codes = reinterpret_cast<uint8_t*>(ws + pl.o_codes);
  int8_t* o = reinterpret_cast<int8_t*>(ws + pl.o_o) + t0 * D;
  float* xbar = reinterpret_cast<float*>(ws + pl.o_xbar) + t0 * D;
  int8_t* hid = reinterpret_cast<int8_t*>(ws + pl.o_hid) + t0 * Dm;
  const int64_t T = nbatch * seq;
  const float* x = x_all + t0 * D;
  float* y = y_all + t0 * D;
  const int ba = p->bits_a;

  // Row sums of the stored activation codes: required by centered 8-bit weights; with packed 4-bit weights they let the
  // GEMM multiply raw nibbles.  The LayerNorm kernel emits them for free; computing them for the attention output and the
  // MLP hidden layer would cost a pass of its own, so there only the weights that need them get them.
  auto need_rowsum = [](const rq_qlinear& l) { return l.format == RQ_W_I8_CENTERED; };
  auto ln_rowsum = [](const rq_qlinear& l) { return l.format == RQ_W_I8_CENTERED || l.format == RQ_W_U4; };

  // ---- LN1 + layer-wise quant -------------------------------------------------------------------------
  const int off1 = rq_store_offset(ba, p->ln1_z);
  {
    rq_ln_desc d;
    std::memset(&d, 0, sizeof d);
    d.T = T; d.D = D; d.norm_kind = p->norm_kind; d.eps = p->eps; d.x = x; d.ldx = D;
    d.gamma_t = p->ln1_gamma_t; d.beta_t = p->ln1_beta_t; d.s_tilde = p->ln1_s; d.z_tilde = p->ln1_z; d.bits = ba;
    d.store_off = off1; d.q = a; d.ldq = D; d.rowsum = ln_rowsum(p->qkv) ? rowsum : nullptr;
    rq_prof_begin(ctx, RQ_STEP_LN1);
    st = rq_ln_quant(ctx, &d);
    rq_prof_end(ctx);
    if (st != RQ_OK) return st;
  }
  // ---- QKV projection, re-quantized to the three static activation quantizers ---------------------------
  const int offq = rq_store_offset(ba, p->z_q), offk = rq_store_offset(ba, p->z_k), offv = rq_store_offset(ba, p->z_v);
  {
    rq_gemm_desc g;
    fill_linear(g, p->qkv, a, T, D, p->ln1_s, p->ln1_z, off1, ln_rowsum(p->qkv) ? rowsum : nullptr);
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
  const bool fused = use_fused(p, seq);
  const bool whole = use_whole(p, seq);
  for (int64_t b0 = 0; b0 < nbatch; b0 += pl.bchunk) {
    const int64_t nb = (nbatch - b0) < pl.bchunk ? (nbatch - b0) : pl.bchunk;
    const int8_t* qkv_c = qkv + b0 * seq * 3 * D;
    if (whole) {
      // Q.K^T, Softmax-log2 codes and P.V in one kernel: neither logits nor codes reach memory
      rq_attn_fused_desc d;
      std::memset(&d, 0, sizeof d);
      d.batch = nb; d.H = H; d.N = (int)seq; d.d_head = dh; d.Q = qkv_c; d.K = qkv_c + D; d.V = qkv_c + 2 * D; d.ld_tok = 3 * D;
      d.q_off = offq; d.z_q = p->z_q; d.k_off = offk; d.z_k = p->z_k; d.v_off = offv; d.z_v = p->z_v;
      d.logit_scale = (double)p->s_q * (double)p->s_k / std::sqrt((double)dh);
      d.s_log = p->s_log; d.s_v = p->s_v; d.bits_p = p->bits_p; d.bias = p->rel_bias; d.flags = p->flags;
      d.out_q = o + b0 * seq * D; d.ldq = D; d.s_o = p->s_o; d.z_o = p->z_o; d.off_o = offo; d.bits_o = ba;
      rq_prof_begin(ctx, RQ_STEP_QK);
      st = rq_launch_attn_fused(ctx, &d);
      rq_prof_end(ctx);
      if (st != RQ_OK) return st;
      continue;
    }
    if (fused) {
      rq_prof_begin(ctx, RQ_STEP_QK);
      st = rq_launch_qk_softmax(ctx, qkv_c, qkv_c + D, 3 * D, nb, H, (int)seq, dh, offq, p->z_q, offk, p->z_k,
                                (double)p->s_q * (double)p->s_k / std::sqrt((double)dh), p->rel_bias, p->mask, p->s_log,
                                p->bits_p, codes, pl.ld);
      rq_prof_end(ctx);
      if (st != RQ_OK) return st;
    } else {
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
    }
    {
      rq_pv_desc d;
      std::memset(&d, 0, sizeof d);
      d.batch = nb; d.H = H; d.Nq = (int)seq; d.Nk = (int)seq; d.d_head = dh; d.ld = pl.ld; d.codes = codes;
      d.V = qkv_c + 2 * D; d.ldv = 3 * D; d.s_log = p->s_log; d.s_v = p->s_v; d.z_v = p->z_v; d.v_off = offv;
      d.bits_p = p->bits_p; d.mask = p->mask; d.flags = p->flags;
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
  // ---- output projection + residual, LN2 + layer-wise quant ------------------------------------------------------
  // (one kernel whose workgroups own whole rows where it exists, else the projection followed by the row kernel)
  const int off2 = rq_store_offset(ba, p->ln2_z);
  {
    rq_gemm_desc g;
    fill_linear(g, p->proj, o, T, D, p->s_o, p->z_o, offo, need_rowsum(p->proj) ? rowsum : nullptr);
    g.residual = x; g.ldr = D; g.out_f32 = xbar; g.ldf = D;
    rq_ln_desc d;
    std::memset(&d, 0, sizeof d);
    d.T = T; d.D = D; d.norm_kind = p->norm_kind; d.eps = p->eps; d.x = xbar; d.ldx = D;
    d.gamma_t = p->ln2_gamma_t; d.beta_t = p->ln2_beta_t; d.s_tilde = p->ln2_s; d.z_tilde = p->ln2_z; d.bits = ba;
    d.store_off = off2; d.q = a; d.ldq = D; d.rowsum = ln_rowsum(p->fc1) ? rowsum : nullptr;
    if (p->proj_ln_fused && rq_qgemm_rowln_applies(&g, &d)) {
      rq_prof_begin(ctx, RQ_STEP_PROJ);
      st = rq_qgemm_ln_quant(ctx, &g, &d);
      rq_prof_end(ctx);
      if (st != RQ_OK) return st;
    } else {
      rq_prof_begin(ctx, RQ_STEP_PROJ);
      st = rq_qgemm(ctx, &g);
      rq_prof_end(ctx);
      if (st != RQ_OK) return st;
      rq_prof_begin(ctx, RQ_STEP_LN2);
      st = rq_ln_quant(ctx, &d);
      rq_prof_end(ctx);
      if (st != RQ_OK) return st;
    }
  }
  // ---- FC1 + activation, re-quantized ------------------------------------------------------------------------------
  const int offh = rq_store_offset(ba, p->z_h);
  {
    rq_gemm_desc g;
    fill_linear(g, p->fc1, a, T, D, p->ln2_s, p->ln2_z, off2, ln_rowsum(p->fc1) ? rowsum : nullptr);
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
    fill_linear(g, p->fc2, hid, T, Dm, p->s_h, p->z_h, offh, need_rowsum(p->fc2) ? rowsum : nullptr);
    g.residual = xbar; g.ldr = D; g.out_f32 = y; g.ldf = D;
    rq_prof_begin(ctx, RQ_STEP_FC2);
    st = rq_qgemm(ctx, &g);
    rq_prof_end(ctx);
    if (st != RQ_OK) return st;
  }
  return RQ_OK;
  };
  // Two halves of the batch on two streams where neither half needs attention scratch (the one-kernel attention) and each is
  // a launch of its own right: the tail of one half's kernel -- the chip running empty while the last tiles finish -- is
  // filled by the other half's.  Same kernels on the same rows: the output bits do not depend on the split.
  const bool split = ctx->block_streams >= 2 && ctx->stream2 && !ctx->profiling && use_whole(p, seq) && batch >= 2 &&
                     (ctx->block_streams == 3 || pl.T * D >= (16ll << 20));
  if (!split) return run_part(0, batch);
  const int64_t b1 = (batch + 1) / 2;
  RQ_HIP(hipEventRecord(ctx->ev_fork, ctx->stream));
  RQ_HIP(hipStreamWaitEvent(ctx->stream2, ctx->ev_fork, 0));
  rq_status st1 = run_part(0, b1);
  hipStream_t main_stream = ctx->stream;
  ctx->stream = ctx->stream2;
  rq_status st2 = run_part(b1, batch - b1);
  ctx->stream = main_stream;
  RQ_HIP(hipEventRecord(ctx->ev_join, ctx->stream2));
  RQ_HIP(hipStreamWaitEvent(ctx->stream, ctx->ev_join, 0));
  return st1 != RQ_OK ? st1 : st2;
}

// ---- rq_block_forward_noalloc: the same pass with its scratch in a fixed device array of this library ----------------
}  // extern "C"

// Scratch of rq_block_forward_noalloc.  One copy of the array exists on every GPU the library is loaded on, at an address of
// its own; host code never uses the array's name as an address: the per-device address comes from hipGetSymbolAddress,
// taken once per device with that device current, and is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[RQ_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_DEVICES] = {nullptr};
}  // namespace

// Called by rq_create for a device context (and again, harmlessly, by the entry point): resolves this device's copy.
rq_status rq_noalloc_scratch_init(rq_ctx* ctx, void** out) {
  const int dev = ctx->device;
  if (dev < 0 || dev >= MAX_DEVICES) return rq_fail(ctx, RQ_ERR_UNSUPPORTED, "rq_block_forward_noalloc: device %d outside 0..%d", dev, MAX_DEVICES - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    int prev = -1;
    RQ_HIP(hipGetDevice(&prev));
    if (prev != dev) RQ_HIP(hipSetDevice(dev));
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (prev != dev) (void)hipSetDevice(prev);
    if (e != hipSuccess || !ptr)
      return rq_fail(ctx, RQ_ERR_HIP, "rq_block_forward_noalloc: hipGetSymbolAddress(scratch) on device %d failed: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  if (out) *out = g_scratch_ptr[dev];
  return RQ_OK;
}

extern "C" {

size_t rq_block_noalloc_scratch_bytes(void) { return (size_t)RQ_NOALLOC_SCRATCH_BYTES; }

rq_status rq_block_forward_noalloc(rq_ctx* ctx, const rq_block_params* p, const float* x, float* y, int64_t batch, int64_t seq) {
  if (!ctx) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_block_forward_noalloc: ctx is NULL");
  RQ_REQUIRE(p && x && y, RQ_ERR_INVALID_ARG, "rq_block_forward_noalloc: params, x, y must be non-NULL");
  RQ_REQUIRE(batch > 0 && seq > 0 && p->D > 0 && p->H > 0 && p->Dm > 0, RQ_ERR_SHAPE,
             "rq_block_forward_noalloc: batch = %lld, seq = %lld, D = %d, H = %d, Dm = %d", (long long)batch, (long long)seq, p->D, p->H,
             p->Dm);
  const size_t need = make_plan(p, batch, seq).total;
  RQ_REQUIRE(need <= (size_t)RQ_NOALLOC_SCRATCH_BYTES, RQ_ERR_WORKSPACE,
             "rq_block_forward_noalloc: this shape needs %zu bytes of scratch, the fixed array holds %zu; use rq_block_forward with a "
             "caller workspace", need, (size_t)RQ_NOALLOC_SCRATCH_BYTES);
  if (ctx->device < 0)      // host-only context: let the shared path finish the validation and refuse
    return rq_block_forward(ctx, p, x, y, batch, seq, reinterpret_cast<void*>(uintptr_t(256)), need);
  void* ptr = nullptr;
  const rq_status st = rq_noalloc_scratch_init(ctx, &ptr);
  if (st != RQ_OK) return st;
  // No region has to start at zero: every byte a kernel of the pass reads was written earlier in the same pass.
  return rq_block_forward(ctx, p, x, y, batch, seq, ptr, (size_t)RQ_NOALLOC_SCRATCH_BYTES);
}

}  // extern "C"

// ---- rq_block_calibrate ---------------------------------------------------------------------------------------
// Algorithm 1 restricted to one block and to min/max bounds: activation quantizer -> scale reparameterization ->
// weight quantization, layer by layer, each layer fed by the already-quantized layers before it.  Every tensor
// operation is one of the library's kernels; the host only turns min/max pairs into (s, z) scalars.
namespace {

struct CalPlan {
  Plan fwd;
  size_t o_cmin, o_cmax, o_sch, o_zch, o_wt, o_bt, o_f32, o_scal, o_clip, o_alpha, o_learn, o_gptq, gptq_bytes, total;
};

CalPlan make_cal_plan(const rq_block_raw* raw, int64_t batch, int64_t seq) {
  // The calibration walks attention with the three separate kernels (it needs the float P.V output of the first pass),
  // so its plan is the three-kernel one whatever the forward pass would choose: int32 logits and codes in regions of
  // their own, sized for one chunk.
  rq_block_params tmp;
  std::memset(&tmp, 0, sizeof tmp);
  tmp.D = raw->D; tmp.H = raw->H; tmp.Dm = raw->Dm;
  tmp.attn_path = RQ_ATTN_THREE_KERNELS;
  tmp.attn_chunk_bytes = raw->attn_chunk_bytes;
  CalPlan c;
  c.fwd = make_plan(&tmp, batch, seq);
  const int D = raw->D, Dm = raw->Dm;
  const int n1 = raw->act == RQ_ACT_SILU_GATED ? 2 * Dm : Dm;
  const int nmax = 3 * D > n1 ? 3 * D : n1;
  size_t o = c.fwd.total;
  c.o_cmin = o; o += up((size_t)D * 8);
  c.o_cmax = o; o += up((size_t)D * 8);
  c.o_sch = o; o += up((size_t)D * 4);
  c.o_zch = o; o += up((size_t)D * 4);
  c.o_wt = o; o += up((size_t)nmax * D * 4);
  c.o_bt = o; o += up((size_t)nmax * 4);
  c.o_f32 = o; o += up((size_t)c.fwd.T * nmax * 4);
  c.o_scal = o; o += up(256);
  c.o_clip = c.o_alpha = c.o_learn = c.o_gptq = o;
  c.gptq_bytes = 0;
  if (raw->learn_clip_iters > 0) {
    c.o_clip = o; o += up((size_t)2 * D * 4);
    c.o_alpha = o; o += up((size_t)2 * D * 8);
    c.o_learn = o; o += up(rq_dual_clip_workspace_bytes(c.fwd.T));
  }
  if (raw->gptq) {
    const size_t need[4] = {rq_gptq_workspace_bytes(3 * D, D, c.fwd.T), rq_gptq_workspace_bytes(D, D, c.fwd.T),
                            rq_gptq_workspace_bytes(n1, D, c.fwd.T), rq_gptq_workspace_bytes(D, Dm, c.fwd.T)};
    for (size_t v : need) c.gptq_bytes = v > c.gptq_bytes ? v : c.gptq_bytes;
    c.o_gptq = o; o += up(c.gptq_bytes);
  }
  c.total = o;
  return c;
}

void qparams_from_minmax(double lo, double hi, int bits, float* s, int32_t* z) {
  *s = (float)((hi - lo) / (double)((1 << bits) - 1));
  *z = (int32_t)std::nearbyint(-lo / (double)*s);
}

}  // namespace

extern "C" {

size_t rq_block_calibrate_workspace_bytes(const rq_block_raw* raw, int64_t batch, int64_t seq) {
  if (!raw || batch <= 0 || seq <= 0 || raw->D <= 0 || raw->H <= 0 || raw->Dm <= 0) return 0;
  return make_cal_plan(raw, batch, seq).total;
}

rq_status rq_block_calibrate_workspace_layout(const rq_block_raw* raw, int64_t batch, int64_t seq, rq_block_layout* out) {
  if (!raw || !out || batch <= 0 || seq <= 0 || raw->D <= 0 || raw->H <= 0 || raw->Dm <= 0)
    return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_block_calibrate_workspace_layout: NULL argument or non-positive size");
  const CalPlan cp = make_cal_plan(raw, batch, seq);
  export_layout(cp.fwd, out);
  out->total = cp.total;
  return RQ_OK;
}

rq_status rq_block_calibrate(rq_ctx* ctx, const rq_block_raw* raw, const float* x, int64_t batch, int64_t seq,
                             rq_block_params* out, void* workspace, size_t workspace_bytes) {
  if (!ctx) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_block_calibrate: ctx is NULL");
  RQ_REQUIRE(raw && x && out && workspace, RQ_ERR_INVALID_ARG, "rq_block_calibrate: raw, x, out, workspace must be non-NULL");
  RQ_REQUIRE(batch > 0 && seq > 0, RQ_ERR_SHAPE, "rq_block_calibrate: batch, seq must be > 0");
  RQ_REQUIRE(raw->D > 0 && raw->H > 0 && raw->Dm > 0 && raw->D % raw->H == 0, RQ_ERR_SHAPE, "rq_block_calibrate: D, H, Dm");
  RQ_REQUIRE(raw->bits_w == 4 || (raw->bits_w >= 2 && raw->bits_w <= 8), RQ_ERR_INVALID_ARG, "rq_block_calibrate: bits_w");
  RQ_REQUIRE(raw->ln1_gamma && raw->ln2_gamma && raw->w_qkv && raw->w_proj && raw->w_fc1 && raw->w_fc2, RQ_ERR_INVALID_ARG,
             "rq_block_calibrate: gammas and weights must be non-NULL");
  RQ_REQUIRE(raw->s_log > 0.f, RQ_ERR_INVALID_ARG, "rq_block_calibrate: s_log must be > 0");
  RQ_REQUIRE(raw->learn_clip_iters >= 0 && raw->learn_clip_iters <= 100000, RQ_ERR_INVALID_ARG,
             "rq_block_calibrate: learn_clip_iters = %d", raw->learn_clip_iters);
  RQ_REQUIRE(raw->attn_chunk_bytes == 0 || raw->attn_chunk_bytes >= (1 << 20), RQ_ERR_INVALID_ARG,
             "rq_block_calibrate: attn_chunk_bytes must be 0 (default) or at least 1 MiB");
  RQ_REQUIRE((raw->flags & ~RQ_LOG_ZERO_AT_MAX_CODE) == 0, RQ_ERR_INVALID_ARG, "rq_block_calibrate: flags = %d", raw->flags);
  if (raw->gptq)
    RQ_REQUIRE(raw->D % 64 == 0 && raw->Dm % 64 == 0 && raw->D <= 8192 && raw->Dm <= 8192 && batch * seq <= 131071,
               RQ_ERR_UNSUPPORTED, "rq_block_calibrate: GPTQ needs D and Dm multiples of 64, at most 8192, and at most 131071 tokens");
  RQ_REQUIRE(out->ln1_gamma_t && out->ln1_beta_t && out->ln2_gamma_t && out->ln2_beta_t, RQ_ERR_INVALID_ARG,
             "rq_block_calibrate: out->ln*_gamma_t / beta_t must point to caller-allocated [D] arrays");
  const rq_qlinear* lins[4] = {&out->qkv, &out->proj, &out->fc1, &out->fc2};
  for (const rq_qlinear* l : lins)
    RQ_REQUIRE(l->w && l->s_w && l->z_w && l->colsum_w && l->bias, RQ_ERR_INVALID_ARG,
               "rq_block_calibrate: every rq_qlinear of out needs w, s_w, z_w, colsum_w, bias allocated by the caller");
  RQ_REQUIRE(rq_aligned(workspace, ALIGN), RQ_ERR_INVALID_ARG, "rq_block_calibrate: workspace needs 256-byte alignment");
  const CalPlan cp = make_cal_plan(raw, batch, seq);
  RQ_REQUIRE(workspace_bytes >= cp.total, RQ_ERR_WORKSPACE, "rq_block_calibrate: workspace has %zu bytes, %zu needed",
             workspace_bytes, cp.total);
  RQ_NEED_DEVICE();

  const int D = raw->D, H = raw->H, Dm = raw->Dm, dh = D / H;
  const bool gated = raw->act == RQ_ACT_SILU_GATED;
  const int n1 = gated ? 2 * Dm : Dm;
  const int ba = raw->bits_a, bw = raw->bits_w;
  const int wfmt = bw == 4 ? RQ_W_U4 : (bw == 8 ? RQ_W_I8_CENTERED : RQ_W_I8_BAKED);
  const int64_t T = batch * seq;
  char* ws = static_cast<char*>(workspace);
  double* cmin = reinterpret_cast<double*>(ws + cp.o_cmin);
  double* cmax = reinterpret_cast<double*>(ws + cp.o_cmax);
  float* s_ch = reinterpret_cast<float*>(ws + cp.o_sch);
  int32_t* z_ch = reinterpret_cast<int32_t*>(ws + cp.o_zch);
  float* wt = reinterpret_cast<float*>(ws + cp.o_wt);
  float* bt = reinterpret_cast<float*>(ws + cp.o_bt);
  float* f32 = reinterpret_cast<float*>(ws + cp.o_f32);
  char* scal = ws + cp.o_scal;   // device scalars: s_tilde (float), z_tilde (int32), min/max (2 doubles at +16)
  const Plan& pl = cp.fwd;
  int8_t* a = reinterpret_cast<int8_t*>(ws + pl.o_a);
  int32_t* rowsum = reinterpret_cast<int32_t*>(ws + pl.o_rowsum);
  int8_t* qkv = reinterpret_cast<int8_t*>(ws + pl.o_qkv);
  int32_t* acc = reinterpret_cast<int32_t*>(ws + pl.o_acc);
  uint8_t* codes = reinterpret_cast<uint8_t*>(ws + pl.o_codes);
  int8_t* o = reinterpret_cast<int8_t*>(ws + pl.o_o);
  float* xbar = reinterpret_cast<float*>(ws + pl.o_xbar);
  rq_status st;

  out->D = D; out->H = H; out->Dm = Dm; out->norm_kind = raw->norm_kind; out->act = raw->act; out->mask = raw->mask;
  out->bits_a = ba; out->bits_p = raw->bits_p; out->eps = raw->eps; out->rel_bias = raw->rel_bias; out->s_log = raw->s_log;
  out->flags = raw->flags;

  auto minmax_host = [&](const float* v, int64_t rows, int64_t cols, int64_t ld, double* lo, double* hi) -> rq_status {
    double* d2 = reinterpret_cast<double*>(scal + 16);
    rq_status s2 = rq_minmax_f32(ctx, v, rows, cols, ld, d2);
    if (s2 != RQ_OK) return s2;
    double h2[2];
    RQ_HIP(hipMemcpyAsync(h2, d2, 16, hipMemcpyDeviceToHost, ctx->stream));
    RQ_HIP(hipStreamSynchronize(ctx->stream));
    *lo = h2[0]; *hi = h2[1];
    return RQ_OK;
  };
  // weight quantization of one Linear; `A` = the codes it is fed (stored form) for GPTQ
  auto quant_linear = [&](rq_qlinear* l, const float* W, const float* b, int N, int K, int gate_rows, const int8_t* A, int a_off,
                          int z_a) -> rq_status {
    l->N = N; l->K = K; l->bits = bw; l->format = wfmt;
    if (raw->gptq) {
      rq_gptq_desc d;
      std::memset(&d, 0, sizeof d);
      d.N = N; d.K = K; d.bits = bw; d.format = wfmt; d.gate_up_rows = gate_rows; d.W = W; d.bias = b;
      d.A = A; d.T = T; d.lda = K; d.a_off = a_off; d.z_a = z_a; d.percdamp = raw->gptq_percdamp > 0.0 ? raw->gptq_percdamp : 0.01;
      d.w_out = const_cast<void*>(l->w); d.s_w = const_cast<float*>(l->s_w); d.z_w = const_cast<int32_t*>(l->z_w);
      d.colsum_w = const_cast<int32_t*>(l->colsum_w); d.bias_out = const_cast<float*>(l->bias);
      d.workspace = ws + cp.o_gptq; d.workspace_bytes = cp.gptq_bytes;
      return rq_gptq_quant_pack(ctx, &d);
    }
    rq_wq_desc d;
    std::memset(&d, 0, sizeof d);
    d.N = N; d.K = K; d.bits = bw; d.format = wfmt; d.gate_up_rows = gate_rows; d.W = W; d.bias = b;
    d.w_out = const_cast<void*>(l->w); d.s_w = const_cast<float*>(l->s_w); d.z_w = const_cast<int32_t*>(l->z_w);
    d.colsum_w = const_cast<int32_t*>(l->colsum_w); d.bias_out = const_cast<float*>(l->bias);
    return rq_weight_quant_pack(ctx, &d);
  };
  // LayerNorm activation: channel-wise (s, z) -> fold into the affine and the next Linear (left in wt / bt)
  auto fold_ln = [&](const float* xin, const float* gamma, const float* beta, const float* cu, const float* cl, const float* W,
                     const float* b, int N, float* gamma_t, float* beta_t, float* s_out, int32_t* z_out) -> rq_status {
    rq_status s2 = rq_ln_channel_minmax(ctx, xin, T, D, D, raw->norm_kind, raw->eps, gamma, beta, cmin, cmax);
    if (s2 != RQ_OK) return s2;
    if (raw->learn_clip_iters > 0) {                       // Algorithm 1: learn the clip factors on this layer's X'
      float* clip = reinterpret_cast<float*>(ws + cp.o_clip);
      double* alpha = reinterpret_cast<double*>(ws + cp.o_alpha);
      rq_dual_clip_desc dc;
      std::memset(&dc, 0, sizeof dc);
      dc.T = T; dc.D = D; dc.ldx = D; dc.x = xin; dc.norm_kind = raw->norm_kind; dc.eps = raw->eps; dc.gamma = gamma; dc.beta = beta;
      dc.bits = ba; dc.iters = raw->learn_clip_iters; dc.lr = raw->learn_clip_lr; dc.alpha0 = raw->learn_clip_alpha0;
      dc.alpha1 = alpha; dc.alpha2 = alpha + D; dc.clip_up = clip; dc.clip_lo = clip + D;
      dc.workspace = ws + cp.o_learn; dc.workspace_bytes = rq_dual_clip_workspace_bytes(T);
      if ((s2 = rq_dual_clip_learn(ctx, &dc)) != RQ_OK) return s2;
      cu = clip; cl = clip + D;
    }
    if ((s2 = rq_launch_channel_qparams(ctx, cmin, cmax, cu, cl, D, ba, s_ch, z_ch)) != RQ_OK) return s2;
    rq_fold_desc f;
    std::memset(&f, 0, sizeof f);
    f.D = D; f.D_out = N; f.s_ch = s_ch; f.z_ch = z_ch; f.gamma = gamma; f.beta = beta; f.W = W; f.b = b;
    f.s_tilde = reinterpret_cast<float*>(scal); f.z_tilde = reinterpret_cast<int32_t*>(scal + 4);
    f.gamma_t = gamma_t; f.beta_t = beta_t; f.W_t = wt; f.b_t = bt;
    if ((s2 = rq_reparam_fold(ctx, &f)) != RQ_OK) return s2;
    char h8[8];
    RQ_HIP(hipMemcpyAsync(h8, scal, 8, hipMemcpyDeviceToHost, ctx->stream));
    RQ_HIP(hipStreamSynchronize(ctx->stream));
    std::memcpy(s_out, h8, 4);
    std::memcpy(z_out, h8 + 4, 4);
    return RQ_OK;
  };
  auto ln_q = [&](const float* xin, const float* gt, const float* btl, float s, int z) -> rq_status {
    rq_ln_desc d;
    std::memset(&d, 0, sizeof d);
    d.T = T; d.D = D; d.norm_kind = raw->norm_kind; d.eps = raw->eps; d.x = xin; d.ldx = D; d.gamma_t = gt; d.beta_t = btl;
    d.s_tilde = s; d.z_tilde = z; d.bits = ba; d.store_off = rq_store_offset(ba, z); d.q = a; d.ldq = D;
    d.rowsum = wfmt == RQ_W_I8_CENTERED ? rowsum : nullptr;
    return rq_ln_quant(ctx, &d);
  };

  // ---- LN1 -> QKV ----
  if ((st = fold_ln(x, raw->ln1_gamma, raw->ln1_beta, raw->ln1_clip_up, raw->ln1_clip_lo, raw->w_qkv, raw->b_qkv, 3 * D,
                    const_cast<float*>(out->ln1_gamma_t), const_cast<float*>(out->ln1_beta_t), &out->ln1_s, &out->ln1_z)) != RQ_OK)
    return st;
  if ((st = ln_q(x, out->ln1_gamma_t, out->ln1_beta_t, out->ln1_s, out->ln1_z)) != RQ_OK) return st;
  const int off1 = rq_store_offset(ba, out->ln1_z);
  if ((st = quant_linear(&out->qkv, wt, bt, 3 * D, D, 0, a, off1, out->ln1_z)) != RQ_OK) return st;
  rq_gemm_desc g;
  const int32_t* const rs_c = wfmt == RQ_W_I8_CENTERED ? rowsum : nullptr;      // the calibration computes row sums only where required
  fill_linear(g, out->qkv, a, T, D, out->ln1_s, out->ln1_z, off1, rs_c);
  g.out_f32 = f32; g.ldf = 3 * D;
  if ((st = rq_qgemm(ctx, &g)) != RQ_OK) return st;
  float* s3[3] = {&out->s_q, &out->s_k, &out->s_v};
  int32_t* z3[3] = {&out->z_q, &out->z_k, &out->z_v};
  for (int i = 0; i < 3; ++i) {
    double lo, hi;
    if ((st = minmax_host(f32 + (int64_t)i * D, T, D, 3 * D, &lo, &hi)) != RQ_OK) return st;
    qparams_from_minmax(lo, hi, ba, s3[i], z3[i]);
  }
  const int offq = rq_store_offset(ba, out->z_q), offk = rq_store_offset(ba, out->z_k), offv = rq_store_offset(ba, out->z_v);
  g.out_f32 = nullptr; g.out_q = qkv; g.ldq = 3 * D; g.bits_o = ba; g.n_seg = 3; g.seg_len = D;
  g.s_o[0] = out->s_q; g.s_o[1] = out->s_k; g.s_o[2] = out->s_v;
  g.z_o[0] = out->z_q; g.z_o[1] = out->z_k; g.z_o[2] = out->z_v;
  g.off_o[0] = offq; g.off_o[1] = offk; g.off_o[2] = offv;
  if ((st = rq_qgemm(ctx, &g)) != RQ_OK) return st;

  // ---- attention: first pass float output for the static scale of its activation, second pass quantized ----
  int offo = 0;
  for (int pass = 0; pass < 2; ++pass) {
    for (int64_t b0 = 0; b0 < batch; b0 += pl.bchunk) {
      const int64_t nb = (batch - b0) < pl.bchunk ? (batch - b0) : pl.bchunk;
      const int8_t* qkv_c = qkv + b0 * seq * 3 * D;
      rq_gemm_desc q;
      std::memset(&q, 0, sizeof q);
      q.M = seq; q.N = (int)seq; q.K = dh; q.A = qkv_c; q.lda = 3 * D; q.a_off = offq; q.z_a = out->z_q; q.s_a = out->s_q;
      q.B = qkv_c + D; q.ldb = 3 * D; q.b_format = RQ_B_ACT_I8; q.b_off = offk; q.z_b_scalar = out->z_k;
      q.out_acc = acc; q.ldacc = pl.ld; q.acc_stride_group = seq * pl.ld; q.batch_outer = nb; q.batch_inner = H;
      q.a_stride_outer = seq * 3 * D; q.a_stride_inner = dh; q.b_stride_outer = seq * 3 * D; q.b_stride_inner = dh;
      q.causal = raw->mask == RQ_MASK_CAUSAL;
      if ((st = rq_qgemm(ctx, &q)) != RQ_OK) return st;
      rq_softmax_desc sd;
      std::memset(&sd, 0, sizeof sd);
      sd.G = nb * H; sd.H = H; sd.Nq = (int)seq; sd.Nk = (int)seq; sd.ld = pl.ld; sd.acc = acc;
      sd.logit_scale = (double)out->s_q * (double)out->s_k / std::sqrt((double)dh);
      sd.bias = raw->rel_bias; sd.mask = raw->mask; sd.s_log = raw->s_log; sd.bits = raw->bits_p; sd.codes = codes;
      if ((st = rq_softmax_log2_quant(ctx, &sd)) != RQ_OK) return st;
      rq_pv_desc pd;
      std::memset(&pd, 0, sizeof pd);
      pd.batch = nb; pd.H = H; pd.Nq = (int)seq; pd.Nk = (int)seq; pd.d_head = dh; pd.ld = pl.ld; pd.codes = codes;
      pd.V = qkv_c + 2 * D; pd.ldv = 3 * D; pd.s_log = raw->s_log; pd.s_v = out->s_v; pd.z_v = out->z_v; pd.v_off = offv;
      pd.bits_p = raw->bits_p; pd.mask = raw->mask; pd.flags = raw->flags;
      if (pass == 0) {
        pd.out_f32 = f32 + b0 * seq * D; pd.ldf = D;
      } else {
        pd.out_q = o + b0 * seq * D; pd.ldq = D; pd.s_o = out->s_o; pd.z_o = out->z_o; pd.off_o = offo; pd.bits_o = ba;
      }
      if ((st = rq_attn_pv(ctx, &pd)) != RQ_OK) return st;
    }
    if (pass == 0) {
      double lo, hi;
      if ((st = minmax_host(f32, T, D, D, &lo, &hi)) != RQ_OK) return st;
      qparams_from_minmax(lo, hi, ba, &out->s_o, &out->z_o);
      offo = rq_store_offset(ba, out->z_o);
    }
  }
  // ---- proj (plain channel-wise weight quantization), residual ----
  if ((st = quant_linear(&out->proj, raw->w_proj, raw->b_proj, D, D, 0, o, offo, out->z_o)) != RQ_OK) return st;
  if (out->proj.format == RQ_W_I8_CENTERED && (st = rq_rowsum_i8(ctx, o, T, D, D, rowsum)) != RQ_OK) return st;
  fill_linear(g, out->proj, o, T, D, out->s_o, out->z_o, offo, rs_c);
  g.residual = x; g.ldr = D; g.out_f32 = xbar; g.ldf = D;
  if ((st = rq_qgemm(ctx, &g)) != RQ_OK) return st;
  // ---- LN2 -> FC1 ----
  if ((st = fold_ln(xbar, raw->ln2_gamma, raw->ln2_beta, raw->ln2_clip_up, raw->ln2_clip_lo, raw->w_fc1, raw->b_fc1, n1,
                    const_cast<float*>(out->ln2_gamma_t), const_cast<float*>(out->ln2_beta_t), &out->ln2_s, &out->ln2_z)) != RQ_OK)
    return st;
  if ((st = ln_q(xbar, out->ln2_gamma_t, out->ln2_beta_t, out->ln2_s, out->ln2_z)) != RQ_OK) return st;
  const int off2 = rq_store_offset(ba, out->ln2_z);
  if ((st = quant_linear(&out->fc1, wt, bt, n1, D, gated ? Dm : 0, a, off2, out->ln2_z)) != RQ_OK) return st;
  fill_linear(g, out->fc1, a, T, D, out->ln2_s, out->ln2_z, off2, rs_c);
  g.act = raw->act; g.out_f32 = f32; g.ldf = Dm;
  if ((st = rq_qgemm(ctx, &g)) != RQ_OK) return st;
  {
    double lo, hi;
    if ((st = minmax_host(f32, T, Dm, Dm, &lo, &hi)) != RQ_OK) return st;
    qparams_from_minmax(lo, hi, ba, &out->s_h, &out->z_h);
  }
  // ---- FC2 (GPTQ wants the codes it is fed: FC1 once more, now quantized) ----
  int8_t* hid = reinterpret_cast<int8_t*>(ws + pl.o_hid);
  const int offh = rq_store_offset(ba, out->z_h);
  if (raw->gptq) {
    g.out_f32 = nullptr; g.out_q = hid; g.ldq = Dm; g.bits_o = ba; g.n_seg = 1; g.seg_len = Dm;
    g.s_o[0] = out->s_h; g.z_o[0] = out->z_h; g.off_o[0] = offh;
    if ((st = rq_qgemm(ctx, &g)) != RQ_OK) return st;
  }
  return quant_linear(&out->fc2, raw->w_fc2, raw->b_fc2, D, Dm, 0, hid, offh, out->z_h);
}

}  // extern "C"
