// C-ABI entry points: context, argument validation, dispatch to the kernel launchers.
// Validation happens before any HIP call so it can be exercised on a host without a GPU.
#include <stdarg.h>

#include <cmath>
#include <vector>

#include "rq_internal.h"

static thread_local std::string g_last_error;

rq_status rq_fail(rq_ctx* ctx, rq_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = buf;
  g_last_error = buf;
  return st;
}

extern "C" {

rq_status rq_create(rq_ctx** out, int device, void* hip_stream) {
  rq_ctx* ctx = nullptr;
  if (!out) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_create: ctx is NULL");
  *out = nullptr;
  rq_ctx* c = new rq_ctx();
  c->device = device;
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  if (device >= 0) {
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) {
      delete c;
      return rq_fail(ctx, RQ_ERR_HIP, "rq_create: hipGetDeviceProperties(%d) failed: %s", device, hipGetErrorString(e));
    }
    c->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    std::string arch = prop.gcnArchName;
    if (arch.rfind("gfx950", 0) != 0) {
      delete c;
      return rq_fail(ctx, RQ_ERR_UNSUPPORTED, "rq_create: device %d is %s; this library is built for gfx950 only", device,
                     arch.c_str());
    }
  }
  c->pending = new std::vector<rq_ctx::EvPair>();
  c->pool = new std::vector<hipEvent_t>();
  if (device >= 0) {      // set-up work that must not happen inside rq_block_forward_noalloc's callers' hot loops
    if (hipStreamCreateWithFlags(&c->stream2, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      if (c->stream2) (void)hipStreamDestroy(c->stream2);
      c->stream2 = nullptr;      // rq_block_forward then stays on one stream
    }
    c->block_streams = c->stream2 ? 2 : 1;
    const rq_status st = rq_noalloc_scratch_init(c, nullptr);
    if (st != RQ_OK) {
      g_last_error = c->err;
      rq_destroy(c);
      return st;
    }
  }
  *out = c;
  return RQ_OK;
}

void rq_destroy(rq_ctx* ctx) {
  if (!ctx) return;
  if (ctx->pending) {
    for (auto& p : *ctx->pending) { hipEventDestroy(p.a); hipEventDestroy(p.b); }
    delete ctx->pending;
  }
  if (ctx->pool) {
    for (auto e : *ctx->pool) hipEventDestroy(e);
    delete ctx->pool;
  }
  if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
  if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
  if (ctx->stream2) (void)hipStreamDestroy(ctx->stream2);
  delete ctx;
}

rq_status rq_set_block_streams(rq_ctx* ctx, int32_t streams) {
  if (!ctx) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_set_block_streams: ctx is NULL");
  RQ_REQUIRE(streams >= 1 && streams <= 3, RQ_ERR_INVALID_ARG, "rq_set_block_streams: %d not in 1..3", streams);
  ctx->block_streams = (streams > 1 && !ctx->stream2 && ctx->device >= 0) ? 1 : streams;
  return RQ_OK;
}

const char* rq_last_error(const rq_ctx* ctx) { return ctx ? ctx->err.c_str() : g_last_error.c_str(); }

int32_t rq_store_offset(int32_t bits, int32_t z) {
  const int qmax = (1 << bits) - 1;
  if (-z >= -128 && qmax - z <= 127) return z;
  return 128;
}

}  // extern "C"

// ---- profiling ------------------------------------------------------------------------------------------
static hipEvent_t prof_event(rq_ctx* ctx) {
  if (!ctx->pool->empty()) {
    hipEvent_t e = ctx->pool->back();
    ctx->pool->pop_back();
    return e;
  }
  hipEvent_t e;
  hipEventCreate(&e);
  return e;
}

void rq_prof_begin(rq_ctx* ctx, int step) {
  if (!ctx->profiling) return;
  rq_ctx::EvPair p{prof_event(ctx), prof_event(ctx), step};
  hipEventRecord(p.a, ctx->stream);
  ctx->pending->push_back(p);
}

void rq_prof_end(rq_ctx* ctx) {
  if (!ctx->profiling) return;
  hipEventRecord(ctx->pending->back().b, ctx->stream);
}

static void prof_drain(rq_ctx* ctx) {
  if (ctx->device < 0) return;
  hipStreamSynchronize(ctx->stream);
  for (auto& p : *ctx->pending) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
      ctx->prof_ms[p.step] += ms;
      ctx->prof_n[p.step] += 1;
    }
    ctx->pool->push_back(p.a);
    ctx->pool->push_back(p.b);
  }
  ctx->pending->clear();
}

extern "C" {

rq_status rq_profile_enable(rq_ctx* ctx, int32_t on) {
  RQ_REQUIRE(ctx, RQ_ERR_INVALID_ARG, "rq_profile_enable: ctx is NULL");
  prof_drain(ctx);
  ctx->profiling = on != 0;
  return RQ_OK;
}

rq_status rq_profile_reset(rq_ctx* ctx) {
  RQ_REQUIRE(ctx, RQ_ERR_INVALID_ARG, "rq_profile_reset: ctx is NULL");
  prof_drain(ctx);
  for (int i = 0; i < RQ_STEP_COUNT; ++i) { ctx->prof_ms[i] = 0; ctx->prof_n[i] = 0; }
  return RQ_OK;
}

int32_t rq_profile_read(rq_ctx* ctx, double* ms_total, int64_t* launches) {
  if (!ctx || !ms_total || !launches) return -1;
  prof_drain(ctx);
  for (int i = 0; i < RQ_STEP_COUNT; ++i) { ms_total[i] = ctx->prof_ms[i]; launches[i] = ctx->prof_n[i]; }
  return RQ_STEP_COUNT;
}

// ---- validation helpers -----------------------------------------------------------------------------------
#define RQ_CHECK_CTX(name)                                                                   \
  do {                                                                                       \
    if (!ctx) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, name ": ctx is NULL");             \
    if (!d) return rq_fail(ctx, RQ_ERR_INVALID_ARG, name ": descriptor is NULL");            \
  } while (0)

static rq_status check_qgemm_weight(rq_ctx* ctx, const rq_gemm_desc* d);

static bool fits_i8(int bits, int off) { return -off >= -128 && ((1 << bits) - 1 - off) <= 127; }

static rq_status check_ln(rq_ctx* ctx, const rq_ln_desc* d, bool need_x) {
  RQ_REQUIRE((d->x || !need_x) && d->gamma_t && d->q, RQ_ERR_INVALID_ARG, "rq_ln_quant: x, gamma_t and q must be non-NULL");
  RQ_REQUIRE(d->norm_kind == RQ_NORM_LAYERNORM || d->norm_kind == RQ_NORM_RMSNORM, RQ_ERR_INVALID_ARG,
             "rq_ln_quant: norm_kind %d", d->norm_kind);
  RQ_REQUIRE(d->bits >= 2 && d->bits <= 8, RQ_ERR_INVALID_ARG, "rq_ln_quant: bits = %d not in 2..8", d->bits);
  RQ_REQUIRE(d->s_tilde > 0.f && std::isfinite(d->s_tilde), RQ_ERR_INVALID_ARG, "rq_ln_quant: s_tilde must be > 0");
  RQ_REQUIRE(d->eps >= 0.0, RQ_ERR_INVALID_ARG, "rq_ln_quant: eps < 0");
  RQ_REQUIRE(fits_i8(d->bits, d->store_off), RQ_ERR_INVALID_ARG,
             "rq_ln_quant: codes of %d bits minus store_off %d do not fit int8", d->bits, d->store_off);
  RQ_REQUIRE(d->T >= 0 && d->D > 0, RQ_ERR_SHAPE, "rq_ln_quant: T = %lld, D = %d", (long long)d->T, d->D);
  RQ_REQUIRE(d->D % 4 == 0 && d->D <= 8192, RQ_ERR_SHAPE, "rq_ln_quant: D = %d must be a multiple of 4, at most 8192", d->D);
  RQ_REQUIRE(d->ldx >= d->D && d->ldx % 4 == 0 && d->ldq >= d->D && d->ldq % 4 == 0, RQ_ERR_SHAPE,
             "rq_ln_quant: ldx/ldq must be >= D and multiples of 4");
  RQ_REQUIRE(rq_aligned(d->x, 16) && rq_aligned(d->q, 4), RQ_ERR_INVALID_ARG, "rq_ln_quant: x needs 16-byte, q 4-byte alignment");
  return RQ_OK;
}

rq_status rq_ln_quant(rq_ctx* ctx, const rq_ln_desc* d) {
  RQ_CHECK_CTX("rq_ln_quant");
  const rq_status st = check_ln(ctx, d, true);
  if (st != RQ_OK) return st;
  RQ_NEED_DEVICE();
  if (d->T == 0) return RQ_OK;
  return rq_launch_ln_quant(ctx, d);
}


rq_status rq_reparam_fold(rq_ctx* ctx, const rq_fold_desc* d) {
  RQ_CHECK_CTX("rq_reparam_fold");
  RQ_REQUIRE(d->D > 0 && d->D_out >= 0, RQ_ERR_SHAPE, "rq_reparam_fold: D = %d, D_out = %d", d->D, d->D_out);
  RQ_REQUIRE(d->s_ch && d->z_ch && d->gamma, RQ_ERR_INVALID_ARG, "rq_reparam_fold: s_ch, z_ch, gamma must be non-NULL");
  RQ_REQUIRE(d->s_tilde && d->z_tilde && d->gamma_t && d->beta_t, RQ_ERR_INVALID_ARG,
             "rq_reparam_fold: s_tilde, z_tilde, gamma_t, beta_t must be non-NULL");
  RQ_REQUIRE(d->D_out == 0 || (d->W && d->W_t && d->b_t), RQ_ERR_INVALID_ARG, "rq_reparam_fold: W, W_t, b_t must be non-NULL");
  RQ_REQUIRE(!d->s_log_pair || (d->s_log > 0.f && std::isfinite(d->s_log)), RQ_ERR_INVALID_ARG,
             "rq_reparam_fold: s_log must be > 0");
  RQ_NEED_DEVICE();
  return rq_launch_fold(ctx, d);
}

rq_status rq_weight_quant_pack(rq_ctx* ctx, const rq_wq_desc* d) {
  RQ_CHECK_CTX("rq_weight_quant_pack");
  RQ_REQUIRE(d->W && d->w_out && d->s_w && d->z_w && d->colsum_w, RQ_ERR_INVALID_ARG,
             "rq_weight_quant_pack: W, w_out, s_w, z_w, colsum_w must be non-NULL");
  RQ_REQUIRE(d->N > 0 && d->K > 0, RQ_ERR_SHAPE, "rq_weight_quant_pack: N = %d, K = %d", d->N, d->K);
  switch (d->format) {
    case RQ_W_U4:
      RQ_REQUIRE(d->bits == 4, RQ_ERR_INVALID_ARG, "rq_weight_quant_pack: RQ_W_U4 needs bits = 4, got %d", d->bits);
      RQ_REQUIRE(d->K % 8 == 0, RQ_ERR_SHAPE, "rq_weight_quant_pack: RQ_W_U4 needs K %% 8 == 0, got %d", d->K);
      break;
    case RQ_W_I8_CENTERED:
      RQ_REQUIRE(d->bits >= 2 && d->bits <= 8, RQ_ERR_INVALID_ARG, "rq_weight_quant_pack: bits = %d not in 2..8", d->bits);
      break;
    case RQ_W_I8_BAKED:
      RQ_REQUIRE(d->bits >= 2 && d->bits <= 7, RQ_ERR_INVALID_ARG,
                 "rq_weight_quant_pack: RQ_W_I8_BAKED needs bits in 2..7, got %d", d->bits);
      break;
    default:
      return rq_fail(ctx, RQ_ERR_INVALID_ARG, "rq_weight_quant_pack: format %d", d->format);
  }
  if (d->gate_up_rows != 0)
    RQ_REQUIRE(d->gate_up_rows > 0 && d->N == 2 * d->gate_up_rows && d->gate_up_rows % 32 == 0, RQ_ERR_SHAPE,
               "rq_weight_quant_pack: gate_up_rows = %d needs N = 2*gate_up_rows and a multiple of 32", d->gate_up_rows);
  RQ_REQUIRE(d->w_out != (const void*)d->W, RQ_ERR_INVALID_ARG, "rq_weight_quant_pack: w_out must not alias W");
  RQ_NEED_DEVICE();
  return rq_launch_weight_quant(ctx, d);
}

rq_status rq_qgemm(rq_ctx* ctx, const rq_gemm_desc* d) {
  RQ_CHECK_CTX("rq_qgemm");
  RQ_REQUIRE(d->A && d->B, RQ_ERR_INVALID_ARG, "rq_qgemm: A and B must be non-NULL");
  RQ_REQUIRE(d->M >= 0 && d->N > 0 && d->K > 0, RQ_ERR_SHAPE, "rq_qgemm: M = %lld, N = %d, K = %d", (long long)d->M, d->N, d->K);
  RQ_REQUIRE(rq_aligned(d->A, 16) && rq_aligned(d->B, 16), RQ_ERR_INVALID_ARG, "rq_qgemm: A and B need 16-byte alignment");
  RQ_REQUIRE(d->lda >= d->K && d->lda % 16 == 0, RQ_ERR_SHAPE, "rq_qgemm: lda = %lld must be >= K and a multiple of 16",
             (long long)d->lda);
  if (d->b_format == RQ_B_ACT_I8) {
    RQ_REQUIRE(d->K == 32 || d->K == 64 || d->K == 128 || d->K == 256, RQ_ERR_SHAPE,
               "rq_qgemm (activation mode): K = %d must be 32, 64, 128 or 256", d->K);
    RQ_REQUIRE(d->ldb >= d->K && d->ldb % 16 == 0, RQ_ERR_SHAPE, "rq_qgemm: ldb must be >= K and a multiple of 16");
    RQ_REQUIRE(d->out_acc && !d->out_f32 && !d->out_q, RQ_ERR_INVALID_ARG,
               "rq_qgemm (activation mode): out_acc is the only output");
    RQ_REQUIRE(rq_aligned(d->out_acc, 16) && d->ldacc >= d->N && d->ldacc % 4 == 0 && d->acc_stride_group % 4 == 0, RQ_ERR_SHAPE,
               "rq_qgemm (activation mode): out_acc needs 16-byte alignment, ldacc >= N, ldacc and group stride multiples of 4");
    RQ_REQUIRE(d->batch_outer >= 1 && d->batch_inner >= 1, RQ_ERR_SHAPE, "rq_qgemm: batch counts must be >= 1");
    RQ_REQUIRE(d->a_stride_outer % 16 == 0 && d->a_stride_inner % 16 == 0 && d->b_stride_outer % 16 == 0 &&
                   d->b_stride_inner % 16 == 0, RQ_ERR_SHAPE, "rq_qgemm: batch strides must be multiples of 16");
    RQ_REQUIRE(d->M < (1ll << 31), RQ_ERR_SHAPE, "rq_qgemm (activation mode): M too large");
    RQ_REQUIRE(!d->causal || d->M == d->N, RQ_ERR_SHAPE, "rq_qgemm: causal needs M == N");
    RQ_NEED_DEVICE();
    if (d->M == 0) return RQ_OK;
    return rq_launch_qgemm_act(ctx, d);
  }
  const rq_status st = check_qgemm_weight(ctx, d);
  if (st != RQ_OK) return st;
  RQ_NEED_DEVICE();
  if (d->M == 0) return RQ_OK;
  return rq_launch_qgemm_weight(ctx, d);
}

static rq_status check_qgemm_weight(rq_ctx* ctx, const rq_gemm_desc* d) {
  RQ_REQUIRE(d->b_format == RQ_W_I8_BAKED || d->b_format == RQ_W_I8_CENTERED || d->b_format == RQ_W_U4, RQ_ERR_INVALID_ARG,
             "rq_qgemm: b_format %d", d->b_format);
  RQ_REQUIRE(d->K % 64 == 0, RQ_ERR_SHAPE, "rq_qgemm: K = %d must be a multiple of 64", d->K);
  RQ_REQUIRE(d->N % 4 == 0, RQ_ERR_SHAPE, "rq_qgemm: N = %d must be a multiple of 4", d->N);
  const int64_t ldb_min = d->b_format == RQ_W_U4 ? d->K / 2 : d->K;
  RQ_REQUIRE(d->ldb >= ldb_min && d->ldb % 16 == 0, RQ_ERR_SHAPE, "rq_qgemm: ldb = %lld must be >= %lld and a multiple of 16",
             (long long)d->ldb, (long long)ldb_min);
  RQ_REQUIRE(d->s_b, RQ_ERR_INVALID_ARG, "rq_qgemm: s_b must be non-NULL");
  RQ_REQUIRE(d->s_a > 0.f && std::isfinite(d->s_a), RQ_ERR_INVALID_ARG, "rq_qgemm: s_a must be > 0");
  RQ_REQUIRE(d->b_format == RQ_W_I8_BAKED || d->z_b, RQ_ERR_INVALID_ARG, "rq_qgemm: z_b is required for this weight format");
  RQ_REQUIRE(d->b_format != RQ_W_I8_CENTERED || d->rowsum_a, RQ_ERR_INVALID_ARG,
             "rq_qgemm: rowsum_a is required for RQ_W_I8_CENTERED");
  RQ_REQUIRE(d->a_off == d->z_a || d->colsum_b, RQ_ERR_INVALID_ARG, "rq_qgemm: colsum_b is required when a_off != z_a");
  RQ_REQUIRE(d->act == RQ_ACT_NONE || d->act == RQ_ACT_GELU || d->act == RQ_ACT_SILU_GATED, RQ_ERR_INVALID_ARG,
             "rq_qgemm: act %d", d->act);
  RQ_REQUIRE(d->out_acc || d->out_f32 || d->out_q, RQ_ERR_INVALID_ARG, "rq_qgemm: no output requested");
  const bool gated = d->act == RQ_ACT_SILU_GATED;
  if (gated) {
    RQ_REQUIRE(d->N % 64 == 0, RQ_ERR_SHAPE, "rq_qgemm: gated activation needs N %% 64 == 0");
    RQ_REQUIRE(!d->out_acc, RQ_ERR_INVALID_ARG, "rq_qgemm: out_acc is not available with the gated activation");
  }
  const int n_out = gated ? d->N / 2 : d->N;
  RQ_REQUIRE(!d->out_acc || (rq_aligned(d->out_acc, 16) && d->ldacc >= d->N && d->ldacc % 4 == 0), RQ_ERR_SHAPE,
             "rq_qgemm: out_acc alignment / ldacc");
  RQ_REQUIRE(!d->out_f32 || (rq_aligned(d->out_f32, 16) && d->ldf >= n_out && d->ldf % 4 == 0), RQ_ERR_SHAPE,
             "rq_qgemm: out_f32 alignment / ldf");
  RQ_REQUIRE(!d->residual || (rq_aligned(d->residual, 16) && d->ldr >= n_out && d->ldr % 4 == 0), RQ_ERR_SHAPE,
             "rq_qgemm: residual alignment / ldr");
  if (d->out_q) {
    RQ_REQUIRE(rq_aligned(d->out_q, 4) && d->ldq >= n_out && d->ldq % 4 == 0, RQ_ERR_SHAPE, "rq_qgemm: out_q alignment / ldq");
    RQ_REQUIRE(d->bits_o >= 2 && d->bits_o <= 8, RQ_ERR_INVALID_ARG, "rq_qgemm: bits_o = %d not in 2..8", d->bits_o);
    const int ns = d->n_seg > 0 ? d->n_seg : 1;
    RQ_REQUIRE(ns <= 4, RQ_ERR_INVALID_ARG, "rq_qgemm: n_seg = %d > 4", ns);
    RQ_REQUIRE(ns == 1 || (d->seg_len > 0 && d->seg_len % 4 == 0 && (int64_t)d->seg_len * ns >= n_out), RQ_ERR_SHAPE,
               "rq_qgemm: seg_len = %d must be a multiple of 4 and cover N", d->seg_len);
    for (int i = 0; i < ns; ++i) {
      RQ_REQUIRE(d->s_o[i] > 0.f && std::isfinite(d->s_o[i]), RQ_ERR_INVALID_ARG, "rq_qgemm: s_o[%d] must be > 0", i);
      RQ_REQUIRE(fits_i8(d->bits_o, d->off_o[i]), RQ_ERR_INVALID_ARG, "rq_qgemm: off_o[%d] = %d does not fit int8 at %d bits", i,
                 d->off_o[i], d->bits_o);
    }
  }
  RQ_REQUIRE(d->batch_outer <= 1 && d->batch_inner <= 1, RQ_ERR_UNSUPPORTED, "rq_qgemm: weight mode is not batched");
  return RQ_OK;
}

rq_status rq_qgemm_ln_quant(rq_ctx* ctx, const rq_gemm_desc* d, const rq_ln_desc* ln) {
  RQ_CHECK_CTX("rq_qgemm_ln_quant");
  RQ_REQUIRE(ln, RQ_ERR_INVALID_ARG, "rq_qgemm_ln_quant: the LayerNorm descriptor is NULL");
  RQ_REQUIRE(d->A && d->B, RQ_ERR_INVALID_ARG, "rq_qgemm: A and B must be non-NULL");
  RQ_REQUIRE(d->M >= 0 && d->N > 0 && d->K > 0, RQ_ERR_SHAPE, "rq_qgemm: M = %lld, N = %d, K = %d", (long long)d->M, d->N, d->K);
  RQ_REQUIRE(rq_aligned(d->A, 16) && rq_aligned(d->B, 16), RQ_ERR_INVALID_ARG, "rq_qgemm: A and B need 16-byte alignment");
  RQ_REQUIRE(d->lda >= d->K && d->lda % 16 == 0, RQ_ERR_SHAPE, "rq_qgemm: lda = %lld must be >= K and a multiple of 16",
             (long long)d->lda);
  rq_status st = check_qgemm_weight(ctx, d);
  if (st != RQ_OK) return st;
  if ((st = check_ln(ctx, ln, false)) != RQ_OK) return st;
  RQ_REQUIRE(ln->T == d->M && ln->D == d->N, RQ_ERR_SHAPE, "rq_qgemm_ln_quant: the normalization is %lld x %d, the GEMM output %lld x %d",
             (long long)ln->T, ln->D, (long long)d->M, d->N);
  RQ_REQUIRE(rq_qgemm_rowln_applies(d, ln), RQ_ERR_UNSUPPORTED,
             "rq_qgemm_ln_quant: needs packed 4-bit weights, N in {256, 512, 768}, a residual, out_f32 as the only GEMM output, no "
             "activation, codes of at most 6 bits and no rowsum; use rq_qgemm + rq_ln_quant otherwise");
  RQ_NEED_DEVICE();
  if (d->M == 0) return RQ_OK;
  return rq_launch_qgemm_rowln(ctx, d, ln);
}

rq_status rq_softmax_log2_quant(rq_ctx* ctx, const rq_softmax_desc* d) {
  RQ_CHECK_CTX("rq_softmax_log2_quant");
  RQ_REQUIRE(d->acc && d->codes, RQ_ERR_INVALID_ARG, "rq_softmax_log2_quant: acc and codes must be non-NULL");
  RQ_REQUIRE(d->G >= 0 && d->Nq > 0 && d->Nk > 0 && d->H > 0, RQ_ERR_SHAPE, "rq_softmax_log2_quant: G = %lld, H = %d, Nq = %d, Nk = %d",
             (long long)d->G, d->H, d->Nq, d->Nk);
  RQ_REQUIRE(d->ld >= d->Nk && d->ld % 4 == 0 && d->ld <= 4096, RQ_ERR_SHAPE,
             "rq_softmax_log2_quant: ld = %lld must be >= Nk, a multiple of 4 and at most 4096", (long long)d->ld);
  RQ_REQUIRE(rq_aligned(d->acc, 16) && rq_aligned(d->codes, 4), RQ_ERR_INVALID_ARG,
             "rq_softmax_log2_quant: acc needs 16-byte, codes 4-byte alignment");
  RQ_REQUIRE(d->bits >= 2 && d->bits <= 8, RQ_ERR_INVALID_ARG, "rq_softmax_log2_quant: bits = %d not in 2..8", d->bits);
  RQ_REQUIRE(d->s_log > 0.f && std::isfinite(d->s_log), RQ_ERR_INVALID_ARG, "rq_softmax_log2_quant: s_log must be > 0");
  RQ_REQUIRE(d->logit_scale > 0.0 && std::isfinite(d->logit_scale), RQ_ERR_INVALID_ARG,
             "rq_softmax_log2_quant: logit_scale must be > 0");
  RQ_REQUIRE(d->mask == RQ_MASK_NONE || d->mask == RQ_MASK_CAUSAL, RQ_ERR_INVALID_ARG, "rq_softmax_log2_quant: mask %d", d->mask);
  RQ_REQUIRE(d->mask != RQ_MASK_CAUSAL || d->Nq == d->Nk, RQ_ERR_SHAPE, "rq_softmax_log2_quant: causal needs Nq == Nk");
  RQ_REQUIRE((d->flags & ~RQ_LOG_ZERO_AT_MAX_CODE) == 0, RQ_ERR_INVALID_ARG, "rq_softmax_log2_quant: flags = %d", d->flags);
  RQ_NEED_DEVICE();
  if (d->G == 0) return RQ_OK;
  return rq_launch_softmax(ctx, d);
}

rq_status rq_qk_softmax_log2_quant(rq_ctx* ctx, const rq_qk_softmax_desc* d) {
  RQ_CHECK_CTX("rq_qk_softmax_log2_quant");
  RQ_REQUIRE(d->Q && d->K && d->codes, RQ_ERR_INVALID_ARG, "rq_qk_softmax_log2_quant: Q, K and codes must be non-NULL");
  RQ_REQUIRE(d->batch >= 0 && d->H > 0 && d->N > 0, RQ_ERR_SHAPE, "rq_qk_softmax_log2_quant: batch = %lld, H = %d, N = %d",
             (long long)d->batch, d->H, d->N);
  RQ_REQUIRE(d->d_head == 32 || d->d_head == 64 || d->d_head == 128, RQ_ERR_SHAPE,
             "rq_qk_softmax_log2_quant: d_head = %d must be 32, 64 or 128", d->d_head);
  RQ_REQUIRE(rq_qk_softmax_supported(d->N, d->d_head, d->bias != nullptr), RQ_ERR_SHAPE,
             "rq_qk_softmax_log2_quant: N = %d exceeds %s; use rq_qgemm + rq_softmax_log2_quant", d->N,
             d->bias ? "288 (rows with a bias)" : "65536");
  RQ_REQUIRE(d->ld_tok >= (int64_t)d->H * d->d_head && d->ld_tok % 16 == 0, RQ_ERR_SHAPE,
             "rq_qk_softmax_log2_quant: ld_tok = %lld must be >= H*d_head and a multiple of 16", (long long)d->ld_tok);
  RQ_REQUIRE(rq_aligned(d->Q, 16) && rq_aligned(d->K, 16) && rq_aligned(d->codes, 16), RQ_ERR_INVALID_ARG,
             "rq_qk_softmax_log2_quant: Q, K and codes need 16-byte alignment");
  RQ_REQUIRE(d->ld >= d->N && d->ld % 16 == 0, RQ_ERR_SHAPE, "rq_qk_softmax_log2_quant: ld = %lld must be >= N and a multiple of 16",
             (long long)d->ld);
  RQ_REQUIRE(d->q_off >= 0 && d->q_off <= 128 && d->k_off >= 0 && d->k_off <= 128 && d->z_q >= 0 && d->z_q <= 255 && d->z_k >= 0 &&
                 d->z_k <= 255,
             RQ_ERR_INVALID_ARG, "rq_qk_softmax_log2_quant: offsets must be in 0..128 and zero-points in 0..255");
  RQ_REQUIRE(d->bits >= 2 && d->bits <= 8, RQ_ERR_INVALID_ARG, "rq_qk_softmax_log2_quant: bits = %d not in 2..8", d->bits);
  RQ_REQUIRE(d->s_log > 0.f && std::isfinite(d->s_log), RQ_ERR_INVALID_ARG, "rq_qk_softmax_log2_quant: s_log must be > 0");
  RQ_REQUIRE(d->logit_scale > 0.0 && std::isfinite(d->logit_scale), RQ_ERR_INVALID_ARG,
             "rq_qk_softmax_log2_quant: logit_scale must be > 0");
  RQ_REQUIRE(d->mask == RQ_MASK_NONE || d->mask == RQ_MASK_CAUSAL, RQ_ERR_INVALID_ARG, "rq_qk_softmax_log2_quant: mask %d", d->mask);
  RQ_NEED_DEVICE();
  if (d->batch == 0) return RQ_OK;
  return rq_launch_qk_softmax(ctx, d->Q, d->K, d->ld_tok, d->batch, d->H, d->N, d->d_head, d->q_off, d->z_q, d->k_off, d->z_k,
                              d->logit_scale, d->bias, d->mask, d->s_log, d->bits, d->codes, d->ld);
}

rq_status rq_attn_fused(rq_ctx* ctx, const rq_attn_fused_desc* d) {
  RQ_CHECK_CTX("rq_attn_fused");
  RQ_REQUIRE(d->Q && d->K && d->V, RQ_ERR_INVALID_ARG, "rq_attn_fused: Q, K and V must be non-NULL");
  RQ_REQUIRE(d->out_f32 || d->out_q, RQ_ERR_INVALID_ARG, "rq_attn_fused: no output requested");
  RQ_REQUIRE(d->batch >= 0 && d->H > 0 && d->N > 0, RQ_ERR_SHAPE, "rq_attn_fused: batch = %lld, H = %d, N = %d", (long long)d->batch,
             d->H, d->N);
  RQ_REQUIRE(d->bits_p >= 2 && d->bits_p <= 8, RQ_ERR_INVALID_ARG, "rq_attn_fused: bits_p = %d not in 2..8", d->bits_p);
  RQ_REQUIRE((d->flags & ~RQ_LOG_ZERO_AT_MAX_CODE) == 0, RQ_ERR_INVALID_ARG, "rq_attn_fused: flags = %d", d->flags);
  RQ_REQUIRE(rq_attn_fused_supported(d->N, d->d_head, d->bits_p, d->bias != nullptr), RQ_ERR_SHAPE,
             "rq_attn_fused: N = %d, d_head = %d, bits_p = %d%s outside the fused kernel's range; use the separate calls", d->N,
             d->d_head, d->bits_p, d->bias ? " with a bias" : "");
  RQ_REQUIRE(rq_aligned(d->bias, 4), RQ_ERR_INVALID_ARG, "rq_attn_fused: bias needs 4-byte alignment");
  RQ_REQUIRE(d->ld_tok >= (int64_t)d->H * d->d_head && d->ld_tok % 16 == 0, RQ_ERR_SHAPE,
             "rq_attn_fused: ld_tok = %lld must be >= H*d_head and a multiple of 16", (long long)d->ld_tok);
  RQ_REQUIRE(rq_aligned(d->Q, 16) && rq_aligned(d->K, 16) && rq_aligned(d->V, 4), RQ_ERR_INVALID_ARG,
             "rq_attn_fused: Q and K need 16-byte, V 4-byte alignment");
  RQ_REQUIRE(!d->codes || (rq_aligned(d->codes, 16) && d->ld >= d->N && d->ld % 16 == 0), RQ_ERR_SHAPE,
             "rq_attn_fused: codes need 16-byte alignment and ld >= N, a multiple of 16");
  RQ_REQUIRE(d->q_off >= 0 && d->q_off <= 128 && d->k_off >= 0 && d->k_off <= 128 && d->v_off >= 0 && d->v_off <= 128 &&
                 d->z_q >= 0 && d->z_q <= 255 && d->z_k >= 0 && d->z_k <= 255 && d->z_v >= 0 && d->z_v <= 255,
             RQ_ERR_INVALID_ARG, "rq_attn_fused: offsets must be in 0..128 and zero-points in 0..255");
  RQ_REQUIRE(d->s_log > 0.f && std::isfinite(d->s_log) && d->s_v > 0.f && std::isfinite(d->s_v), RQ_ERR_INVALID_ARG,
             "rq_attn_fused: s_log and s_v must be > 0");
  RQ_REQUIRE(d->logit_scale > 0.0 && std::isfinite(d->logit_scale), RQ_ERR_INVALID_ARG, "rq_attn_fused: logit_scale must be > 0");
  const int64_t width = (int64_t)d->H * d->d_head;
  RQ_REQUIRE(!d->out_f32 || (rq_aligned(d->out_f32, 16) && d->ldf >= width && d->ldf % 4 == 0), RQ_ERR_SHAPE,
             "rq_attn_fused: out_f32 alignment / ldf");
  if (d->out_q) {
    RQ_REQUIRE(rq_aligned(d->out_q, 4) && d->ldq >= width && d->ldq % 4 == 0, RQ_ERR_SHAPE, "rq_attn_fused: out_q alignment / ldq");
    RQ_REQUIRE(d->bits_o >= 2 && d->bits_o <= 8 && d->s_o > 0.f && fits_i8(d->bits_o, d->off_o), RQ_ERR_INVALID_ARG,
               "rq_attn_fused: bad output quantizer (bits_o = %d, s_o = %g, off_o = %d)", d->bits_o, (double)d->s_o, d->off_o);
  }
  RQ_NEED_DEVICE();
  if (d->batch == 0) return RQ_OK;
  return rq_launch_attn_fused(ctx, d);
}

rq_status rq_attn_pv(rq_ctx* ctx, const rq_pv_desc* d) {
  RQ_CHECK_CTX("rq_attn_pv");
  RQ_REQUIRE(d->codes && d->V, RQ_ERR_INVALID_ARG, "rq_attn_pv: codes and V must be non-NULL");
  RQ_REQUIRE(d->out_f32 || d->out_q, RQ_ERR_INVALID_ARG, "rq_attn_pv: no output requested");
  RQ_REQUIRE(d->batch >= 0 && d->H > 0 && d->Nq > 0 && d->Nk > 0, RQ_ERR_SHAPE, "rq_attn_pv: batch = %lld, H = %d, Nq = %d, Nk = %d",
             (long long)d->batch, d->H, d->Nq, d->Nk);
  RQ_REQUIRE(d->d_head == 32 || d->d_head == 64 || d->d_head == 128, RQ_ERR_SHAPE, "rq_attn_pv: d_head = %d must be 32, 64 or 128",
             d->d_head);
  RQ_REQUIRE(d->ld >= d->Nk && d->ld % 16 == 0, RQ_ERR_SHAPE, "rq_attn_pv: ld = %lld must be >= Nk and a multiple of 16",
             (long long)d->ld);
  RQ_REQUIRE(rq_aligned(d->codes, 16) && rq_aligned(d->V, 16), RQ_ERR_INVALID_ARG, "rq_attn_pv: codes and V need 16-byte alignment");
  RQ_REQUIRE(d->ldv >= (int64_t)d->H * d->d_head && d->ldv % 16 == 0, RQ_ERR_SHAPE, "rq_attn_pv: ldv must be >= H*d_head and a multiple of 16");
  RQ_REQUIRE(d->bits_p >= 2 && d->bits_p <= 8, RQ_ERR_INVALID_ARG, "rq_attn_pv: bits_p = %d not in 2..8", d->bits_p);
  RQ_REQUIRE((d->flags & ~RQ_LOG_ZERO_AT_MAX_CODE) == 0, RQ_ERR_INVALID_ARG, "rq_attn_pv: flags = %d", d->flags);
  RQ_REQUIRE(d->s_log > 0.f && d->s_v > 0.f, RQ_ERR_INVALID_ARG, "rq_attn_pv: s_log and s_v must be > 0");
  RQ_REQUIRE(d->mask == RQ_MASK_NONE || d->mask == RQ_MASK_CAUSAL, RQ_ERR_INVALID_ARG, "rq_attn_pv: mask %d", d->mask);
  RQ_REQUIRE(d->mask != RQ_MASK_CAUSAL || d->Nq == d->Nk, RQ_ERR_SHAPE, "rq_attn_pv: causal needs Nq == Nk");
  const int64_t width = (int64_t)d->H * d->d_head;
  RQ_REQUIRE(!d->out_f32 || (rq_aligned(d->out_f32, 16) && d->ldf >= width && d->ldf % 4 == 0), RQ_ERR_SHAPE,
             "rq_attn_pv: out_f32 alignment / ldf");
  if (d->out_q) {
    RQ_REQUIRE(rq_aligned(d->out_q, 4) && d->ldq >= width && d->ldq % 4 == 0, RQ_ERR_SHAPE, "rq_attn_pv: out_q alignment / ldq");
    RQ_REQUIRE(d->bits_o >= 2 && d->bits_o <= 8 && d->s_o > 0.f && fits_i8(d->bits_o, d->off_o), RQ_ERR_INVALID_ARG,
               "rq_attn_pv: bad output quantizer (bits_o = %d, s_o = %g, off_o = %d)", d->bits_o, (double)d->s_o, d->off_o);
  }
  RQ_NEED_DEVICE();
  if (d->batch == 0) return RQ_OK;
  return rq_launch_pv(ctx, d);
}

rq_status rq_rowsum_i8(rq_ctx* ctx, const int8_t* A, int64_t M, int32_t K, int64_t lda, int32_t* rowsum) {
  if (!ctx) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_rowsum_i8: ctx is NULL");
  RQ_REQUIRE(A && rowsum, RQ_ERR_INVALID_ARG, "rq_rowsum_i8: A and rowsum must be non-NULL");
  RQ_REQUIRE(M >= 0 && K > 0 && K % 4 == 0 && lda >= K && lda % 4 == 0 && rq_aligned(A, 4), RQ_ERR_SHAPE,
             "rq_rowsum_i8: K and lda must be multiples of 4, A 4-byte aligned");
  RQ_NEED_DEVICE();
  if (M == 0) return RQ_OK;
  return rq_launch_rowsum(ctx, A, M, K, lda, rowsum);
}

rq_status rq_ln_channel_minmax(rq_ctx* ctx, const float* x, int64_t T, int32_t D, int64_t ldx, int32_t norm_kind, double eps,
                               const float* gamma, const float* beta, double* cmin, double* cmax) {
  if (!ctx) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_ln_channel_minmax: ctx is NULL");
  RQ_REQUIRE(x && gamma && cmin && cmax, RQ_ERR_INVALID_ARG, "rq_ln_channel_minmax: x, gamma, cmin, cmax must be non-NULL");
  RQ_REQUIRE(T > 0 && D > 0 && D % 4 == 0 && D <= 8192 && ldx >= D && ldx % 4 == 0 && rq_aligned(x, 16), RQ_ERR_SHAPE,
             "rq_ln_channel_minmax: T > 0, D a multiple of 4 and <= 8192, ldx a multiple of 4, x 16-byte aligned");
  RQ_REQUIRE(norm_kind == RQ_NORM_LAYERNORM || norm_kind == RQ_NORM_RMSNORM, RQ_ERR_INVALID_ARG, "rq_ln_channel_minmax: norm_kind");
  RQ_NEED_DEVICE();
  return rq_launch_ln_channel_minmax(ctx, x, T, D, ldx, norm_kind, eps, gamma, beta, cmin, cmax);
}

rq_status rq_minmax_f32(rq_ctx* ctx, const float* v, int64_t rows, int64_t cols, int64_t ld, double* out2) {
  if (!ctx) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_minmax_f32: ctx is NULL");
  RQ_REQUIRE(v && out2, RQ_ERR_INVALID_ARG, "rq_minmax_f32: v and out2 must be non-NULL");
  RQ_REQUIRE(rows > 0 && cols > 0 && ld >= cols, RQ_ERR_SHAPE, "rq_minmax_f32: rows, cols > 0 and ld >= cols");
  RQ_NEED_DEVICE();
  return rq_launch_minmax_f32(ctx, v, rows, cols, ld, out2);
}

rq_status rq_dual_clip_learn(rq_ctx* ctx, const rq_dual_clip_desc* d) {
  RQ_CHECK_CTX("rq_dual_clip_learn");
  RQ_REQUIRE(d->x && d->alpha1 && d->alpha2, RQ_ERR_INVALID_ARG, "rq_dual_clip_learn: x, alpha1 and alpha2 must be non-NULL");
  RQ_REQUIRE(d->T >= 1 && d->D >= 1 && d->ldx >= d->D, RQ_ERR_SHAPE, "rq_dual_clip_learn: T = %lld, D = %d, ldx = %lld",
             (long long)d->T, d->D, (long long)d->ldx);
  RQ_REQUIRE(rq_aligned(d->x, 4) && rq_aligned(d->alpha1, 8) && rq_aligned(d->alpha2, 8) && rq_aligned(d->up, 8) &&
                 rq_aligned(d->lo, 8) && rq_aligned(d->loss0, 8) && rq_aligned(d->loss, 8) && rq_aligned(d->clip_up, 4) &&
                 rq_aligned(d->clip_lo, 4),
             RQ_ERR_INVALID_ARG, "rq_dual_clip_learn: float32 arrays need 4-byte, float64 arrays 8-byte alignment");
  RQ_REQUIRE(d->bits >= 2 && d->bits <= 16, RQ_ERR_INVALID_ARG, "rq_dual_clip_learn: bits = %d not in 2..16", d->bits);
  RQ_REQUIRE(d->iters >= 0 && d->iters <= 100000, RQ_ERR_INVALID_ARG, "rq_dual_clip_learn: iters = %d", d->iters);
  RQ_REQUIRE(d->waves >= 0 && d->waves <= 16, RQ_ERR_INVALID_ARG, "rq_dual_clip_learn: waves = %d not in 0..16", d->waves);
  RQ_REQUIRE(d->lr > 0.0 && std::isfinite(d->lr) && std::isfinite(d->alpha0), RQ_ERR_INVALID_ARG,
             "rq_dual_clip_learn: lr must be positive and finite, alpha0 finite");
  if (d->gamma) {
    RQ_REQUIRE(d->norm_kind == RQ_NORM_LAYERNORM || d->norm_kind == RQ_NORM_RMSNORM, RQ_ERR_INVALID_ARG,
               "rq_dual_clip_learn: norm_kind %d", d->norm_kind);
    RQ_REQUIRE(d->eps > 0.0 && std::isfinite(d->eps), RQ_ERR_INVALID_ARG, "rq_dual_clip_learn: eps must be positive and finite");
    RQ_REQUIRE(d->D % 4 == 0 && d->ldx % 4 == 0 && rq_aligned(d->x, 16), RQ_ERR_SHAPE,
               "rq_dual_clip_learn: with a normalization D and ldx must be multiples of 4 and x 16-byte aligned");
    RQ_REQUIRE(d->workspace && rq_aligned(d->workspace, 16) && d->workspace_bytes >= rq_dual_clip_workspace_bytes(d->T),
               RQ_ERR_WORKSPACE, "rq_dual_clip_learn: workspace of %zu bytes, %zu needed (16-byte aligned)", d->workspace_bytes,
               rq_dual_clip_workspace_bytes(d->T));
  }
  RQ_NEED_DEVICE();
  return rq_launch_dual_clip(ctx, d);
}

rq_status rq_ln_channel_percentile(rq_ctx* ctx, const float* x, int64_t T, int32_t D, int64_t ldx, int32_t norm_kind, double eps,
                                   const float* gamma, const float* beta, double q_lo, double q_hi, double* lo, double* hi,
                                   void* workspace, size_t workspace_bytes) {
  if (!ctx) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_ln_channel_percentile: ctx is NULL");
  RQ_REQUIRE(x && lo && hi, RQ_ERR_INVALID_ARG, "rq_ln_channel_percentile: x, lo, hi must be non-NULL");
  RQ_REQUIRE(T > 0 && D > 0 && ldx >= D, RQ_ERR_SHAPE, "rq_ln_channel_percentile: T = %lld, D = %d, ldx = %lld", (long long)T, D,
             (long long)ldx);
  RQ_REQUIRE(q_lo >= 0.0 && q_lo <= q_hi && q_hi <= 1.0, RQ_ERR_INVALID_ARG,
             "rq_ln_channel_percentile: fractions must satisfy 0 <= q_lo <= q_hi <= 1");
  RQ_REQUIRE(rq_aligned(x, 4) && rq_aligned(lo, 8) && rq_aligned(hi, 8), RQ_ERR_INVALID_ARG, "rq_ln_channel_percentile: alignment");
  if (gamma) {
    RQ_REQUIRE(norm_kind == RQ_NORM_LAYERNORM || norm_kind == RQ_NORM_RMSNORM, RQ_ERR_INVALID_ARG,
               "rq_ln_channel_percentile: norm_kind %d", norm_kind);
    RQ_REQUIRE(eps > 0.0 && std::isfinite(eps), RQ_ERR_INVALID_ARG, "rq_ln_channel_percentile: eps must be positive and finite");
    RQ_REQUIRE(D % 4 == 0 && ldx % 4 == 0 && rq_aligned(x, 16), RQ_ERR_SHAPE,
               "rq_ln_channel_percentile: with a normalization D and ldx must be multiples of 4 and x 16-byte aligned");
    RQ_REQUIRE(workspace && rq_aligned(workspace, 16) && workspace_bytes >= (size_t)T * 16, RQ_ERR_WORKSPACE,
               "rq_ln_channel_percentile: workspace of %zu bytes, %zu needed (16-byte aligned)", workspace_bytes, (size_t)T * 16);
  }
  RQ_NEED_DEVICE();
  return rq_launch_ln_channel_percentile(ctx, x, T, D, ldx, norm_kind, eps, gamma, beta, q_lo, q_hi, lo, hi, workspace);
}

rq_status rq_gptq_quant_pack(rq_ctx* ctx, const rq_gptq_desc* d) {
  RQ_CHECK_CTX("rq_gptq_quant_pack");
  RQ_REQUIRE(d->W && d->A && d->w_out && d->s_w && d->z_w && d->colsum_w, RQ_ERR_INVALID_ARG,
             "rq_gptq_quant_pack: W, A, w_out, s_w, z_w, colsum_w must be non-NULL");
  RQ_REQUIRE(d->N > 0 && d->K > 0 && d->K % 64 == 0 && d->K <= 8192, RQ_ERR_SHAPE,
             "rq_gptq_quant_pack: N = %d, K = %d (K must be a multiple of 64, at most 8192)", d->N, d->K);
  RQ_REQUIRE(d->T >= 1 && d->T <= 131071 && d->lda >= d->K, RQ_ERR_SHAPE,
             "rq_gptq_quant_pack: T = %lld must be in 1..131071 (int32 Gram sums) and lda = %lld >= K", (long long)d->T, (long long)d->lda);
  RQ_REQUIRE(rq_aligned(d->W, 4) && rq_aligned(d->w_out, 4) && rq_aligned(d->s_w, 4) && rq_aligned(d->z_w, 4) &&
                 rq_aligned(d->colsum_w, 4) && rq_aligned(d->bias, 4) && rq_aligned(d->bias_out, 4),
             RQ_ERR_INVALID_ARG, "rq_gptq_quant_pack: arrays need 4-byte alignment");
  switch (d->format) {
    case RQ_W_U4:
      RQ_REQUIRE(d->bits == 4, RQ_ERR_INVALID_ARG, "rq_gptq_quant_pack: RQ_W_U4 needs bits = 4, got %d", d->bits);
      break;
    case RQ_W_I8_CENTERED:
      RQ_REQUIRE(d->bits >= 2 && d->bits <= 8, RQ_ERR_INVALID_ARG, "rq_gptq_quant_pack: bits = %d not in 2..8", d->bits);
      break;
    case RQ_W_I8_BAKED:
      RQ_REQUIRE(d->bits >= 2 && d->bits <= 7, RQ_ERR_INVALID_ARG, "rq_gptq_quant_pack: RQ_W_I8_BAKED needs bits in 2..7, got %d",
                 d->bits);
      break;
    default:
      return rq_fail(ctx, RQ_ERR_INVALID_ARG, "rq_gptq_quant_pack: format %d", d->format);
  }
  if (d->gate_up_rows != 0)
    RQ_REQUIRE(d->gate_up_rows > 0 && d->N == 2 * d->gate_up_rows && d->gate_up_rows % 32 == 0, RQ_ERR_SHAPE,
               "rq_gptq_quant_pack: gate_up_rows = %d needs N = 2*gate_up_rows and a multiple of 32", d->gate_up_rows);
  RQ_REQUIRE(d->a_off - d->z_a >= -255 && d->a_off - d->z_a <= 255, RQ_ERR_INVALID_ARG, "rq_gptq_quant_pack: a_off - z_a = %d",
             d->a_off - d->z_a);
  RQ_REQUIRE(d->percdamp > 0.0 && std::isfinite(d->percdamp), RQ_ERR_INVALID_ARG, "rq_gptq_quant_pack: percdamp must be > 0");
  RQ_REQUIRE(d->workspace && rq_aligned(d->workspace, 256) && d->workspace_bytes >= rq_gptq_workspace_bytes(d->N, d->K, d->T),
             RQ_ERR_WORKSPACE, "rq_gptq_quant_pack: workspace of %zu bytes, %zu needed (256-byte aligned)", d->workspace_bytes,
             rq_gptq_workspace_bytes(d->N, d->K, d->T));
  RQ_NEED_DEVICE();
  return rq_launch_gptq(ctx, d);
}

}  // extern "C"
