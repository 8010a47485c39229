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
  delete ctx;
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

static bool fits_i8(int bits, int off) { return -off >= -128 && ((1 << bits) - 1 - off) <= 127; }

rq_status rq_ln_quant(rq_ctx* ctx, const rq_ln_desc* d) {
  RQ_CHECK_CTX("rq_ln_quant");
  RQ_REQUIRE(d->x && d->gamma_t && d->q, RQ_ERR_INVALID_ARG, "rq_ln_quant: x, gamma_t and q must be non-NULL");
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
  RQ_NEED_DEVICE();
  if (d->T == 0) return RQ_OK;
  return rq_launch_ln_quant(ctx, d);
}

}  // extern "C"
