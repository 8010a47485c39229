// Block parameters as one flat little-endian blob: size, save (device -> host), check (host only) and load
// (host -> one device arena).  Host code only; the copies are plain hipMemcpyAsync on the context's stream.
#include <cstring>

#include "rq_internal.h"

namespace {

constexpr uint64_t ALIGN = 256;
constexpr char MAGIC[8] = {'R', 'Q', 'B', 'L', 'O', 'C', 'K', '\0'};

uint64_t up(uint64_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

struct Shapes {
  uint64_t len[RQ_BLOB_ARRAYS];      // bytes of every array a complete block of these shapes holds (bias / rel_bias optional)
};

// byte lengths from the scalar fields of a header; false if a field is out of range (message in *why)
bool shapes_of(const rq_blob_header& h, Shapes* s, const char** why) {
  *why = nullptr;
  if (h.D <= 0 || h.H <= 0 || h.Dm <= 0 || h.D > (1 << 20) || h.Dm > (1 << 22)) { *why = "D, H or Dm out of range"; return false; }
  if (h.rel_bias_elems < 0 || h.rel_bias_elems > ((int64_t)1 << 40)) { *why = "rel_bias_elems out of range"; return false; }
  for (int i = 0; i < 4; ++i) s->len[i] = (uint64_t)h.D * 4;
  for (int k = 0; k < 4; ++k) {
    const int64_t N = h.lin[k][0], K = h.lin[k][1];
    const int fmt = h.lin[k][3];
    if (N <= 0 || K <= 0 || N > (1 << 24) || K > (1 << 24)) { *why = "a linear layer's N or K is out of range"; return false; }
    if (fmt != RQ_W_I8_BAKED && fmt != RQ_W_I8_CENTERED && fmt != RQ_W_U4) { *why = "a linear layer's weight format is unknown"; return false; }
    if (fmt == RQ_W_U4 && (K & 1)) { *why = "packed 4-bit weights need an even K"; return false; }
    s->len[4 + 5 * k] = fmt == RQ_W_U4 ? (uint64_t)N * (uint64_t)(K / 2) : (uint64_t)N * (uint64_t)K;
    for (int j = 1; j < 5; ++j) s->len[4 + 5 * k + j] = (uint64_t)N * 4;
  }
  s->len[24] = (uint64_t)h.rel_bias_elems * 4;
  return true;
}

bool optional_array(int i) { return i == 24 || (i >= 4 && (i - 4) % 5 == 4) || i == 1 || i == 3; }      // rel_bias, biases, beta~ (RMSNorm)

const void* array_ptr(const rq_block_params* p, int i) {
  const rq_qlinear* lin[4] = {&p->qkv, &p->proj, &p->fc1, &p->fc2};
  switch (i) {
    case 0: return p->ln1_gamma_t;
    case 1: return p->ln1_beta_t;
    case 2: return p->ln2_gamma_t;
    case 3: return p->ln2_beta_t;
    case 24: return p->rel_bias;
  }
  const rq_qlinear* l = lin[(i - 4) / 5];
  switch ((i - 4) % 5) {
    case 0: return l->w;
    case 1: return l->s_w;
    case 2: return l->z_w;
    case 3: return l->colsum_w;
  }
  return l->bias;
}

// header of the blob of *p: scalars, shapes, offsets; false if p is inconsistent
bool make_header(const rq_block_params* p, int64_t rel_bias_elems, rq_blob_header* h, const char** why) {
  std::memset(h, 0, sizeof *h);
  std::memcpy(h->magic, MAGIC, 8);
  h->header_bytes = (uint32_t)sizeof(rq_blob_header);
  h->version = RQ_BLOB_VERSION;
  h->D = p->D; h->H = p->H; h->Dm = p->Dm; h->norm_kind = p->norm_kind; h->act = p->act; h->mask = p->mask;
  h->bits_a = p->bits_a; h->bits_p = p->bits_p; h->eps = p->eps;
  h->ln1_s = p->ln1_s; h->ln2_s = p->ln2_s; h->s_q = p->s_q; h->s_k = p->s_k; h->s_v = p->s_v; h->s_log = p->s_log;
  h->s_o = p->s_o; h->s_h = p->s_h;
  h->ln1_z = p->ln1_z; h->ln2_z = p->ln2_z; h->z_q = p->z_q; h->z_k = p->z_k; h->z_v = p->z_v; h->z_o = p->z_o; h->z_h = p->z_h;
  h->attn_path = p->attn_path; h->proj_ln_fused = p->proj_ln_fused; h->flags = p->flags; h->attn_chunk_bytes = p->attn_chunk_bytes;
  const rq_qlinear* lin[4] = {&p->qkv, &p->proj, &p->fc1, &p->fc2};
  for (int k = 0; k < 4; ++k) {
    h->lin[k][0] = lin[k]->N; h->lin[k][1] = lin[k]->K; h->lin[k][2] = lin[k]->bits; h->lin[k][3] = lin[k]->format;
  }
  h->rel_bias_elems = p->rel_bias ? rel_bias_elems : 0;
  if (p->rel_bias && rel_bias_elems <= 0) { *why = "rel_bias is set but rel_bias_elems is not positive"; return false; }
  Shapes s;
  if (!shapes_of(*h, &s, why)) return false;
  uint64_t o = up(sizeof(rq_blob_header));
  for (int i = 0; i < RQ_BLOB_ARRAYS; ++i) {
    const bool present = array_ptr(p, i) != nullptr && s.len[i] > 0;
    if (!present && !optional_array(i)) { *why = "a required array of the block is NULL"; return false; }
    h->off[i] = present ? o : 0;
    h->len[i] = present ? s.len[i] : 0;
    if (present) o += up(s.len[i]);
  }
  h->total_bytes = o;
  return true;
}

rq_status check_blob(rq_ctx* ctx, const void* blob, size_t bytes, rq_blob_header* h) {
  RQ_REQUIRE(blob != nullptr, RQ_ERR_INVALID_ARG, "block blob: NULL blob");
  RQ_REQUIRE(bytes >= sizeof(rq_blob_header), RQ_ERR_SHAPE, "block blob: %zu bytes do not hold a header (%zu)", bytes,
             sizeof(rq_blob_header));
  std::memcpy(h, blob, sizeof *h);
  RQ_REQUIRE(std::memcmp(h->magic, MAGIC, 8) == 0, RQ_ERR_INVALID_ARG, "block blob: bad magic");
  RQ_REQUIRE(h->version == RQ_BLOB_VERSION, RQ_ERR_UNSUPPORTED, "block blob: version %u, this library reads version %d",
             h->version, (int)RQ_BLOB_VERSION);
  RQ_REQUIRE(h->header_bytes == sizeof(rq_blob_header), RQ_ERR_SHAPE, "block blob: header of %u bytes, expected %zu",
             h->header_bytes, sizeof(rq_blob_header));
  RQ_REQUIRE(h->total_bytes <= bytes, RQ_ERR_SHAPE, "block blob: truncated (%zu bytes of %llu)", bytes,
             (unsigned long long)h->total_bytes);
  Shapes s;
  const char* why = nullptr;
  RQ_REQUIRE(shapes_of(*h, &s, &why), RQ_ERR_SHAPE, "block blob: %s", why);
  uint64_t lo = up(sizeof(rq_blob_header));
  for (int i = 0; i < RQ_BLOB_ARRAYS; ++i) {
    if (h->len[i] == 0 && h->off[i] == 0) {
      RQ_REQUIRE(optional_array(i) || s.len[i] == 0, RQ_ERR_SHAPE, "block blob: required array %d is absent", i);
      continue;
    }
    RQ_REQUIRE(h->len[i] == s.len[i], RQ_ERR_SHAPE, "block blob: array %d holds %llu bytes, its shape needs %llu", i,
               (unsigned long long)h->len[i], (unsigned long long)s.len[i]);
    // arrays follow each other in index order, so they cannot overlap
    RQ_REQUIRE(h->off[i] % ALIGN == 0 && h->off[i] >= lo && h->off[i] <= h->total_bytes && h->len[i] <= h->total_bytes - h->off[i],
               RQ_ERR_SHAPE, "block blob: array %d at offset %llu (+%llu) leaves the blob or overlaps its neighbour", i,
               (unsigned long long)h->off[i], (unsigned long long)h->len[i]);
    lo = h->off[i] + up(h->len[i]);
  }
  return RQ_OK;
}

}  // namespace

extern "C" {

size_t rq_block_blob_bytes(const rq_block_params* p, int64_t rel_bias_elems) {
  if (!p) return 0;
  rq_blob_header h;
  const char* why = nullptr;
  return make_header(p, rel_bias_elems, &h, &why) ? (size_t)h.total_bytes : 0;
}

rq_status rq_block_blob_save(rq_ctx* ctx, const rq_block_params* p, int64_t rel_bias_elems, void* blob_host, size_t blob_bytes) {
  RQ_REQUIRE(ctx != nullptr, RQ_ERR_INVALID_ARG, "rq_block_blob_save: ctx is NULL");
  RQ_REQUIRE(p && blob_host, RQ_ERR_INVALID_ARG, "rq_block_blob_save: NULL argument");
  rq_blob_header h;
  const char* why = nullptr;
  RQ_REQUIRE(make_header(p, rel_bias_elems, &h, &why), RQ_ERR_INVALID_ARG, "rq_block_blob_save: %s", why);
  RQ_REQUIRE(blob_bytes >= h.total_bytes, RQ_ERR_WORKSPACE, "rq_block_blob_save: blob of %zu bytes, %llu needed", blob_bytes,
             (unsigned long long)h.total_bytes);
  RQ_REQUIRE(ctx->device >= 0, RQ_ERR_UNSUPPORTED, "rq_block_blob_save: host-only context");
  std::memset(blob_host, 0, (size_t)h.total_bytes);      // padding bytes are zero: equal parameters give equal blobs
  std::memcpy(blob_host, &h, sizeof h);
  for (int i = 0; i < RQ_BLOB_ARRAYS; ++i)
    if (h.len[i])
      RQ_HIP(hipMemcpyAsync(static_cast<char*>(blob_host) + h.off[i], array_ptr(p, i), (size_t)h.len[i], hipMemcpyDeviceToHost,
                            ctx->stream));
  RQ_HIP(hipStreamSynchronize(ctx->stream));
  return RQ_OK;
}

rq_status rq_block_blob_check(const void* blob_host, size_t blob_bytes, size_t* arena_bytes) {
  rq_ctx* ctx = nullptr;
  rq_blob_header h;
  const rq_status st = check_blob(ctx, blob_host, blob_bytes, &h);
  if (st != RQ_OK) return st;
  if (arena_bytes) *arena_bytes = (size_t)h.total_bytes;
  return RQ_OK;
}

rq_status rq_block_blob_load(rq_ctx* ctx, const void* blob_host, size_t blob_bytes, void* arena_device, size_t arena_bytes,
                             rq_block_params* out) {
  RQ_REQUIRE(ctx != nullptr, RQ_ERR_INVALID_ARG, "rq_block_blob_load: ctx is NULL");
  RQ_REQUIRE(out != nullptr, RQ_ERR_INVALID_ARG, "rq_block_blob_load: out is NULL");
  rq_blob_header h;
  const rq_status st = check_blob(ctx, blob_host, blob_bytes, &h);
  if (st != RQ_OK) return st;
  RQ_REQUIRE(arena_device != nullptr && reinterpret_cast<uintptr_t>(arena_device) % ALIGN == 0, RQ_ERR_INVALID_ARG,
             "rq_block_blob_load: the arena is NULL or not 256-byte aligned");
  RQ_REQUIRE(arena_bytes >= h.total_bytes, RQ_ERR_WORKSPACE, "rq_block_blob_load: arena of %zu bytes, %llu needed", arena_bytes,
             (unsigned long long)h.total_bytes);
  RQ_REQUIRE(ctx->device >= 0, RQ_ERR_UNSUPPORTED, "rq_block_blob_load: host-only context");
  RQ_HIP(hipMemcpyAsync(arena_device, blob_host, (size_t)h.total_bytes, hipMemcpyHostToDevice, ctx->stream));
  RQ_HIP(hipStreamSynchronize(ctx->stream));
  std::memset(out, 0, sizeof *out);
  out->D = h.D; out->H = h.H; out->Dm = h.Dm; out->norm_kind = h.norm_kind; out->act = h.act; out->mask = h.mask;
  out->bits_a = h.bits_a; out->bits_p = h.bits_p; out->eps = h.eps;
  out->ln1_s = h.ln1_s; out->ln2_s = h.ln2_s; out->s_q = h.s_q; out->s_k = h.s_k; out->s_v = h.s_v; out->s_log = h.s_log;
  out->s_o = h.s_o; out->s_h = h.s_h;
  out->ln1_z = h.ln1_z; out->ln2_z = h.ln2_z; out->z_q = h.z_q; out->z_k = h.z_k; out->z_v = h.z_v; out->z_o = h.z_o; out->z_h = h.z_h;
  out->attn_path = h.attn_path; out->proj_ln_fused = h.proj_ln_fused; out->flags = h.flags; out->attn_chunk_bytes = h.attn_chunk_bytes;
  const char* base = static_cast<const char*>(arena_device);
  auto at = [&](int i) -> const void* { return h.len[i] ? base + h.off[i] : nullptr; };
  out->ln1_gamma_t = static_cast<const float*>(at(0)); out->ln1_beta_t = static_cast<const float*>(at(1));
  out->ln2_gamma_t = static_cast<const float*>(at(2)); out->ln2_beta_t = static_cast<const float*>(at(3));
  out->rel_bias = static_cast<const float*>(at(24));
  rq_qlinear* lin[4] = {&out->qkv, &out->proj, &out->fc1, &out->fc2};
  for (int k = 0; k < 4; ++k) {
    rq_qlinear* l = lin[k];
    l->N = h.lin[k][0]; l->K = h.lin[k][1]; l->bits = h.lin[k][2]; l->format = h.lin[k][3];
    l->w = at(4 + 5 * k);
    l->s_w = static_cast<const float*>(at(5 + 5 * k));
    l->z_w = static_cast<const int32_t*>(at(6 + 5 * k));
    l->colsum_w = static_cast<const int32_t*>(at(7 + 5 * k));
    l->bias = static_cast<const float*>(at(8 + 5 * k));
  }
  return RQ_OK;
}

}  // extern "C"
