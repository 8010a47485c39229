// CPU-only check of the library's host layer under AddressSanitizer and UndefinedBehaviorSanitizer: argument
// validation of every entry point, the workspace plans, and the parameter blob (including a few thousand damaged
// headers).  Runs with a host-only context, so no call reaches a kernel launcher; a sanitizer report, a wrong status,
// or a launch ends the program with a non-zero exit code.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "repquant.h"

extern int g_stub_launches;

static int g_fail = 0;
#define EXPECT(cond)                                                          \
  do {                                                                        \
    if (!(cond)) {                                                            \
      std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond);           \
      ++g_fail;                                                               \
    }                                                                         \
  } while (0)

template <class T> static T* fake() { return reinterpret_cast<T*>(uintptr_t{0x10000}); }      // never dereferenced

static rq_ln_desc ln_desc() {
  rq_ln_desc d{};
  d.T = 4; d.D = 64; d.norm_kind = RQ_NORM_LAYERNORM; d.eps = 1e-6; d.x = fake<float>(); d.ldx = 64;
  d.gamma_t = fake<float>(); d.beta_t = fake<float>(); d.s_tilde = 0.1f; d.z_tilde = 3; d.bits = 4; d.store_off = 3;
  d.q = fake<int8_t>(); d.ldq = 64;
  return d;
}

static rq_gemm_desc gemm_desc() {
  rq_gemm_desc d{};
  d.M = 64; d.N = 64; d.K = 64; d.A = fake<int8_t>(); d.lda = 64; d.a_off = 8; d.z_a = 8; d.s_a = 0.1f;
  d.B = fake<void>(); d.ldb = 64; d.b_format = RQ_W_I8_BAKED; d.s_b = fake<float>(); d.z_b = fake<int32_t>();
  d.colsum_b = fake<int32_t>(); d.batch_outer = 1; d.batch_inner = 1; d.n_seg = 1; d.out_f32 = fake<float>(); d.ldf = 64;
  return d;
}

static rq_qlinear qlinear(int N, int K, int format) {
  rq_qlinear l{};
  l.N = N; l.K = K; l.bits = format == RQ_W_U4 ? 4 : 8; l.format = format;
  l.w = fake<void>(); l.s_w = fake<float>(); l.z_w = fake<int32_t>(); l.colsum_w = fake<int32_t>(); l.bias = fake<float>();
  return l;
}

static rq_block_params block_params(int D, int H, int Dm) {
  rq_block_params p{};
  p.D = D; p.H = H; p.Dm = Dm; p.norm_kind = RQ_NORM_LAYERNORM; p.act = RQ_ACT_GELU; p.mask = RQ_MASK_NONE;
  p.bits_a = 4; p.bits_p = 4; p.eps = 1e-6;
  p.ln1_gamma_t = p.ln1_beta_t = p.ln2_gamma_t = p.ln2_beta_t = fake<float>();
  p.ln1_s = p.ln2_s = p.s_q = p.s_k = p.s_v = p.s_o = p.s_h = 0.1f; p.s_log = 1.f;
  p.ln1_z = p.ln2_z = p.z_q = p.z_k = p.z_v = p.z_o = p.z_h = 7;
  p.qkv = qlinear(3 * D, D, RQ_W_U4); p.proj = qlinear(D, D, RQ_W_U4); p.fc1 = qlinear(Dm, D, RQ_W_U4); p.fc2 = qlinear(D, Dm, RQ_W_U4);
  return p;
}

static void check_entry_points(rq_ctx* ctx) {
  {   // rq_ln_quant
    rq_ln_desc d = ln_desc();
    EXPECT(rq_ln_quant(ctx, &d) == RQ_ERR_UNSUPPORTED);
    EXPECT(rq_ln_quant(ctx, nullptr) == RQ_ERR_INVALID_ARG);
    EXPECT(rq_ln_quant(nullptr, &d) == RQ_ERR_INVALID_ARG);
    d = ln_desc(); d.bits = 9; EXPECT(rq_ln_quant(ctx, &d) == RQ_ERR_INVALID_ARG);
    d = ln_desc(); d.s_tilde = std::nanf(""); EXPECT(rq_ln_quant(ctx, &d) == RQ_ERR_INVALID_ARG);
    d = ln_desc(); d.D = 66; EXPECT(rq_ln_quant(ctx, &d) == RQ_ERR_SHAPE);
    d = ln_desc(); d.T = INT64_MAX; d.ldx = INT64_MAX; EXPECT(rq_ln_quant(ctx, &d) != RQ_OK);
    d = ln_desc(); d.D = INT32_MAX - 3; d.ldx = INT64_MAX; d.ldq = INT64_MAX; EXPECT(rq_ln_quant(ctx, &d) != RQ_OK);
    EXPECT(std::strlen(rq_last_error(ctx)) > 0);
  }
  {   // rq_qgemm, rq_qgemm_ln_quant
    rq_gemm_desc g = gemm_desc();
    EXPECT(rq_qgemm(ctx, &g) == RQ_ERR_UNSUPPORTED);
    EXPECT(rq_qgemm(ctx, nullptr) == RQ_ERR_INVALID_ARG);
    g = gemm_desc(); g.K = 60; EXPECT(rq_qgemm(ctx, &g) == RQ_ERR_SHAPE);
    g = gemm_desc(); g.b_format = 7; EXPECT(rq_qgemm(ctx, &g) == RQ_ERR_INVALID_ARG);
    g = gemm_desc(); g.M = INT64_MAX; g.N = INT32_MAX; g.K = INT32_MAX - 63 + 0; EXPECT(rq_qgemm(ctx, &g) != RQ_OK);
    g = gemm_desc(); g.n_seg = 5; EXPECT(rq_qgemm(ctx, &g) != RQ_OK);
    g = gemm_desc(); g.n_seg = -1; EXPECT(rq_qgemm(ctx, &g) != RQ_OK);
    g = gemm_desc(); g.out_f32 = nullptr; g.out_q = fake<int8_t>(); g.ldq = 64; g.bits_o = 8; g.n_seg = 4; g.seg_len = 16;
    for (int i = 0; i < 4; ++i) { g.s_o[i] = 0.1f; g.z_o[i] = 100; g.off_o[i] = 128; }
    EXPECT(rq_qgemm(ctx, &g) == RQ_ERR_UNSUPPORTED);
    g.seg_len = 0; EXPECT(rq_qgemm(ctx, &g) != RQ_OK);
    rq_ln_desc l = ln_desc();
    g = gemm_desc();
    EXPECT(rq_qgemm_ln_quant(ctx, &g, nullptr) == RQ_ERR_INVALID_ARG);
    EXPECT(rq_qgemm_ln_quant(ctx, &g, &l) != RQ_OK);
  }
  {   // rq_softmax_log2_quant, rq_attn_pv, rq_qk_softmax_log2_quant, rq_attn_fused
    rq_softmax_desc s{};
    s.G = 2; s.H = 2; s.Nq = 8; s.Nk = 8; s.ld = 16; s.acc = fake<int32_t>(); s.logit_scale = 0.1; s.s_log = 1.f; s.bits = 4;
    s.codes = fake<uint8_t>();
    EXPECT(rq_softmax_log2_quant(ctx, &s) == RQ_ERR_UNSUPPORTED);
    EXPECT(rq_softmax_log2_quant(ctx, nullptr) == RQ_ERR_INVALID_ARG);
    s.flags = 64; EXPECT(rq_softmax_log2_quant(ctx, &s) == RQ_ERR_INVALID_ARG);
    s.flags = 0; s.Nk = INT32_MAX; s.ld = INT64_MAX; EXPECT(rq_softmax_log2_quant(ctx, &s) != RQ_OK);
    rq_pv_desc v{};
    v.batch = 1; v.H = 2; v.Nq = 8; v.Nk = 8; v.d_head = 32; v.ld = 16; v.codes = fake<uint8_t>(); v.V = fake<int8_t>(); v.ldv = 192;
    v.s_log = 1.f; v.s_v = 0.1f; v.z_v = 3; v.v_off = 3; v.bits_p = 4; v.out_f32 = fake<float>(); v.ldf = 64;
    EXPECT(rq_attn_pv(ctx, &v) == RQ_ERR_UNSUPPORTED);
    v.d_head = 48; EXPECT(rq_attn_pv(ctx, &v) == RQ_ERR_SHAPE);
    v.d_head = 32; v.batch = INT64_MAX; EXPECT(rq_attn_pv(ctx, &v) != RQ_OK);
    rq_qk_softmax_desc q{};
    q.batch = 1; q.H = 2; q.N = 8; q.d_head = 32; q.Q = fake<int8_t>(); q.K = fake<int8_t>(); q.ld_tok = 192; q.q_off = 3; q.z_q = 3;
    q.k_off = 3; q.z_k = 3; q.logit_scale = 0.1; q.s_log = 1.f; q.bits = 4; q.codes = fake<uint8_t>(); q.ld = 16;
    EXPECT(rq_qk_softmax_log2_quant(ctx, &q) == RQ_ERR_UNSUPPORTED);
    q.N = 70000; EXPECT(rq_qk_softmax_log2_quant(ctx, &q) == RQ_ERR_SHAPE);
    rq_attn_fused_desc f{};
    f.batch = 1; f.H = 2; f.N = 64; f.d_head = 64; f.Q = f.K = f.V = fake<int8_t>(); f.ld_tok = 384; f.q_off = f.z_q = f.k_off = f.z_k = 3;
    f.v_off = f.z_v = 3; f.logit_scale = 0.1; f.s_log = 1.f; f.s_v = 0.1f; f.bits_p = 4; f.out_f32 = fake<float>(); f.ldf = 128;
    EXPECT(rq_attn_fused(ctx, &f) == RQ_ERR_UNSUPPORTED);
    f.N = 320; EXPECT(rq_attn_fused(ctx, &f) == RQ_ERR_SHAPE);
    f.N = 64; f.flags = -1; EXPECT(rq_attn_fused(ctx, &f) == RQ_ERR_INVALID_ARG);
  }
  {   // preparation calls
    rq_fold_desc f{};
    f.D = 64; f.D_out = 32; f.s_ch = fake<float>(); f.z_ch = fake<int32_t>(); f.gamma = f.beta = f.W = f.b = fake<float>(); f.s_log = 1.f;
    f.s_tilde = fake<float>(); f.z_tilde = fake<int32_t>(); f.gamma_t = f.beta_t = f.W_t = f.b_t = fake<float>();
    EXPECT(rq_reparam_fold(ctx, &f) == RQ_ERR_UNSUPPORTED);
    f.D = 0; EXPECT(rq_reparam_fold(ctx, &f) == RQ_ERR_SHAPE);
    f.D = INT32_MAX; f.D_out = INT32_MAX; EXPECT(rq_reparam_fold(ctx, &f) != RQ_OK || true);
    rq_wq_desc w{};
    EXPECT(rq_weight_quant_pack(ctx, &w) != RQ_OK);
    EXPECT(rq_weight_quant_pack(ctx, nullptr) == RQ_ERR_INVALID_ARG);
    rq_dual_clip_desc c{};
    EXPECT(rq_dual_clip_learn(ctx, &c) != RQ_OK);
    EXPECT(rq_dual_clip_learn(ctx, nullptr) == RQ_ERR_INVALID_ARG);
    rq_gptq_desc g{};
    EXPECT(rq_gptq_quant_pack(ctx, &g) != RQ_OK);
    EXPECT(rq_gptq_quant_pack(ctx, nullptr) == RQ_ERR_INVALID_ARG);
  }
}

static void check_block_plans(rq_ctx* ctx) {
  const int shapes[][5] = {{384, 6, 1536, 8, 197}, {768, 12, 3072, 64, 197}, {128, 4, 512, 4096, 49}, {4096, 32, 11008, 1, 2048},
                           {1024, 16, 4096, 128, 257}, {64, 1, 64, 1, 1}, {512, 4, 1024, 1, 4096}};
  for (const auto& s : shapes)
    for (int path = 0; path <= 2; ++path)
      for (int64_t chunk : {int64_t{0}, int64_t{1} << 20, int64_t{1} << 34}) {
        rq_block_params p = block_params(s[0], s[1], s[2]);
        p.attn_path = path; p.attn_chunk_bytes = chunk;
        rq_block_layout lay{};
        EXPECT(rq_block_workspace_layout(&p, s[3], s[4], &lay) == RQ_OK);
        const size_t need = rq_block_workspace_bytes(&p, s[3], s[4]);
        EXPECT(need == lay.total && need > 0);
        EXPECT(lay.batch_chunk >= 1 && lay.batch_chunk <= s[3]);
        EXPECT(lay.a < lay.total && lay.qkv < lay.total && lay.o < lay.total && lay.xbar < lay.total && lay.hidden < lay.total);
        EXPECT(lay.logits + lay.logits_bytes <= lay.total && lay.codes + lay.codes_bytes <= lay.total);
        // a valid forward call gets as far as the host-only refusal; a workspace one byte short is refused for that
        const rq_status st = rq_block_forward(ctx, &p, fake<float>(), fake<float>(), s[3], s[4], fake<void>(), need);
        if (st != RQ_ERR_UNSUPPORTED) std::printf("shape %d %d %d %d %d path %d: status %d: %s\n", s[0], s[1], s[2], s[3], s[4], path, (int)st, rq_last_error(ctx));
        EXPECT(st == RQ_ERR_UNSUPPORTED);
        EXPECT(rq_block_forward(ctx, &p, fake<float>(), fake<float>(), s[3], s[4], fake<void>(), need - 1) == RQ_ERR_WORKSPACE);
        rq_block_raw raw{};
        raw.D = s[0]; raw.H = s[1]; raw.Dm = s[2]; raw.attn_chunk_bytes = chunk;
        rq_block_layout cal{};
        EXPECT(rq_block_calibrate_workspace_layout(&raw, s[3], s[4], &cal) == RQ_OK);
        EXPECT(cal.logits_bytes > 0 && cal.codes_bytes > 0 && cal.codes >= cal.logits + cal.logits_bytes);
        EXPECT(rq_block_calibrate_workspace_bytes(&raw, s[3], s[4]) >= cal.total);
      }
  rq_block_params p = block_params(512, 4, 1024);      // rows beyond the block's limit
  EXPECT(rq_block_forward(ctx, &p, fake<float>(), fake<float>(), 1, 65536, fake<void>(), size_t{1} << 40) == RQ_ERR_SHAPE);
  p = block_params(384, 6, 1536);
  EXPECT(rq_block_workspace_bytes(nullptr, 1, 8) == 0 && rq_block_workspace_bytes(&p, 0, 8) == 0 && rq_block_workspace_bytes(&p, 1, -3) == 0);
  p.attn_path = 7;
  EXPECT(rq_block_forward(ctx, &p, fake<float>(), fake<float>(), 1, 8, fake<void>(), size_t{1} << 30) == RQ_ERR_INVALID_ARG);
  p = block_params(384, 6, 1536); p.attn_chunk_bytes = 5;
  EXPECT(rq_block_forward(ctx, &p, fake<float>(), fake<float>(), 1, 8, fake<void>(), size_t{1} << 30) == RQ_ERR_INVALID_ARG);
  p = block_params(384, 6, 1536); p.qkv.N = 100;
  EXPECT(rq_block_forward(ctx, &p, fake<float>(), fake<float>(), 1, 8, fake<void>(), size_t{1} << 30) == RQ_ERR_SHAPE);
  p = block_params(384, 5, 1536);      // D not a multiple of H
  EXPECT(rq_block_forward(ctx, &p, fake<float>(), fake<float>(), 1, 8, fake<void>(), size_t{1} << 30) != RQ_OK);
  // the no-allocation entry point: host-only contexts have no scratch
  p = block_params(384, 6, 1536);
  EXPECT(rq_block_noalloc_scratch_bytes() == RQ_NOALLOC_SCRATCH_BYTES);
  EXPECT(rq_block_forward_noalloc(ctx, &p, fake<float>(), fake<float>(), 1, 8) != RQ_OK);
  EXPECT(rq_block_forward_noalloc(nullptr, &p, fake<float>(), fake<float>(), 1, 8) == RQ_ERR_INVALID_ARG);
}

static void check_blob(rq_ctx* ctx) {
  rq_block_params p = block_params(64, 2, 128);
  const size_t n = rq_block_blob_bytes(&p, 0);
  EXPECT(n > sizeof(rq_blob_header));
  std::vector<unsigned char> blob(n);      // exactly n bytes: a read past the end is a sanitizer report
  EXPECT(rq_block_blob_save(ctx, &p, 0, blob.data(), n - 1) == RQ_ERR_WORKSPACE);
  EXPECT(rq_block_blob_save(ctx, &p, 0, blob.data(), n) == RQ_ERR_UNSUPPORTED);      // host-only: header not written either
  // a well-formed image, built through the public header struct
  rq_blob_header h{};
  std::memcpy(h.magic, "RQBLOCK", 8);
  h.header_bytes = sizeof h; h.version = RQ_BLOB_VERSION; h.D = 64; h.H = 2; h.Dm = 128; h.bits_a = h.bits_p = 4; h.eps = 1e-6;
  const int lin[4][2] = {{192, 64}, {64, 64}, {128, 64}, {64, 128}};
  uint64_t o = (sizeof h + 255) / 256 * 256;
  auto put = [&](int i, uint64_t len) { h.off[i] = o; h.len[i] = len; o += (len + 255) / 256 * 256; };
  for (int i = 0; i < 4; ++i) put(i, 64 * 4);
  for (int k = 0; k < 4; ++k) {
    h.lin[k][0] = lin[k][0]; h.lin[k][1] = lin[k][1]; h.lin[k][2] = 4; h.lin[k][3] = RQ_W_U4;
    put(4 + 5 * k, (uint64_t)lin[k][0] * lin[k][1] / 2);
    for (int j = 1; j < 5; ++j) put(4 + 5 * k + j, (uint64_t)lin[k][0] * 4);
  }
  h.total_bytes = o;
  EXPECT(o == n);
  std::memcpy(blob.data(), &h, sizeof h);
  size_t arena = 0;
  EXPECT(rq_block_blob_check(blob.data(), n, &arena) == RQ_OK && arena == n);
  EXPECT(rq_block_blob_check(blob.data(), n, nullptr) == RQ_OK);
  EXPECT(rq_block_blob_check(nullptr, n, &arena) == RQ_ERR_INVALID_ARG);
  rq_block_params out{};
  EXPECT(rq_block_blob_load(ctx, blob.data(), n, fake<void>(), n, &out) == RQ_ERR_UNSUPPORTED);
  EXPECT(rq_block_blob_load(ctx, blob.data(), n, fake<void>(), n - 1, &out) == RQ_ERR_WORKSPACE);
  for (size_t cut : {size_t{0}, size_t{1}, sizeof h - 1, sizeof h, n - 1}) {
    std::vector<unsigned char> part(blob.begin(), blob.begin() + cut);
    EXPECT(rq_block_blob_check(part.data(), cut, &arena) != RQ_OK);
  }
  // damaged headers: every 8-byte word of the header replaced by a few hostile values, then random byte flips; the checker
  // must answer (anything but a crash or an out-of-bounds read), and whatever it accepts must stay inside the buffer
  const uint64_t hostile[] = {0, 1, 255, 256, n, n + 1, UINT64_MAX, uint64_t{1} << 63, uint64_t{1} << 40, 0x8000000080000000ull};
  for (size_t w = 0; w + 8 <= sizeof h; w += 8)
    for (uint64_t v : hostile) {
      std::vector<unsigned char> bad(blob);
      std::memcpy(bad.data() + w, &v, 8);
      const rq_status st = rq_block_blob_check(bad.data(), n, &arena);
      if (st == RQ_OK) EXPECT(arena <= n);
    }
  uint64_t lcg = 12345;
  for (int it = 0; it < 4000; ++it) {
    std::vector<unsigned char> bad(blob);
    for (int k = 0; k < 3; ++k) {
      lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
      bad[(lcg >> 33) % sizeof h] ^= (unsigned char)(1u << ((lcg >> 20) & 7));
    }
    const rq_status st = rq_block_blob_check(bad.data(), n, &arena);
    if (st == RQ_OK) {
      EXPECT(arena <= n);
      EXPECT(rq_block_blob_load(ctx, bad.data(), n, fake<void>(), n, &out) == RQ_ERR_UNSUPPORTED);
    }
  }
}

int main() {
  rq_ctx* ctx = nullptr;
  if (rq_create(&ctx, -1, nullptr) != RQ_OK || !ctx) {
    std::printf("FAILED: no host-only context: %s\n", rq_last_error(nullptr));
    return 2;
  }
  EXPECT(rq_create(nullptr, -1, nullptr) == RQ_ERR_INVALID_ARG);
  check_entry_points(ctx);
  check_block_plans(ctx);
  check_blob(ctx);
  EXPECT(g_stub_launches == 0);
  rq_destroy(ctx);
  rq_destroy(nullptr);
  std::printf("%s: %d failed expectations, %d launches\n", g_fail ? "FAILED" : "OK", g_fail, g_stub_launches);
  return g_fail ? 1 : 0;
}
