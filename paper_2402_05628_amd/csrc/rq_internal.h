// Internal declarations shared by the translation units of librepquant.so (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include <mutex>
#include <string>
#include <vector>

#include "repquant.h"

struct rq_ctx {
  int device = -1;            // < 0: host-only (validation) context
  hipStream_t stream = nullptr;
  int num_cu = 256;
  int gemm_tile = 0;          // rq_set_gemm_tile: 0 = kernel and tile of the weight-mode GEMM chosen by shape
  int gemm_no_raw = 0;        // rq_set_gemm_tile + 256: packed 4-bit weights never take the raw-nibble variant (1); + 512: whenever row sums are given (-1)
  // rq_block_forward over two halves of the batch at once: a second stream of this context and the two events that fork it
  // from `stream` and join it again (created with the context).  block_streams: see rq_set_block_streams
  int block_streams = 1;
  hipStream_t stream2 = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  std::string err;
  // per-kernel profiling of rq_block_forward
  bool profiling = false;
  struct EvPair { hipEvent_t a, b; int step; };
  std::vector<EvPair>* pending = nullptr;
  std::vector<hipEvent_t>* pool = nullptr;
  double prof_ms[RQ_STEP_COUNT] = {0};
  int64_t prof_n[RQ_STEP_COUNT] = {0};
};

rq_status rq_fail(rq_ctx* ctx, rq_status st, const char* fmt, ...);

#define RQ_REQUIRE(cond, st, ...)                         \
  do {                                                    \
    if (!(cond)) return rq_fail(ctx, st, __VA_ARGS__);    \
  } while (0)

#define RQ_HIP(call)                                                                          \
  do {                                                                                        \
    hipError_t e__ = (call);                                                                  \
    if (e__ != hipSuccess)                                                                    \
      return rq_fail(ctx, RQ_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e__));        \
  } while (0)

// A kernel that takes more than 64 KB of dynamic LDS needs hipFuncAttributeMaxDynamicSharedMemorySize raised, once per
// device: `once` is a function-local static of the launcher (one per kernel instantiation) that remembers the devices done.
struct rq_once_per_device {
  std::mutex mu;
  uint64_t done[2] = {0, 0};   // devices 0..127
};
inline hipError_t rq_allow_dynamic_lds(const rq_ctx* ctx, rq_once_per_device& once, const void* kernel, int bytes) {
  const int dev = ctx->device;
  if (dev < 0 || dev >= 128) return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  std::lock_guard<std::mutex> lock(once.mu);
  if ((once.done[dev >> 6] >> (dev & 63)) & 1u) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) once.done[dev >> 6] |= 1ull << (dev & 63);
  return e;
}

static inline bool rq_aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Returns RQ_ERR_UNSUPPORTED for a host-only context (after validation has passed).
#define RQ_NEED_DEVICE()                                                                              \
  do {                                                                                                \
    if (ctx->device < 0) return rq_fail(ctx, RQ_ERR_UNSUPPORTED, "host-only context: no GPU work");   \
  } while (0)

// kernel launchers (defined next to their kernels); all arguments already validated
rq_status rq_launch_ln_quant(rq_ctx* ctx, const rq_ln_desc* d);
rq_status rq_launch_qgemm_weight(rq_ctx* ctx, const rq_gemm_desc* d);
rq_status rq_launch_qgemm_act(rq_ctx* ctx, const rq_gemm_desc* d);
rq_status rq_launch_softmax(rq_ctx* ctx, const rq_softmax_desc* d);
rq_status rq_launch_pv(rq_ctx* ctx, const rq_pv_desc* d);
bool rq_qk_softmax_supported(int N, int d_head, bool has_bias);
bool rq_attn_fused_preferred(int N, int d_head, int bits_p, bool has_bias);
bool rq_qgemm_rowln_applies(const rq_gemm_desc* g, const rq_ln_desc* ln);
rq_status rq_launch_qgemm_rowln(rq_ctx* ctx, const rq_gemm_desc* g, const rq_ln_desc* ln);
rq_status rq_launch_attn_fused(rq_ctx* ctx, const rq_attn_fused_desc* d);
rq_status rq_launch_qk_softmax(rq_ctx* ctx, const int8_t* Q, const int8_t* K, int64_t ld_tok, int64_t batch, int H, int N,
                               int d_head, int q_off, int z_q, int k_off, int z_k, double logit_scale, const float* bias,
                               int mask, float s_log, int bits, uint8_t* codes, int64_t ld);
rq_status rq_launch_fold(rq_ctx* ctx, const rq_fold_desc* d);
rq_status rq_launch_weight_quant(rq_ctx* ctx, const rq_wq_desc* d);
rq_status rq_launch_rowsum(rq_ctx* ctx, const int8_t* A, int64_t M, int32_t K, int64_t lda, int32_t* rowsum);
rq_status rq_launch_ln_channel_minmax(rq_ctx* ctx, const float* x, int64_t T, int32_t D, int64_t ldx, int32_t norm_kind,
                                      double eps, const float* gamma, const float* beta, double* cmin, double* cmax);
rq_status rq_launch_minmax_f32(rq_ctx* ctx, const float* v, int64_t rows, int64_t cols, int64_t ld, double* out2);

rq_status rq_launch_channel_qparams(rq_ctx* ctx, const double* cmin, const double* cmax, const float* clip_up,
                                    const float* clip_lo, int D, int bits, float* s_ch, int32_t* z_ch);

// mean and 1 / sqrt(var + eps) of every row, float64, interleaved: stats[2 * row], stats[2 * row + 1]
rq_status rq_launch_row_stats(rq_ctx* ctx, const float* x, int64_t T, int32_t D, int64_t ldx, int32_t norm_kind, double eps,
                              double* stats);
rq_status rq_launch_ln_channel_percentile(rq_ctx* ctx, const float* x, int64_t T, int32_t D, int64_t ldx, int32_t norm_kind,
                                          double eps, const float* gamma, const float* beta, double q_lo, double q_hi,
                                          double* lo, double* hi, void* workspace);
rq_status rq_launch_gptq(rq_ctx* ctx, const rq_gptq_desc* d);
rq_status rq_launch_dual_clip(rq_ctx* ctx, const rq_dual_clip_desc* d);

// resolves (once per device) the address of the fixed scratch array of rq_block_forward_noalloc; out may be NULL
rq_status rq_noalloc_scratch_init(rq_ctx* ctx, void** out);

// profiling hooks used by rq_block_forward
void rq_prof_begin(rq_ctx* ctx, int step);
void rq_prof_end(rq_ctx* ctx);

// ---- device helpers ---------------------------------------------------------------------------------
#ifdef __HIPCC__
__device__ __forceinline__ double rq_wave_sum_xor(double v, int width) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1)
    if (m < width) v += __shfl_xor(v, m, 64);
  return v;
}
// 0xFF in every byte of x that equals the matching byte of ref4, 0 elsewhere (any byte values)
__device__ __forceinline__ unsigned rq_byte_eq_mask(unsigned x, unsigned ref4) {
  const unsigned d = x ^ ref4;
  const unsigned nz = (((d & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | d) & 0x80808080u;   // 0x80 where the byte differs
  const unsigned z = nz ^ 0x80808080u;                                          // 0x80 where it is equal
  return (z << 1) - (z >> 7);
}
__device__ __forceinline__ int rq_pack4(int c0, int c1, int c2, int c3) {
  return (c0 & 0xFF) | ((c1 & 0xFF) << 8) | ((c2 & 0xFF) << 16) | (c3 << 24);
}
#endif
