// Stand-ins for the kernel launchers and shape predicates that live next to the kernels, so that the host layer of the
// library (argument validation, workspace plans, the parameter blob) links into a CPU-only, sanitizer-instrumented
// program.  Under a host-only context no entry point may get as far as a launcher: every stub counts the call and the
// check program fails if the count is not zero.
#include "rq_internal.h"

int g_stub_launches = 0;

#define RQ_STUB(...)     \
  {                      \
    ++g_stub_launches;   \
    return RQ_ERR_HIP;   \
  }

rq_status rq_launch_ln_quant(rq_ctx*, const rq_ln_desc*) RQ_STUB()
rq_status rq_launch_qgemm_weight(rq_ctx*, const rq_gemm_desc*) RQ_STUB()
rq_status rq_launch_qgemm_act(rq_ctx*, const rq_gemm_desc*) RQ_STUB()
rq_status rq_launch_softmax(rq_ctx*, const rq_softmax_desc*) RQ_STUB()
rq_status rq_launch_pv(rq_ctx*, const rq_pv_desc*) RQ_STUB()
rq_status rq_launch_qgemm_rowln(rq_ctx*, const rq_gemm_desc*, const rq_ln_desc*) RQ_STUB()
rq_status rq_launch_attn_fused(rq_ctx*, const rq_attn_fused_desc*) RQ_STUB()
rq_status rq_launch_qk_softmax(rq_ctx*, const int8_t*, const int8_t*, int64_t, int64_t, int, int, int, int, int, int, int, double,
                               const float*, int, float, int, uint8_t*, int64_t) RQ_STUB()
rq_status rq_launch_fold(rq_ctx*, const rq_fold_desc*) RQ_STUB()
rq_status rq_launch_weight_quant(rq_ctx*, const rq_wq_desc*) RQ_STUB()
rq_status rq_launch_rowsum(rq_ctx*, const int8_t*, int64_t, int32_t, int64_t, int32_t*) RQ_STUB()
rq_status rq_launch_ln_channel_minmax(rq_ctx*, const float*, int64_t, int32_t, int64_t, int32_t, double, const float*, const float*,
                                      double*, double*) RQ_STUB()
rq_status rq_launch_minmax_f32(rq_ctx*, const float*, int64_t, int64_t, int64_t, double*) RQ_STUB()
rq_status rq_launch_channel_qparams(rq_ctx*, const double*, const double*, const float*, const float*, int32_t, int32_t, float*,
                                    int32_t*) RQ_STUB()
rq_status rq_launch_ln_channel_percentile(rq_ctx*, const float*, int64_t, int32_t, int64_t, int32_t, double, const float*,
                                          const float*, double, double, double*, double*, void*) RQ_STUB()
rq_status rq_launch_gptq(rq_ctx*, const rq_gptq_desc*) RQ_STUB()
rq_status rq_launch_dual_clip(rq_ctx*, const rq_dual_clip_desc*) RQ_STUB()

// shape predicates: the plans only need consistent answers
bool rq_qk_softmax_supported(int N, int d_head, bool has_bias) {
  return (N <= 288 || (!has_bias && N <= 65536)) && (d_head == 32 || d_head == 64 || d_head == 128);
}
bool rq_attn_fused_preferred(int N, int, int bits_p, bool has_bias) { return N <= 256 && bits_p <= 4 && !has_bias; }
bool rq_qgemm_rowln_applies(const rq_gemm_desc*, const rq_ln_desc*) { return false; }
extern "C" int32_t rq_attn_fused_supported(int32_t N, int32_t, int32_t bits_p, int32_t has_bias) {
  return N > 0 && N <= 288 && bits_p <= 4 && !has_bias;
}
extern "C" size_t rq_dual_clip_workspace_bytes(int64_t T) { return T > 0 ? (size_t)T * 16 : 0; }
extern "C" size_t rq_gptq_workspace_bytes(int32_t N, int32_t K, int64_t T) {
  return N > 0 && K > 0 && T > 0 ? ((size_t)N * K + 4 * (size_t)K * K) * 8 : 0;
}
