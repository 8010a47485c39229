// Fused Q.K^T + Softmax-log2 kernels for d_head = 64: instantiations for 1..9 key tiles.
#include "qk_softmax.h"

rq_status rq_launch_qk_softmax_d64(rq_ctx* ctx, const rqks::QksParams& p, int64_t groups) { return rqks::launch_nt<2>(ctx, p, groups); }
