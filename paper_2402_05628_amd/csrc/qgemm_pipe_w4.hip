// Pipelined weight-mode GEMM, packed 4-bit weights (RQ_W_U4): instantiations.
#include "qgemm_pipe.h"

rq_status rq_launch_qgemm_pipe_w4(rq_ctx* ctx, rqg::GemmParams& p) { return rqg::launch_pipe<true, 4>(ctx, p); }
