// Pipelined weight-mode GEMM, int8 weight storage (RQ_W_I8_BAKED, RQ_W_I8_CENTERED): instantiations.
#include "qgemm_pipe.h"

rq_status rq_launch_qgemm_pipe_i8(rq_ctx* ctx, rqg::GemmParams& p) { return rqg::launch_pipe<false, 3>(ctx, p); }
