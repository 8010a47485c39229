// rq_qgemm, weight mode: C[m, n] = sum_k (qa[m, k] - z_a)(qw[n, k] - z_w[n]) on the int8 matrix cores,
// with the de-quantize / activation / residual / re-quantize epilogue fused in
// (Section "Transformer blocks", last paragraph; de-quantizer of Section "Efficient quantizers").
//
// Tiling (CDNA4, 64-wide wavefronts): a workgroup of 4 wavefronts owns a BM x BN output tile and walks K
// in steps of 64 through a double-buffered LDS stage.  The weights are the ROW operand of
// v_mfma_i32_32x32x32_i8 and the activations the COLUMN operand, so each lane ends up with 4 consecutive
// output channels of one token: the epilogue reads scale/bias as 16-byte LDS vectors and writes float4
// or 4 packed codes per lane.  LDS rows are 64 B; their four 16-byte chunks are XOR-swizzled over a
// 128-byte line pair so that both the 16-byte stores and the MFMA operand loads spread over all banks.
// 4-bit weights travel packed (two codes per byte) from HBM/L2 into registers and are unpacked nibble-wise,
// zero-point subtracted, on their way into LDS: the MFMA loop is the same for every weight format.
// The rank-1 zero-point corrections are folded into the accumulator's initial value.
#include "qgemm_common.h"

rq_status rq_launch_qgemm_pipe_w4(rq_ctx* ctx, rqg::GemmParams& p);
bool rq_qgemv_applies(const rqg::GemmParams& p, bool w4);
rq_status rq_launch_qgemv_w4(rq_ctx* ctx, const rqg::GemmParams& p);
rq_status rq_launch_qgemm_pipe_i8(rq_ctx* ctx, rqg::GemmParams& p);

namespace {

using namespace rqg;

template <int BM, int BN, bool W4>
__global__ __launch_bounds__(256, 2) void qgemm_kernel(const GemmParams p) {
  constexpr int WM = BM / 2, WN = BN / 2;        // wavefront tile
  constexpr int TM = WM / 32, TN = WN / 32;      // MFMA tiles per wavefront
  constexpr int A_BYTES = BM * 64, B_BYTES = BN * 64;
  constexpr int A_IT = BM * 4 / 256;             // 16-byte chunks per thread per stage
  constexpr int B_IT = W4 ? (BN * 2 / 256) : (BN * 4 / 256);
  __shared__ __align__(16) int8_t lds[2 * (A_BYTES + B_BYTES)];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int tile_n = blockIdx.x % p.tiles_n;
  const int tile_m = blockIdx.x / p.tiles_n;
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = tile_n * BN;
  const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

  // global -> register staging pointers
  const int8_t* aptr[A_IT];
  int a_lds[A_IT];
#pragma unroll
  for (int i = 0; i < A_IT; ++i) {
    const int id = tid + 256 * i;
    const int row = id >> 2, c = id & 3;
    int64_t m = m0 + row;
    m = m < p.M ? m : p.M - 1;
    aptr[i] = p.A + m * p.lda + c * 16;
    a_lds[i] = swz(row, c);
  }
  const uint8_t* bptr[B_IT];
  int b_lds[B_IT];
  int zb4[B_IT];
#pragma unroll
  for (int i = 0; i < B_IT; ++i) {
    const int id = tid + 256 * i;
    if (W4) {
      const int row = id >> 1, pc = id & 1;
      int n = n0 + row;
      n = n < p.N ? n : p.N - 1;
      bptr[i] = p.B + (int64_t)n * p.ldb + pc * 16;
      b_lds[i] = row * 8 + pc;   // decoded below (two chunks)
      zb4[i] = p.z_b[n] * 0x01010101;
    } else {
      const int row = id >> 2, c = id & 3;
      int n = n0 + row;
      n = n < p.N ? n : p.N - 1;
      bptr[i] = p.B + (int64_t)n * p.ldb + c * 16;
      b_lds[i] = swz(row, c);
      zb4[i] = 0;
    }
  }

  v4i ra[A_IT], rb[B_IT];
  auto gload = [&](int kt) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) ra[i] = *reinterpret_cast<const v4i*>(aptr[i] + (int64_t)kt * 64);
#pragma unroll
    for (int i = 0; i < B_IT; ++i) rb[i] = *reinterpret_cast<const v4i*>(bptr[i] + (int64_t)kt * (W4 ? 32 : 64));
  };
  auto lstore = [&](int buf) {
    int8_t* la = lds + buf * (A_BYTES + B_BYTES);
    int8_t* lb = la + A_BYTES;
#pragma unroll
    for (int i = 0; i < A_IT; ++i) *reinterpret_cast<v4i*>(la + a_lds[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
      if (W4) {
        const int row = b_lds[i] >> 3, pc = b_lds[i] & 1;
        v4i c0, c1;
        unpack_u4(rb[i], zb4[i], c0, c1);
        *reinterpret_cast<v4i*>(lb + swz(row, 2 * pc)) = c0;
        *reinterpret_cast<v4i*>(lb + swz(row, 2 * pc + 1)) = c1;
      } else {
        *reinterpret_cast<v4i*>(lb + b_lds[i]) = rb[i];
      }
    }
  };

  v16i acc[TN][TM];
  init_acc<TM, TN>(p, acc, m0, n0, wm0, wn0, lane);

  const int nk = p.K / 64;
  gload(0);
  lstore(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) gload(kt + 1);
    const int8_t* la = lds + buf * (A_BYTES + B_BYTES);
    const int8_t* lb = la + A_BYTES;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int c = s * 2 + (lane >> 5);
      v4i fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const v4i*>(la + swz(wm0 + i * 32 + (lane & 31), c));
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const v4i*>(lb + swz(wn0 + j * 32 + (lane & 31), c));
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
          acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[j], fa[i], acc[j][i], 0, 0, 0);
    }
    if (kt + 1 < nk) lstore(buf ^ 1);
    __syncthreads();
  }

  epilogue<TM, TN>(p, acc, m0, n0, wm0, wn0, lane);
}

template <int BM, int BN, bool W4>
void launch_tile(rq_ctx* ctx, GemmParams& p) {
  const int64_t tiles_m = (p.M + BM - 1) / BM;
  p.tiles_m = (int)tiles_m;
  p.tiles_n = (p.N + BN - 1) / BN;
  hipLaunchKernelGGL((qgemm_kernel<BM, BN, W4>), dim3((unsigned)(tiles_m * p.tiles_n)), dim3(256), 0, ctx->stream, p);
}

}  // namespace

// ctx->gemm_tile: 0: choose by shape, 1: 128x128 simple, 2: 256x128 simple, 3: pipelined; 4 .. 7: pipelined with 320- / 192- /
// 128- / 256-row tiles where they exist; 8: 256 x 256 tiles
extern "C" rq_status rq_set_gemm_tile(rq_ctx* ctx, int32_t tile) {
  if (!ctx) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_set_gemm_tile: ctx is NULL");
  RQ_REQUIRE(tile >= 0 && (tile & 0xFF) <= 8 && (tile & ~0x3FF) == 0 && (tile >> 8) != 3, RQ_ERR_INVALID_ARG,
             "rq_set_gemm_tile: %d not in 0..8 (+ 256 or + 512)", tile);
  ctx->gemm_tile = tile & 0xFF;
  ctx->gemm_no_raw = (tile >> 8) == 1 ? 1 : ((tile >> 8) == 2 ? -1 : 0);
  return RQ_OK;
}

rq_status rq_launch_qgemm_weight(rq_ctx* ctx, const rq_gemm_desc* d) {
  GemmParams p;
  const int g_gemm_tile = ctx->gemm_tile;
  p.M = d->M; p.N = d->N; p.K = d->K;
  p.A = d->A; p.lda = d->lda;
  p.B = static_cast<const uint8_t*>(d->B); p.ldb = d->ldb;
  p.s_b = d->s_b; p.z_b = d->z_b; p.colsum_b = d->colsum_b; p.rowsum_a = d->rowsum_a; p.bias = d->bias;
  p.s_a = d->s_a; p.da = d->a_off - d->z_a; p.centered = d->b_format == RQ_W_I8_CENTERED;
  p.act = d->act; p.residual = d->residual; p.ldr = d->ldr;
  p.out_acc = d->out_acc; p.ldacc = d->ldacc; p.out_f32 = d->out_f32; p.ldf = d->ldf; p.out_q = d->out_q; p.ldq = d->ldq;
  p.n_seg = d->n_seg > 0 ? d->n_seg : 1; p.seg_len = d->seg_len > 0 ? d->seg_len : d->N;
  for (int i = 0; i < 4; ++i) {
    const bool on = d->out_q && i < p.n_seg;
    p.inv_so_d[i] = on ? 1.0 / (double)d->s_o[i] : 0.0;
    p.inv_so[i] = on ? 1.0f / d->s_o[i] : 0.f;
    p.zo[i] = on ? (float)(d->z_o[i] - d->off_o[i]) : 0.f;
    p.zcode[i] = on ? (float)d->z_o[i] : 0.f;
    p.off4[i] = on ? (int)((unsigned)(d->off_o[i] & 0xFF) * 0x01010101u) : 0;
    p.lo[i] = on ? -d->off_o[i] : 0;
    p.hi[i] = on ? (1 << d->bits_o) - 1 - d->off_o[i] : 0;
  }
  const bool w4 = d->b_format == RQ_W_U4;
  p.qmaxf = d->out_q ? (float)((1 << d->bits_o) - 1) : 0.f;
  // Tile choice: the larger tile halves LDS traffic per MAC; the smaller one fills the chip on narrow outputs.
  const int64_t big_tiles = ((d->M + 255) / 256) * ((d->N + 127) / 128);
  const bool big = g_gemm_tile ? g_gemm_tile == 2 : big_tiles >= 2 * (int64_t)ctx->num_cu;
  const bool fits32 = (double)d->M * (double)d->lda < 4.0e9 && (double)d->N * (double)d->ldb < 4.0e9;
  p.no_raw = ctx->gemm_no_raw;
  p.force_rows = g_gemm_tile == 4 ? 5 : (g_gemm_tile == 5 ? 3 : (g_gemm_tile == 6 ? 2 : (g_gemm_tile == 7 ? 4 : (g_gemm_tile == 8 ? 6 : 0))));
  if (g_gemm_tile == 0 && rq_qgemv_applies(p, w4)) return rq_launch_qgemv_w4(ctx, p);   // a few tokens: weight-bandwidth bound
  if ((g_gemm_tile == 3 || g_gemm_tile == 0 || g_gemm_tile >= 4) && d->N % 32 == 0 && fits32) {
    const rq_status st = w4 ? rq_launch_qgemm_pipe_w4(ctx, p) : rq_launch_qgemm_pipe_i8(ctx, p);
    if (st != RQ_OK) return st;
  } else if (big) {
    if (w4) launch_tile<256, 128, true>(ctx, p); else launch_tile<256, 128, false>(ctx, p);
  } else {
    if (w4) launch_tile<128, 128, true>(ctx, p); else launch_tile<128, 128, false>(ctx, p);
  }
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}
