// rq_qgemm, activation mode: batched Q.K^T on quantized codes, exact int32 accumulators out
// (attention Eq. of Section "Transformer blocks"; both operands quantized).
//
// The reduction length is one head (32..256 bytes), so the operands go straight from global memory into
// the MFMA operand layout (each lane owns 16 contiguous bytes of one row) with no LDS stage, and the
// kernel is bound by writing the [G, Nq, ld] int32 accumulators.  Keys are the ROW operand and queries
// the COLUMN operand, so a lane holds groups of 4 consecutive keys of one query row; a 32 x 32 tile is turned
// into whole 128-byte row segments through LDS before it is stored.
// Zero-point corrections: sum (q'+dq)(k'+dk) = sum q'k' + dk*rowsum(q') + dq*rowsum(k') + K*dq*dk; the two
// row sums come from two extra MFMAs against an all-ones operand.
#include "rq_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct QkParams {
  const int8_t* A;
  const int8_t* B;
  int64_t lda, ldb;
  int64_t a_so, a_si, b_so, b_si;
  int batch_inner;
  int Nq, Nk, K;
  int dq, dk;     // storage offset minus zero-point of Q and of K
  int32_t* acc;
  int64_t ldacc, acc_sg;
  int causal;
  int tiles_i;
  int64_t total_waves;
};

template <int KSTEPS>
__global__ __launch_bounds__(256) void qk_kernel(const QkParams p) {
  const int lane = threadIdx.x & 63;
  const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= p.total_waves) return;
  const int64_t g = w / p.tiles_i;
  int it = (int)(w % p.tiles_i);
  // With a causal mask query tile t has t + 1 key tiles to do: neighbouring wavefronts take tiles from the two ends
  // of the group in turn (0, T-1, 1, T-2, ...), so that every workgroup carries about the same amount of work.
  if (p.causal) it = (it & 1) ? p.tiles_i - 1 - (it >> 1) : (it >> 1);
  const int64_t go = g / p.batch_inner;
  const int gi = (int)(g % p.batch_inner);
  const int8_t* Q = p.A + go * p.a_so + gi * p.a_si;
  const int8_t* Kp = p.B + go * p.b_so + gi * p.b_si;
  int32_t* out = p.acc + g * p.acc_sg;

  constexpr int PITCH = 36;
  __shared__ int stage_all[4][32 * PITCH];
  int* const stage = stage_all[threadIdx.x >> 6];
  const int l32 = lane & 31, half = lane >> 5;
  const int rrow = lane >> 3, rcol = (lane & 7) * 4;         // read-back: 8 rows x 8 pieces of 16 bytes per pass
  int qi = it * 32 + l32;
  const int qi_ld = qi < p.Nq ? qi : p.Nq - 1;
  v4i fq[KSTEPS];
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) fq[s] = *reinterpret_cast<const v4i*>(Q + (int64_t)qi_ld * p.lda + s * 32 + half * 16);

  const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
  const bool corr = (p.dq != 0) || (p.dk != 0);
  v16i base;
#pragma unroll
  for (int e = 0; e < 16; ++e) base[e] = 0;
  if (corr) {
    v16i rq = base;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) rq = __builtin_amdgcn_mfma_i32_32x32x32_i8(ones, fq[s], rq, 0, 0, 0);
#pragma unroll
    for (int e = 0; e < 16; ++e) base[e] = p.dk * rq[e] + p.K * p.dq * p.dk;
  }

  int jt_end = (p.Nk + 31) / 32;
  if (p.causal) {
    const int lim = it + 1;   // keys j <= i only: tiles strictly above the diagonal are skipped
    jt_end = jt_end < lim ? jt_end : lim;
  }
  // the next key tile's operands are requested before this tile's products and stores: a group has few wavefronts
  // (one per 32 queries), so the latency of these loads is not hidden by other wavefronts
  v4i fk_next[KSTEPS];
  auto request = [&](int jt) {
    int kj = jt * 32 + l32;
    kj = kj < p.Nk ? kj : p.Nk - 1;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s)
      fk_next[s] = *reinterpret_cast<const v4i*>(Kp + (int64_t)kj * p.ldb + s * 32 + half * 16);
  };
  if (jt_end > 0) request(0);
  for (int jt = 0; jt < jt_end; ++jt) {
    v4i fk[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) fk[s] = fk_next[s];
    if (jt + 1 < jt_end) request(jt + 1);
    v16i acc = base;
    if (corr && p.dq != 0) {
      v16i ck;
#pragma unroll
      for (int e = 0; e < 16; ++e) ck[e] = 0;
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) ck = __builtin_amdgcn_mfma_i32_32x32x32_i8(fk[s], ones, ck, 0, 0, 0);
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] += p.dq * ck[e];
    }
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fk[s], fq[s], acc, 0, 0, 0);
    // A lane holds key columns 8 g + 4 half + e of its query row (g = 0..3): stored directly, every instruction would
    // send 64 separate 16-byte pieces of 32 rows to the L2.  The tile goes through this wavefront's own 4.5 KB of LDS
    // (row pitch 36 ints: conflict-free both ways) and leaves as whole 128-byte row segments, 8 lanes per row.
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const v4i t = {acc[4 * gq], acc[4 * gq + 1], acc[4 * gq + 2], acc[4 * gq + 3]};
      *reinterpret_cast<v4i*>(stage + l32 * PITCH + 8 * gq + half * 4) = t;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // this wavefront's own writes; no other wavefront touches `stage`
    const int j = jt * 32 + rcol;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = r * 8 + rrow;
      const v4i t = *reinterpret_cast<const v4i*>(stage + row * PITCH + rcol);
      const int q = it * 32 + row;
      if (q < p.Nq && j < p.ldacc) *reinterpret_cast<v4i*>(out + (int64_t)q * p.ldacc + j) = t;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // reads done before the next tile overwrites the region
  }
}

}  // namespace

rq_status rq_launch_qgemm_act(rq_ctx* ctx, const rq_gemm_desc* d) {
  QkParams p;
  p.A = d->A; p.B = static_cast<const int8_t*>(d->B);
  p.lda = d->lda; p.ldb = d->ldb;
  p.a_so = d->a_stride_outer; p.a_si = d->a_stride_inner; p.b_so = d->b_stride_outer; p.b_si = d->b_stride_inner;
  p.batch_inner = d->batch_inner;
  p.Nq = (int)d->M; p.Nk = d->N; p.K = d->K;
  p.dq = d->a_off - d->z_a; p.dk = d->b_off - d->z_b_scalar;
  p.acc = d->out_acc; p.ldacc = d->ldacc; p.acc_sg = d->acc_stride_group;
  p.causal = d->causal;
  p.tiles_i = (p.Nq + 31) / 32;
  p.total_waves = d->batch_outer * d->batch_inner * p.tiles_i;
  const unsigned blocks = (unsigned)((p.total_waves + 3) / 4);
  switch (d->K / 32) {
    case 1: hipLaunchKernelGGL(qk_kernel<1>, dim3(blocks), dim3(256), 0, ctx->stream, p); break;
    case 2: hipLaunchKernelGGL(qk_kernel<2>, dim3(blocks), dim3(256), 0, ctx->stream, p); break;
    case 4: hipLaunchKernelGGL(qk_kernel<4>, dim3(blocks), dim3(256), 0, ctx->stream, p); break;
    case 8: hipLaunchKernelGGL(qk_kernel<8>, dim3(blocks), dim3(256), 0, ctx->stream, p); break;
    default: return rq_fail(ctx, RQ_ERR_SHAPE, "rq_qgemm (activation mode): K = %d must be 32, 64, 128 or 256", d->K);
  }
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}
