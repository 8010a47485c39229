// Per-channel dual-clipping learner (Section "Per-channel dual clipping": Eqs. for X'_up, X'_low and the arg-min Eq.;
// Section "Implementation details": Adam, 100 iterations, learning rate 0.01).
//
// The objective is a sum over channels and Adam updates every parameter on its own, so the D channels are D separate
// two-parameter problems.  One workgroup owns one channel for the whole optimization: it reads its column of the
// activation ONCE, keeps X' in registers as float64 (up to RPT rows per lane; rows beyond that are re-read and
// re-normalized every pass), and runs all passes with one barrier each.  Every pass takes five sums over the tokens --
//   loss = sum e^2,  A = sum e (q - z),  C = sum e,  Cin = sum_in e,  Dx = sum_in e x'      (e = x^ - x')
// -- from which every lane derives the same straight-through gradient
//   dL/ds = 2 (A + (lo Cin - Dx)/s - lo C/s),  dL/dlo|_s = 2 (C - Cin),  s = (up - lo)/qmax,
//   dL/dalpha1 = dL/ds / qmax * max * sig'(alpha1),   dL/dalpha2 = (dL/dlo|_s - dL/ds / qmax) * min * sig'(alpha2)
// and the same Adam step.  All arithmetic is float64: the vector ALUs run it at half the float32 rate and the result
// then differs from a float64 reference only through the order of the sums.
#include <cfloat>
#include <cmath>

#include "rq_internal.h"

namespace {

constexpr int NSUM = 5;

// mean and 1/sqrt(var + eps) of every row (float64), one wavefront per row
__global__ __launch_bounds__(256) void row_stats_kernel(const float* __restrict__ x, int64_t T, int D, int64_t ldx, int norm_kind,
                                                        double eps, double* __restrict__ stats) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T) return;
  const float* xr = x + row * ldx;
  double s1 = 0.0, s2 = 0.0;
  for (int c = lane; c < D / 4; c += 64) {
    const float4 v = *reinterpret_cast<const float4*>(xr + c * 4);
    const double a = v.x, b = v.y, cc = v.z, dd = v.w;
    s1 += (a + b) + (cc + dd);
    s2 = fma(a, a, s2); s2 = fma(b, b, s2); s2 = fma(cc, cc, s2); s2 = fma(dd, dd, s2);
  }
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) { s1 += __shfl_xor(s1, m, 64); s2 += __shfl_xor(s2, m, 64); }
  double mean = 0.0, var;
  if (norm_kind == RQ_NORM_LAYERNORM) {
    mean = s1 / (double)D;
    var = fma(-mean, mean, s2 / (double)D);
    var = var < 0.0 ? 0.0 : var;
  } else {
    var = s2 / (double)D;
  }
  if (lane == 0) {
    stats[2 * row] = mean;
    stats[2 * row + 1] = 1.0 / sqrt(var + eps);
  }
}

struct ChannelState {          // identical in every lane of the workgroup
  double s, inv_s, z, lo, qmax;
};

struct Sums { double v[NSUM]; };

// one token of the channel: quantize, de-quantize, accumulate the five sums
__device__ __forceinline__ void accumulate(double xp, const ChannelState& c, Sums& a) {
  double u = xp * c.inv_s;
  double r = rint(u);
  // x'/s is what the quantizer rounds; the product with 1/s differs from it by an ulp or two, which matters only next
  // to a tie (or for quotients so large that an ulp is no longer tiny): those take the exact division
  if (fabs(fabs(u - r) - 0.5) < 1e-6 || !(fabs(u) < 1048576.0)) r = rint(xp / c.s);
  const double v = r + c.z;
  const bool in = v >= 0.0 && v <= c.qmax;
  const double q = fmin(fmax(v, 0.0), c.qmax);
  const double d = q - c.z;
  const double e = c.s * d - xp;
  const double ein = in ? e : 0.0;
  a.v[0] = fma(e, e, a.v[0]);
  a.v[1] = fma(e, d, a.v[1]);
  a.v[2] += e;
  a.v[3] += ein;
  a.v[4] = fma(ein, xp, a.v[4]);
}

struct LearnParams {
  const float* x; int64_t T; int64_t ldx; int D;
  const double* stats;        // mean, rstd per row, or NULL when x already is X'
  const float* gamma; const float* beta;
  int bits, iters; double lr, alpha0;
  double* alpha1; double* alpha2; float* clip_up; float* clip_lo; double* loss0; double* loss; double* up; double* lo;
};

template <int RPT>
__global__ __launch_bounds__(1024) void dual_clip_kernel(const LearnParams p) {
  __shared__ double part[2][16][NSUM];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nthreads = blockDim.x, nwaves = nthreads >> 6;
  // workgroups b, b + 8, ... share an XCD and its L2: give them neighbouring channels, whose columns share cache lines
  const int per_xcd = (p.D + 7) / 8;
  const int ch = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (ch >= p.D) return;
  const double g = p.gamma ? (double)p.gamma[ch] : 1.0, b = (p.gamma && p.beta) ? (double)p.beta[ch] : 0.0;
  auto fetch = [&](int64_t row) {
    const double xv = (double)p.x[row * p.ldx + ch];
    if (!p.stats) return xv;
    return (xv - p.stats[2 * row]) * p.stats[2 * row + 1] * g + b;
  };
  // ---- this lane's rows: tid, tid + nthreads, ...; the first RPT of them stay in registers ----
  double xp[RPT];
  double mn = DBL_MAX, mx = -DBL_MAX;
#pragma unroll
  for (int r = 0; r < RPT; ++r) {
    const int64_t row = (int64_t)r * nthreads + tid;
    xp[r] = 0.0;
    if (row < p.T) {
      xp[r] = fetch(row);
      mn = fmin(mn, xp[r]);
      mx = fmax(mx, xp[r]);
    }
  }
  const int64_t first_extra = (int64_t)RPT * nthreads + tid;
  for (int64_t row = first_extra; row < p.T; row += nthreads) {
    const double v = fetch(row);
    mn = fmin(mn, v);
    mx = fmax(mx, v);
  }
  const int64_t mine = p.T > tid ? (p.T - tid + nthreads - 1) / nthreads : 0;      // rows this lane owns
  const int held = mine < RPT ? (int)mine : RPT;
  // ---- channel extremes ----
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) { mn = fmin(mn, __shfl_xor(mn, m, 64)); mx = fmax(mx, __shfl_xor(mx, m, 64)); }
  if (lane == 0) { part[0][wave][0] = mn; part[0][wave][1] = mx; }
  __syncthreads();
  mn = part[0][0][0]; mx = part[0][0][1];
  for (int w = 1; w < nwaves; ++w) { mn = fmin(mn, part[0][w][0]); mx = fmax(mx, part[0][w][1]); }
  __syncthreads();
  const double qmax = (double)((1 << p.bits) - 1);
  double a1 = p.alpha0, a2 = p.alpha0, m1 = 0.0, v1 = 0.0, m2 = 0.0, v2 = 0.0, pb1 = 1.0, pb2 = 1.0;
  constexpr double B1 = 0.9, B2 = 0.999, ADAM_EPS = 1e-8;
  double loss_first = 0.0, loss_last = 0.0;
  const bool live = mx > mn;                            // a constant channel has s = 0: nothing to learn
  for (int pass = 0; live && pass <= p.iters; ++pass) {
    const double sg1 = 1.0 / (1.0 + exp(-a1)), sg2 = 1.0 / (1.0 + exp(-a2));
    const double up = mx * sg1, lo = mn * sg2;
    ChannelState c;
    c.s = (up - lo) / qmax;
    c.inv_s = 1.0 / c.s;
    c.z = rint(-lo / c.s);
    c.lo = lo;
    c.qmax = qmax;
    Sums acc;
#pragma unroll
    for (int i = 0; i < NSUM; ++i) acc.v[i] = 0.0;
#pragma unroll
    for (int r = 0; r < RPT; ++r)
      if (r < held) accumulate(xp[r], c, acc);
    for (int64_t row = first_extra; row < p.T; row += nthreads) accumulate(fetch(row), c, acc);
    // ---- the five sums over the workgroup; every lane adds the wavefronts' parts in the same order ----
#pragma unroll
    for (int i = 0; i < NSUM; ++i)
#pragma unroll
      for (int m = 1; m < 64; m <<= 1) acc.v[i] += __shfl_xor(acc.v[i], m, 64);
    double (*buf)[NSUM] = part[pass & 1];
    if (lane == 0)
#pragma unroll
      for (int i = 0; i < NSUM; ++i) buf[wave][i] = acc.v[i];
    __syncthreads();                                    // the other buffer is free again after the next pass's barrier
    double t[NSUM];
#pragma unroll
    for (int i = 0; i < NSUM; ++i) t[i] = buf[0][i];
    for (int w = 1; w < nwaves; ++w)
#pragma unroll
      for (int i = 0; i < NSUM; ++i) t[i] += buf[w][i];
    if (pass == 0) loss_first = t[0];
    loss_last = t[0];
    if (pass == p.iters) break;
    // ---- gradient and Adam step (the same in every lane) ----
    const double dL_ds = 2.0 * (t[1] + (lo * t[3] - t[4]) / c.s - lo / c.s * t[2]);
    const double dL_dlo = 2.0 * (t[2] - t[3]);
    const double g1 = dL_ds / qmax * mx * sg1 * (1.0 - sg1);
    const double g2 = (dL_dlo - dL_ds / qmax) * mn * sg2 * (1.0 - sg2);
    pb1 *= B1;
    pb2 *= B2;
    m1 = B1 * m1 + (1.0 - B1) * g1;
    v1 = B2 * v1 + (1.0 - B2) * g1 * g1;
    m2 = B1 * m2 + (1.0 - B1) * g2;
    v2 = B2 * v2 + (1.0 - B2) * g2 * g2;
    a1 -= p.lr * (m1 / (1.0 - pb1)) / (sqrt(v1 / (1.0 - pb2)) + ADAM_EPS);
    a2 -= p.lr * (m2 / (1.0 - pb1)) / (sqrt(v2 / (1.0 - pb2)) + ADAM_EPS);
  }
  if (tid == 0) {
    const double sg1 = 1.0 / (1.0 + exp(-a1)), sg2 = 1.0 / (1.0 + exp(-a2));
    p.alpha1[ch] = a1;
    p.alpha2[ch] = a2;
    if (p.clip_up) p.clip_up[ch] = (float)sg1;
    if (p.clip_lo) p.clip_lo[ch] = (float)sg2;
    if (p.up) p.up[ch] = mx * sg1;
    if (p.lo) p.lo[ch] = mn * sg2;
    if (p.loss0) p.loss0[ch] = loss_first;
    if (p.loss) p.loss[ch] = loss_last;
  }
}

// Wavefronts per workgroup: every workgroup is one channel, a compute unit holds 16 wavefronts of this kernel (128
// registers each), so nw wavefronts per channel give floor(16 / nw) channels per compute unit at a time; the time of a
// round is the number of rows per lane.  Rows beyond `max_rpt` per lane are re-read every pass: priced three times.
int choose_waves(int64_t T, int D, int num_cu, int max_rpt) {
  int best = 16;
  double best_cost = 1e300;
  for (int nw = 1; nw <= 16; ++nw) {
    const int64_t rpt = (T + 64 * nw - 1) / (64 * nw);
    const double rows = rpt <= max_rpt ? (double)rpt : max_rpt + 3.0 * (double)(rpt - max_rpt);
    const int64_t slots = (int64_t)num_cu * (16 / nw);
    const double rounds = (double)((D + slots - 1) / slots);
    const double cost = rounds * (rows + 4.0);           // + the per-pass reduction and update
    if (cost < best_cost * 0.999) { best_cost = cost; best = nw; }
  }
  return best;
}

}  // namespace

size_t rq_dual_clip_workspace_bytes(int64_t T) { return T > 0 ? (size_t)T * 2 * sizeof(double) : 0; }

rq_status rq_launch_dual_clip(rq_ctx* ctx, const rq_dual_clip_desc* d) {
  LearnParams p;
  p.x = d->x; p.T = d->T; p.ldx = d->ldx; p.D = d->D;
  p.stats = nullptr;
  p.gamma = d->gamma; p.beta = d->beta;
  p.bits = d->bits; p.iters = d->iters; p.lr = d->lr; p.alpha0 = d->alpha0;
  p.alpha1 = d->alpha1; p.alpha2 = d->alpha2; p.clip_up = d->clip_up; p.clip_lo = d->clip_lo;
  p.loss0 = d->loss0; p.loss = d->loss; p.up = d->up; p.lo = d->lo;
  if (d->gamma) {
    double* stats = static_cast<double*>(d->workspace);
    hipLaunchKernelGGL(row_stats_kernel, dim3((unsigned)((d->T + 3) / 4)), dim3(256), 0, ctx->stream, d->x, d->T, d->D, d->ldx,
                       d->norm_kind, d->eps, stats);
    p.stats = stats;
  }
  constexpr int MAX_RPT = 24;           // 2 registers per held row; more would spill under the 128-register bound
  const int nw = choose_waves(d->T, d->D, ctx->num_cu, MAX_RPT);
  const int64_t rpt = (d->T + 64 * nw - 1) / (64 * nw);
  const dim3 grid((unsigned)(8 * ((d->D + 7) / 8))), block(64 * nw);
  if (rpt <= 8) hipLaunchKernelGGL(dual_clip_kernel<8>, grid, block, 0, ctx->stream, p);
  else if (rpt <= 16) hipLaunchKernelGGL(dual_clip_kernel<16>, grid, block, 0, ctx->stream, p);
  else hipLaunchKernelGGL(dual_clip_kernel<MAX_RPT>, grid, block, 0, ctx->stream, p);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}
