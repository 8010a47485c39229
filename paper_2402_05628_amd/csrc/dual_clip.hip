// Per-channel dual-clipping learner (Section "Per-channel dual clipping": Eqs. for X'_up, X'_low and the arg-min Eq.;
// Section "Implementation details": Adam, 100 iterations, learning rate 0.01).
//
// The objective is a sum over channels and Adam updates every parameter on its own, so the D channels are D separate
// two-parameter problems.  One workgroup owns one channel for the whole optimization: it reads its column of the
// activation ONCE, keeps X' as float64 (up to RPT rows per lane in registers, further rows in LDS; what still does not
// fit is re-read and re-normalized every pass), and runs all passes with two barriers each.  With u = x'/s, r = round(u), v = r + z,
// q = clip(v), d = q - z, e = s d - x' every pass takes three sums over the tokens,
//   L = sum e^2,   G = sum_{v inside} e (r - u) + sum_{v clipped} e d,   Cout = sum_{v clipped} e,
// which give the straight-through gradient (both roundings with derivative 1, the clip passing it on [0, qmax])
//   dL/ds = 2 (G - lo Cout / s),   dL/dlo at fixed s = 2 Cout,   s = (up - lo) / qmax,
//   dL/dalpha1 = dL/ds / qmax * max * sig'(alpha1),   dL/dalpha2 = (2 Cout - dL/ds / qmax) * min * sig'(alpha2).
// Wavefront 0 adds the wavefronts' parts in a fixed order, takes the Adam step and publishes the next pass's s, 1/s, z.
// All arithmetic is float64: the vector ALUs run it at half the float32 rate and the result then differs from a
// float64 reference only through the order of the sums.
#include <cfloat>
#include <cmath>

#include "rq_internal.h"

namespace {

constexpr int NSUM = 3;

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
  double s, inv_s, z, qmax;
  bool exact;                  // quotients too large for the reciprocal shortcut: divide every time
};

struct Sums { double v[NSUM]; };

// one token of the channel: quantize, de-quantize, accumulate the three sums
// (clipping on the int32 image of v and 0/1 factors instead of selects were tried: slower than this form)
__device__ __forceinline__ void accumulate(double xp, const ChannelState& c, Sums& a) {
  const double u = xp * c.inv_s;
  double r = rint(u);
  double w = r - u;
  // x'/s is what the quantizer rounds; the product with 1/s differs from it by an ulp or two, which can change the
  // rounded value only next to a tie: those (and channels whose quotients are huge) take the exact division
  if (fabs(fabs(w) - 0.5) < 1e-6 || c.exact) r = rint(xp / c.s);
  const double v = r + c.z;
  const double q = fmin(fmax(v, 0.0), c.qmax);
  const double d = q - c.z;
  const double e = c.s * d - xp;
  const bool in = q == v;                               // the clip passes the gradient on [0, qmax], end points included
  a.v[0] = fma(e, e, a.v[0]);
  a.v[1] = fma(e, in ? w : d, a.v[1]);
  a.v[2] += in ? 0.0 : e;
}

// sum over the 16 lanes of a DPP row (every lane of the row gets it)
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)b, CTRL, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xF, 0xF, true);
  return __longlong_as_double(((long long)hi << 32) | (unsigned)lo);
}
__device__ __forceinline__ double row_sum(double v) {
  v += dpp_f64<0xB1>(v);       // lane ^ 1
  v += dpp_f64<0x4E>(v);       // lane ^ 2
  v += dpp_f64<0x141>(v);      // row_half_mirror
  v += dpp_f64<0x140>(v);      // row_mirror
  return v;
}

struct LearnParams {
  const float* x; int64_t T; int64_t ldx; int D;
  const double* stats;        // mean, rstd per row, or NULL when x already is X'
  const float* gamma; const float* beta;
  int bits, iters; double lr, alpha0;
  double* alpha1; double* alpha2; float* clip_up; float* clip_lo; double* loss0; double* loss; double* up; double* lo;
};

// Learner state of one channel in LDS, touched by wavefront 0 only.  The two factors are updated side by side: even
// lanes carry alpha_1 (with the channel maximum), odd lanes alpha_2 (with the minimum), so one instruction stream
// takes both Sigmoids, both Adam steps and both bounds.
struct Factor { double a, m, v, sg; };                  // alpha, Adam moments, Sigmoid(alpha)
struct Learner {
  Factor f[2];
  double pb1, pb2, loss_first, loss_last;
};

__device__ __forceinline__ double swap_pair(double v) { return dpp_f64<0xB1>(v); }      // the value of lane ^ 1

template <int RPT>
__global__ __launch_bounds__(1024) void dual_clip_kernel(const LearnParams p, int lds_rows) {
  extern __shared__ double lrows[];                     // [lds_rows][nthreads]: rows RPT .. RPT + lds_rows - 1 of every lane
  __shared__ double part[64][NSUM];                     // one entry per 16-lane row of every wavefront
  __shared__ double cs[2][4];                           // s, 1/s, z of the pass (two copies, alternating)
  __shared__ Learner st;
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
  // ---- this lane's rows: tid, tid + nthreads, ...: the first RPT in registers, the next lds_rows in LDS, the rest
  //      re-read every pass.  Rows r < nfull exist for every lane, row nfull for the lanes below the remainder ----
  const int64_t nfull64 = p.T / nthreads;
  const int64_t mine = nfull64 + (tid < (int)(p.T - nfull64 * nthreads) ? 1 : 0);
  const int nfull = nfull64 < RPT ? (int)nfull64 : RPT;
  const bool has_tail = nfull64 < RPT && mine > nfull64;
  const int lds_end = (int)(mine < RPT + lds_rows ? mine : RPT + lds_rows);       // rows RPT .. lds_end - 1 sit in LDS
  const int lds_full = nfull64 <= RPT ? 0 : (nfull64 - RPT < lds_rows ? (int)(nfull64 - RPT) : lds_rows);      // ... for every lane
  const bool lds_tail = lds_end - RPT > lds_full;                                  // and one more for this lane
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
  for (int r = RPT; r < lds_end; ++r) {
    const double v = fetch((int64_t)r * nthreads + tid);
    lrows[(r - RPT) * nthreads + tid] = v;              // read back by this lane only
    mn = fmin(mn, v);
    mx = fmax(mx, v);
  }
  const int64_t first_extra = (int64_t)(RPT + lds_rows) * nthreads + tid;
  for (int64_t row = first_extra; row < p.T; row += nthreads) {
    const double v = fetch(row);
    mn = fmin(mn, v);
    mx = fmax(mx, v);
  }
  // ---- channel extremes ----
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) { mn = fmin(mn, __shfl_xor(mn, m, 64)); mx = fmax(mx, __shfl_xor(mx, m, 64)); }
  if (lane == 0) { part[wave][0] = mn; part[wave][1] = mx; }
  __syncthreads();
  mn = part[0][0]; mx = part[0][1];
  for (int w = 1; w < nwaves; ++w) { mn = fmin(mn, part[w][0]); mx = fmax(mx, part[w][1]); }
  __syncthreads();
  const double qmax = (double)((1 << p.bits) - 1);
  constexpr double B1 = 0.9, B2 = 0.999, ADAM_EPS = 1e-8;
  const bool live = mx > mn;                            // a constant channel has s = 0: nothing to learn
  const int k = lane & 1;                               // which factor this lane carries in wavefront 0
  const double ext = k ? mn : mx;
  // the quantizer of a pass from this lane's contracted bound and its neighbour's
  auto publish = [&](int slot, double bnd) {
    const double other = swap_pair(bnd);
    const double up = k ? other : bnd, lo = k ? bnd : other;
    const double s = (up - lo) / qmax;
    if (lane == 0) {
      cs[slot][0] = s;
      cs[slot][1] = 1.0 / s;
      cs[slot][2] = rint(-lo / s);
    }
  };
  if (wave == 0) {
    const double sg0 = 1.0 / (1.0 + exp(-p.alpha0));
    if (lane < 2) st.f[k] = Factor{p.alpha0, 0.0, 0.0, sg0};
    if (lane == 0) { st.pb1 = 1.0; st.pb2 = 1.0; st.loss_first = 0.0; st.loss_last = 0.0; }
    publish(0, ext * sg0);
  }
  __syncthreads();
  for (int pass = 0; live && pass <= p.iters; ++pass) {
    ChannelState c;
    c.s = cs[pass & 1][0];
    c.inv_s = cs[pass & 1][1];
    c.z = cs[pass & 1][2];
    c.qmax = qmax;
    // |x'/s| can only matter up to about |z| + qmax; the reciprocal shortcut is good while an ulp of that is < 1e-6
    c.exact = !(fabs(c.z) < 1073741824.0);
    Sums acc;
#pragma unroll
    for (int i = 0; i < NSUM; ++i) acc.v[i] = 0.0;
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
      if (r < nfull) accumulate(xp[r], c, acc);
      else if (r == nfull && has_tail) accumulate(xp[r], c, acc);
    }
    {                                                   // LDS rows: four in flight, then the leftovers
      const double* lp = lrows + tid;
      int r = 0;
      for (; r + 4 <= lds_full; r += 4) {
        const double v0 = lp[(r + 0) * nthreads], v1 = lp[(r + 1) * nthreads], v2 = lp[(r + 2) * nthreads], v3 = lp[(r + 3) * nthreads];
        accumulate(v0, c, acc);
        accumulate(v1, c, acc);
        accumulate(v2, c, acc);
        accumulate(v3, c, acc);
      }
      for (; r < lds_full; ++r) accumulate(lp[r * nthreads], c, acc);
      if (lds_tail) accumulate(lp[lds_full * nthreads], c, acc);
    }
    for (int64_t row = first_extra; row < p.T; row += nthreads) accumulate(fetch(row), c, acc);
#pragma unroll
    for (int i = 0; i < NSUM; ++i) acc.v[i] = row_sum(acc.v[i]);
    if ((lane & 15) == 0)
#pragma unroll
      for (int i = 0; i < NSUM; ++i) part[wave * 4 + (lane >> 4)][i] = acc.v[i];
    __syncthreads();
    if (wave == 0) {
      // lane l takes part l (4 per wavefront); a fixed tree adds them, so every lane ends with the same sums
      double t[NSUM];
#pragma unroll
      for (int i = 0; i < NSUM; ++i) {
        t[i] = row_sum(lane < nwaves * 4 ? part[lane][i] : 0.0);
        t[i] += __shfl_xor(t[i], 16, 64);
        t[i] += __shfl_xor(t[i], 32, 64);
      }
      if (lane == 0) {
        if (pass == 0) st.loss_first = t[0];
        st.loss_last = t[0];
      }
      if (pass < p.iters) {
        // ---- straight-through gradient and one Adam step, alpha_1 in the even lanes, alpha_2 in the odd ones ----
        Factor f = st.f[k];
        const double bnd = ext * f.sg, other = swap_pair(bnd);
        const double lo = k ? bnd : other;
        const double dL_dup = 2.0 * (t[1] - lo * c.inv_s * t[2]) / qmax;      // (dL/ds) / qmax
        const double grad = (k ? 2.0 * t[2] - dL_dup : dL_dup) * ext * f.sg * (1.0 - f.sg);
        const double pb1 = st.pb1 * B1, pb2 = st.pb2 * B2;
        f.m = B1 * f.m + (1.0 - B1) * grad;
        f.v = B2 * f.v + (1.0 - B2) * grad * grad;
        f.a -= p.lr * (f.m / (1.0 - pb1)) / (sqrt(f.v / (1.0 - pb2)) + ADAM_EPS);
        f.sg = 1.0 / (1.0 + exp(-f.a));
        if (lane < 2) st.f[k] = f;
        if (lane == 0) { st.pb1 = pb1; st.pb2 = pb2; }
        publish((pass + 1) & 1, ext * f.sg);
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    const double a1 = live ? st.f[0].a : p.alpha0, a2 = live ? st.f[1].a : p.alpha0;
    const double sg1 = 1.0 / (1.0 + exp(-a1)), sg2 = 1.0 / (1.0 + exp(-a2));
    p.alpha1[ch] = a1;
    p.alpha2[ch] = a2;
    if (p.clip_up) p.clip_up[ch] = (float)sg1;
    if (p.clip_lo) p.clip_lo[ch] = (float)sg2;
    if (p.up) p.up[ch] = mx * sg1;
    if (p.lo) p.lo[ch] = mn * sg2;
    if (p.loss0) p.loss0[ch] = live ? st.loss_first : 0.0;
    if (p.loss) p.loss[ch] = live ? st.loss_last : 0.0;
  }
}

constexpr int MAX_RPT = 24;                // rows a lane keeps in registers (2 each) under the 128-register bound
constexpr int LDS_BUDGET = 144 * 1024;     // dynamic LDS all workgroups of a compute unit may take together
constexpr int LDS_PER_WG = 60 * 1024;      // and one workgroup alone

int64_t lds_row_cap(int nw) {
  const int per_wg = LDS_BUDGET / (16 / nw) < LDS_PER_WG ? LDS_BUDGET / (16 / nw) : LDS_PER_WG;
  return per_wg / (8 * 64 * nw);
}

struct Shape { int nw, lds_rows; };

// Wavefronts per workgroup.  A workgroup is one channel; a compute unit holds 16 wavefronts of this kernel, so nw
// wavefronts per channel put floor(16 / nw) channels on a compute unit at a time.  Cost of a pass in units of one
// register-held row per SIMD: LDS rows 2.5, re-read rows 3, the serial update about 25, hidden in part when several
// workgroups share the compute unit; rounds are priced with the number of workgroups a compute unit then holds.
Shape choose_shape(int64_t T, int D, int num_cu) {
  Shape best{16, 0};
  double best_cost = 1e300;
  for (int nw = 1; nw <= 16; ++nw) {
    const int wgs = 16 / nw, nthreads = 64 * nw;
    const int64_t rpt = (T + nthreads - 1) / nthreads;
    const int64_t beyond = rpt > MAX_RPT ? rpt - MAX_RPT : 0;
    const int64_t cap = lds_row_cap(nw);
    const int64_t in_lds = beyond < cap ? beyond : cap;
    const double units = (double)(rpt - beyond) + 2.5 * (double)in_lds + 3.0 * (double)(beyond - in_lds);
    auto round_cost = [&](int64_t w) { return units * (nw / 4.0) * (double)w + 25.0 / (double)w + 3.0; };
    const int64_t slots = (int64_t)num_cu * wgs;
    const int64_t full_rounds = D / slots, rest = D - full_rounds * slots;
    double cost = (double)full_rounds * round_cost(wgs);
    if (rest) cost += round_cost((rest + num_cu - 1) / num_cu);
    if (cost < best_cost * 0.999) { best_cost = cost; best = Shape{nw, (int)in_lds}; }
  }
  return best;
}

template <int RPT>
rq_status launch_learner(rq_ctx* ctx, const LearnParams& p, int nw, int lds_rows) {
  const size_t lds = (size_t)lds_rows * 64 * nw * sizeof(double);
  if (lds > 48 * 1024)
    RQ_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&dual_clip_kernel<RPT>), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)lds));
  hipLaunchKernelGGL(dual_clip_kernel<RPT>, dim3((unsigned)(8 * ((p.D + 7) / 8))), dim3(64 * nw), lds, ctx->stream, p, lds_rows);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

}  // namespace

rq_status rq_launch_row_stats(rq_ctx* ctx, const float* x, int64_t T, int32_t D, int64_t ldx, int32_t norm_kind, double eps,
                              double* stats) {
  hipLaunchKernelGGL(row_stats_kernel, dim3((unsigned)((T + 3) / 4)), dim3(256), 0, ctx->stream, x, T, D, ldx, norm_kind, eps, stats);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

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
    const rq_status rc = rq_launch_row_stats(ctx, d->x, d->T, d->D, d->ldx, d->norm_kind, d->eps, stats);
    if (rc != RQ_OK) return rc;
    p.stats = stats;
  }
  Shape sh = choose_shape(d->T, d->D, ctx->num_cu);
  if (d->waves > 0) {
    sh.nw = d->waves;
    const int64_t rpt = (d->T + 64 * sh.nw - 1) / (64 * sh.nw);
    const int64_t cap = lds_row_cap(sh.nw);
    sh.lds_rows = (int)(rpt > MAX_RPT ? (rpt - MAX_RPT < cap ? rpt - MAX_RPT : cap) : 0);
  }
  const int64_t rpt = (d->T + 64 * sh.nw - 1) / (64 * sh.nw);
  if (rpt <= 8) return launch_learner<8>(ctx, p, sh.nw, 0);
  if (rpt <= 16) return launch_learner<16>(ctx, p, sh.nw, 0);
  return launch_learner<MAX_RPT>(ctx, p, sh.nw, sh.lds_rows);
}

