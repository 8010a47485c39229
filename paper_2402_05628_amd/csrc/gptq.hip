// GPTQ weight reconstruction on the folded weights (Algorithm 1, "perform GPTQ to quantize the layer's weights";
// Section "Sequential Quantization Pipeline").  The method is the published one of Frantar et al. (2022), computed here
// in its Cholesky form:
//   H = A^T A + lambda I                    exact integer Gram matrix of the layer's quantized inputs (int8 MFMA GEMM on a
//                                            transposed copy), lambda = percdamp * mean(diag H), dead columns H_jj = 1
//   U = upper Cholesky factor of H^-1        from ONE factorization: with J the index reversal, J H J = L L^T (blocked
//                                            right-looking Cholesky, float64), X = L^-1 (diagonal blocks merged by doubling),
//                                            and U = J X J, because H = (J L J)(J L J)^T with J L J upper triangular
//   for every column j (blocks of 64):       q_j = quantize(w_j) on the row's fixed min/max grid,
//                                            err_j = (w_j - dequant(q_j)) / U_jj,  W[:, j+1:] -= err_j (x) U[j, j+1:]
// inside a block four lanes sweep one output channel with its 64 columns in their registers; the columns after the block
// get E [16 x 64] times U[block, rest] from the other wavefronts of the workgroup that owns the 16 channels, while the
// next block is swept (the update of a row needs nothing from other rows, so the whole sweep is one launch).  Everything is
// float64 except the Gram matrix (exact integers) so that the codes agree with a float64 reference except next to rounding
// ties.
#include <cfloat>
#include <cmath>

#include "rq_internal.h"

namespace {

constexpr int NB = 64;       // block size of the factorization and of the sweep

// ---- transposed int8 copy: At[k][t] = A[t][k], zero beyond T ------------------------------------------------------
__global__ __launch_bounds__(256) void transpose_i8_kernel(const int8_t* __restrict__ A, int64_t T, int K, int64_t lda,
                                                           int8_t* __restrict__ At, int64_t Tpad) {
  __shared__ int8_t tile[64][65];
  const int64_t t0 = (int64_t)blockIdx.x * 64;
  const int k0 = blockIdx.y * 64;
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int r = i >> 6, c = i & 63;                      // r: token, c: channel
    tile[r][c] = t0 + r < T ? A[(t0 + r) * lda + k0 + c] : (int8_t)0;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int c = i >> 6, r = i & 63;
    At[(int64_t)(k0 + c) * Tpad + t0 + r] = tile[r][c];
  }
}

__global__ void fill_gram_consts_kernel(float* ones, int32_t* zeros, int K) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < K) { ones[i] = 1.f; zeros[i] = 0; }
}

// diag(H) before damping, dead flags, lambda.  With value = stored + delta:
//   H_ij = G_ij + delta (S_i + S_j) + T delta^2,   G = stored^T stored,  S = column sums of stored
__global__ __launch_bounds__(256) void diag_stats_kernel(const int32_t* __restrict__ G, const int32_t* __restrict__ S, int K,
                                                         int64_t T, int delta, double percdamp, int32_t* __restrict__ dead,
                                                         double* __restrict__ scal) {
  __shared__ double red[256];
  double acc = 0.0;
  for (int i = threadIdx.x; i < K; i += 256) {
    const double d = (double)G[(int64_t)i * K + i] + 2.0 * delta * (double)S[i] + (double)T * delta * delta;
    const bool dd = d == 0.0;
    dead[i] = dd ? 1 : 0;
    acc += dd ? 1.0 : d;
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) scal[0] = percdamp * (red[0] / (double)K);
}

// the damped Hessian with both indices reversed
__global__ __launch_bounds__(256) void assemble_kernel(const int32_t* __restrict__ G, const int32_t* __restrict__ S, int K, int64_t T,
                                                       int delta, const int32_t* __restrict__ dead, const double* __restrict__ scal,
                                                       double* __restrict__ H) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)K * K) return;
  const int i = (int)(idx / K), j = (int)(idx % K);
  double v = (double)G[idx] + (double)delta * ((double)S[i] + (double)S[j]) + (double)T * delta * delta;
  if (i == j) v = (dead[i] ? 1.0 : v) + scal[0];
  H[(int64_t)(K - 1 - i) * K + (K - 1 - j)] = v;
}

// ---- generic strided, batched float64 GEMM: C(m,n) = beta C(m,n) + alpha sum_k A(m,k) B(k,n), 64 x 64 tiles ---------
// `tri` lets triangular operands skip the blocks that are zero (or not needed):
//   TRI_B_LOWER: B(k, n) = 0 for k < n   -> the sum starts at the tile's first column
//   TRI_A_LOWER: A(m, k) = 0 for k > m   -> the sum ends at the tile's last row
//   TRI_C_LOWER: only tiles on or below the diagonal are computed (symmetric update, lower triangle in use)
enum { TRI_NONE = 0, TRI_B_LOWER = 1, TRI_A_LOWER = 2, TRI_C_LOWER = 3 };
struct GemmF64 {
  const double* A; int64_t sam, sak, bsa;
  const double* B; int64_t sbk, sbn, bsb;
  double* C; int64_t scm, scn, bsc;
  int64_t M; int N, Kin;         // N and Kin are multiples of 64
  int batch, tri;
  double alpha, beta;
};
__global__ __launch_bounds__(256) void gemm_f64_kernel(const GemmF64 g) {
  __shared__ double As[16][68], Bs[16][68];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int64_t m0 = (int64_t)blockIdx.y * 64;
  const int n0 = blockIdx.x * 64;
  if (g.tri == TRI_C_LOWER && n0 > m0) return;
  const double* A = g.A + (int64_t)blockIdx.z * g.bsa;
  const double* B = g.B + (int64_t)blockIdx.z * g.bsb;
  double* C = g.C + (int64_t)blockIdx.z * g.bsc;
  const int kbeg = g.tri == TRI_B_LOWER ? n0 : 0;
  const int kend = g.tri == TRI_A_LOWER ? (int)(m0 + 64 < g.Kin ? m0 + 64 : g.Kin) : g.Kin;
  // consecutive lanes walk whichever index of the operand is contiguous in memory
  const bool a_kfast = g.sak == 1 || g.sak == -1, b_kfast = g.sbk == 1 || g.sbk == -1;
  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
  // the next 16-deep slice of both operands is requested into registers before the current one is multiplied
  double ra[4], rb[4];
  auto request = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256;                                     // 16 x 64 elements of each operand
      const int ka = a_kfast ? e & 15 : e >> 6, ma = a_kfast ? e >> 4 : e & 63;
      const int64_t m = m0 + ma;
      ra[i] = m < g.M ? A[m * g.sam + (int64_t)(k0 + ka) * g.sak] : 0.0;
      const int kb2 = b_kfast ? e & 15 : e >> 6, nb2 = b_kfast ? e >> 4 : e & 63;
      rb[i] = B[(int64_t)(k0 + kb2) * g.sbk + (int64_t)(n0 + nb2) * g.sbn];
    }
  };
  if (kbeg < kend) request(kbeg);
  for (int k0 = kbeg; k0 < kend; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256;
      As[a_kfast ? e & 15 : e >> 6][a_kfast ? e >> 4 : e & 63] = ra[i];
      Bs[b_kfast ? e & 15 : e >> 6][b_kfast ? e >> 4 : e & 63] = rb[i];
    }
    __syncthreads();
    if (k0 + 16 < kend) request(k0 + 16);
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      double a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fma(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t m = m0 + ty * 4 + i;
    if (m >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      double* c = C + m * g.scm + (int64_t)(n0 + tx * 4 + j) * g.scn;
      *c = g.beta == 0.0 ? g.alpha * acc[i][j] : g.beta * *c + g.alpha * acc[i][j];
    }
  }
}

rq_status gemm_f64(rq_ctx* ctx, const GemmF64& g) {
  if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return RQ_OK;
  hipLaunchKernelGGL(gemm_f64_kernel, dim3((unsigned)(g.N / 64), (unsigned)((g.M + 63) / 64), (unsigned)g.batch), dim3(256), 0,
                     ctx->stream, g);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

// ---- diagonal block: L_kk = chol(H_kk) and its inverse (one wavefront, everything in registers) ------------------------
// Lane i holds row i of the block; an entry of another row comes through v_readlane (the lane index is a compile-time
// constant once the loops are unrolled), so neither LDS nor barriers are involved.
__device__ __forceinline__ double lane_value(double v, int lane) {
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_readlane((int)b, lane), hi = __builtin_amdgcn_readlane((int)(b >> 32), lane);
  return __longlong_as_double(((long long)hi << 32) | (unsigned)lo);
}
// Lane i holds row i of the block in a[]; on return a[] is row i of its Cholesky factor (zeros above the diagonal), and
// Lt (LDS, LP doubles per row) holds the factor as well.  An entry of another row comes from that LDS copy, which every
// lane extends by its new entry after each column: the address is the same for all lanes, two entries per read.  The
// sum of column j + 1 is formed, up to its last term, while the square root and the division of column j are in flight
// (its terms k < j need only columns that are complete); the last term takes l_{j+1, j} from its lane directly.
// Lt is passed through a vector register the compiler cannot see through, so that the reads use one base register and
// immediate offsets instead of a scalar address computation each.
constexpr int LP = 66;
__device__ __forceinline__ const double* opaque_lds(const double* p) {
  int z = 0;
  asm volatile("" : "+v"(z));
  return p + z;
}
__device__ __forceinline__ void diag_factor(double (&a)[NB], int i, double* Lt) {
  // left-looking: l_ij = (h_ij - sum_{k<j} l_ik l_jk) / l_jj
  const double* Lr = opaque_lds(Lt);
  double sum = 0.0;
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const double v = a[j] - sum;
    const double d = sqrt(lane_value(v, j));
    double psum = 0.0;
    if (j + 1 < NB) {
      const double2* row = reinterpret_cast<const double2*>(Lr + (j + 1) * LP);
#pragma unroll
      for (int k = 0; k < j; k += 2) {
        const double2 l = row[k >> 1];
        psum = fma(a[k], l.x, psum);
        if (k + 1 < j) psum = fma(a[k + 1], l.y, psum);
        if ((k & 14) == 14) __builtin_amdgcn_sched_barrier(0);   // at most eight reads in flight: the registers are needed
      }
    }
    a[j] = i == j ? d : (i > j ? v / d : 0.0);
    Lt[i * LP + j] = a[j];
    if (j + 1 < NB) sum = fma(a[j], lane_value(a[j], j + 1), psum);
  }
}
// Lane c takes column c of the inverse of the factor: x(r) = (delta_rc - sum_{m<r} l_rm x(m)) / l_rr, x(m) = 0 for m < c.
// Same arrangement: the sum of row r + 1 without its last term stands before the division of row r.
__device__ __forceinline__ void diag_inverse(double (&x)[NB], int i, const double* __restrict__ Lt) {
  const double* Lr = opaque_lds(Lt);
  double sum = 0.0;
#pragma unroll
  for (int r = 0; r < NB; ++r) {
    double psum = 0.0;
    double last = 0.0;
    if (r + 1 < NB) {
      const double2* row = reinterpret_cast<const double2*>(Lr + (r + 1) * LP);
#pragma unroll
      for (int m = 0; m < r; m += 2) {
        const double2 l = row[m >> 1];
        psum = fma(l.x, x[m], psum);
        if (m + 1 < r) psum = fma(l.y, x[m + 1], psum);
        if ((m & 14) == 14) __builtin_amdgcn_sched_barrier(0);
      }
      last = Lr[(r + 1) * LP + r];
    }
    x[r] = r < i ? 0.0 : ((r == i ? 1.0 : 0.0) - sum) / Lr[r * LP + r];
    if (r + 1 < NB) sum = fma(last, x[r], psum);
  }
}

// ---- one step of the blocked right-looking factorization in one launch ----------------------------------------------
// Step kb: L_kk = chol(H_kk), D = L_kk^-1, panel L_ik = H_ik D^T (i > kb), trailing update H_ij -= L_ik L_jk^T (i >= j > kb).
// One workgroup per trailing tile (i, j).  Each factors and inverts the 64 x 64 diagonal block itself (its first wavefront,
// in registers; the others fetch the tile's two panel blocks meanwhile), forms the two panel blocks it needs and then its
// tile: nothing passes between workgroups inside the launch, at the price of the same small factorization in every one.
// Workgroup 0 stores L_kk and D, the workgroups of the first tile column store the panel.  Sums run over k in ascending
// order, one fma per term.  With more trailing tiles than CUs the repeated factorization (and the panel blocks formed once
// per tile) would cost more than the launches saved: such steps run the kernel for the diagonal block alone (`diag_only`)
// and take panel and trailing update as two launches of the float64 GEMM below, the same sums in the same order.
constexpr int TP = 66;                                      // row pitch of the k-major 64 x 64 tiles in LDS (16-byte rows)
constexpr int CHOL_LDS = (3 * NB * TP + NB * LP) * 8;
__device__ __forceinline__ void tile_product(const double* __restrict__ As, const double* __restrict__ Bs, int ty, int tx,
                                             double (&acc)[4][4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
#pragma unroll 4
  for (int kk = 0; kk < NB; ++kk) {
    const double2* ap = reinterpret_cast<const double2*>(As + kk * TP + ty * 4);
    const double2* bp = reinterpret_cast<const double2*>(Bs + kk * TP + tx * 4);
    const double2 a01 = ap[0], a23 = ap[1], b01 = bp[0], b23 = bp[1];
    const double a[4] = {a01.x, a01.y, a23.x, a23.y}, b[4] = {b01.x, b01.y, b23.x, b23.y};
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = fma(a[i], b[j], acc[i][j]);
  }
}
__global__ __launch_bounds__(256) void chol_step_kernel(double* __restrict__ H, double* __restrict__ L, double* __restrict__ Dinv,
                                                        int K, int kb, int diag_only) {
  extern __shared__ __attribute__((aligned(16))) double chol_lds[];
  double* Bs = chol_lds;                                    // Bs[k][n] = D(n, k)
  double* Ai = chol_lds + NB * TP;                          // Ai[k][m] = H_ik(m, k), later L_ik(m, k)
  double* Aj = chol_lds + 2 * NB * TP;
  double* Lt = chol_lds + 3 * NB * TP;                      // the diagonal block's factor
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int n = diag_only ? 0 : K / NB - kb - 1;            // block rows below the diagonal block that this launch updates
  int ti = 0, tj = (int)blockIdx.x;
  while (tj > ti) { ++ti; tj -= ti; }                       // tile t of the lower triangle: t = ti (ti + 1) / 2 + tj
  const int64_t bi = (int64_t)(kb + 1 + ti) * NB, bj = (int64_t)(kb + 1 + tj) * NB, c0 = (int64_t)kb * NB;
  if (tid < 64) {
    const int i = tid;
    const int64_t base = c0 * K + c0;
    double a[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) a[c] = H[base + (int64_t)i * K + c];        // only c <= i is used (the maintained triangle)
    diag_factor(a, i, Lt);
    double x[NB];
    diag_inverse(x, i, Lt);
#pragma unroll
    for (int r = 0; r < NB; ++r) Bs[i * TP + r] = x[r];
  } else if (n > 0) {
    for (int e = tid - 64; e < NB * NB; e += 192) {
      const int k = e & 63, m = e >> 6;
      Ai[k * TP + m] = H[(bi + m) * K + c0 + k];
      if (ti != tj) Aj[k * TP + m] = H[(bj + m) * K + c0 + k];
    }
  }
  __syncthreads();
  if (blockIdx.x == 0) {                                    // L_kk and its inverse, from their LDS copies
    for (int e = tid; e < NB * NB; e += 256) {
      const int r = e >> 6, c = e & 63;
      L[c0 * K + c0 + (int64_t)r * K + c] = Lt[r * LP + c];
      Dinv[(int64_t)kb * NB * NB + r * NB + c] = Bs[c * TP + r];
    }
  }
  if (n <= 0) return;
  double li[4][4], lj[4][4];
  tile_product(Ai, Bs, ty, tx, li);
  if (ti != tj) tile_product(Aj, Bs, ty, tx, lj);
  if (tj == 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) L[(bi + ty * 4 + i) * K + c0 + tx * 4 + j] = li[i][j];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      Ai[(tx * 4 + j) * TP + ty * 4 + i] = li[i][j];
      if (ti != tj) Aj[(tx * 4 + j) * TP + ty * 4 + i] = lj[i][j];
    }
  __syncthreads();
  double acc[4][4];
  tile_product(Ai, ti != tj ? Aj : Ai, ty, tx, acc);
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      double* c = H + (bi + ty * 4 + i) * K + bj + tx * 4 + j;
      *c = *c - acc[i][j];
    }
}

// X = 0 with the inverted diagonal blocks in place
__global__ __launch_bounds__(256) void init_inverse_kernel(double* __restrict__ X, const double* __restrict__ Dinv, int K) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)K * K) return;
  const int i = (int)(idx / K), j = (int)(idx % K);
  X[idx] = (i / NB == j / NB) ? Dinv[(int64_t)(i / NB) * NB * NB + (i % NB) * NB + (j % NB)] : 0.0;
}

// ---- per output channel: grid from the row's extremes (dead columns count as 0; the range always contains 0, so the
// zero-point is a code of the grid), float64 working copy ----------------
__global__ __launch_bounds__(256) void row_init_kernel(const float* __restrict__ W, int K, int bits, const int32_t* __restrict__ dead,
                                                       double* __restrict__ Wc, double* __restrict__ s64, double* __restrict__ z64) {
  __shared__ float smin[256], smax[256];
  const int tid = threadIdx.x, n = blockIdx.x;
  const float* w = W + (int64_t)n * K;
  float lo = 0.f, hi = 0.f;
  for (int k = tid; k < K; k += 256) {
    const float v = dead[k] ? 0.f : w[k];
    Wc[(int64_t)n * K + k] = (double)v;
    lo = fminf(lo, v);
    hi = fmaxf(hi, v);
  }
  smin[tid] = lo;
  smax[tid] = hi;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) {
      smin[tid] = fminf(smin[tid], smin[tid + s]);
      smax[tid] = fmaxf(smax[tid], smax[tid + s]);
    }
    __syncthreads();
  }
  if (tid == 0) {
    const double dlo = (double)smin[0], dhi = (double)smax[0];
    double s = (double)(float)((dhi - dlo) / (double)((1 << bits) - 1));      // the scale is stored as float32
    if (!(s > 0.0)) s = 1.0;                                                     // a row of zeros
    s64[n] = s;
    z64[n] = rint(-dlo / s);
  }
}

// ---- the sweep inside one block of 64 columns: four lanes per output channel -----------------------------------------
// Lane q of a quad owns columns q, q + 4, ... of its channel's block.  Every step broadcasts the current column's
// weight from its owner, all four lanes take the same code and error, and each updates the columns it owns.
constexpr int SWEEP_ROWS = 16;   // most output channels per workgroup of the sweep (four lanes each in its first wavefront)
constexpr int SWEEP_WAVES = 8;
template <int SRC>
__device__ __forceinline__ double quad_bcast(double v) {
  const long long b = __double_as_longlong(v);
  constexpr int ctrl = SRC * 0x55;                          // quad_perm: [SRC, SRC, SRC, SRC]
  const int lo = __builtin_amdgcn_update_dpp(0, (int)b, ctrl, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), ctrl, 0xF, 0xF, true);
  return __longlong_as_double(((long long)hi << 32) | (unsigned)lo);
}

template <int JJ>
__device__ __forceinline__ void sweep_step(double (&w)[NB / 4], const double (*Ub)[NB], int q, double s, double z, double qmax,
                                           uint8_t* code_row, double* e_col) {
  const double x = quad_bcast<JJ & 3>(w[JJ >> 2]);
  const double c = fmin(fmax(rint(x / s) + z, 0.0), qmax);
  const double err = (x - s * (c - z)) / Ub[JJ][JJ];
  if (q == (JJ & 3)) {
    code_row[JJ] = (uint8_t)c;
    e_col[JJ * SWEEP_ROWS] = err;
  }
#pragma unroll
  for (int t = 0; t < NB / 4; ++t) {
    const int cc = 4 * t + q;                               // the column this lane's w[t] holds
    if (4 * t + 3 > JJ) {                                   // some lane of the quad still has work in this slot
      const double u = Ub[JJ][cc];
      if (cc > JJ) w[t] -= err * u;
    }
  }
  if constexpr (JJ + 1 < NB) sweep_step<JJ + 1>(w, Ub, q, s, z, qmax, code_row, e_col);
}

// The whole sweep in one launch.  A workgroup of 8 wavefronts owns 16 output channels.  Per block b of 64 columns:
//   phase 1 (all wavefronts)   U[block b, block b] -> LDS; the block's own columns get the update of block b - 1,
//                              W[:, b] -= E_{b-1} U[b-1, b]  (two channels per wavefront, lane = column)
//   phase 2 (wavefront 0)      the sweep of block b: codes, errors E_b (kept in LDS, [column][channel])
//           (six others)       meanwhile the columns after block b get the update of block b - 1,
//                              W[:, c] -= E_{b-1} U[b-1, c]  (chunks of 64 columns dealt to the wavefronts, lane = column,
//                              all 16 channels of a column in the lane's registers)
// A column block c thus receives E_0 U, E_1 U, ... E_{c-1} U one after the other, each as one sum over the block's 64
// columns in ascending order.  The working copy of the weights stays in global memory; the wavefronts of a workgroup hand
// it to each other across the barriers (a workgroup's wavefronts share their CU's vector cache, and __syncthreads orders
// their stores and loads at workgroup scope).
template <int ROWS>
__global__ __launch_bounds__(SWEEP_WAVES * 64) void sweep_all_kernel(double* __restrict__ Wc, const double* __restrict__ X, int N, int K,
                                                                   int bits, const double* __restrict__ s64,
                                                                   const double* __restrict__ z64, uint8_t* __restrict__ codes) {
  __shared__ double Ub[NB][NB];                             // U[j0 + jj][j0 + cc] = X[K-1-j0-jj][K-1-j0-cc], upper triangular
  __shared__ __attribute__((aligned(16))) double Es[2][NB][SWEEP_ROWS];
  __shared__ uint8_t code_s[SWEEP_ROWS][NB];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n0 = blockIdx.x * ROWS;
  const int nrows = N - n0 < ROWS ? N - n0 : ROWS;
  const int nb = K / NB;
  const int q = lane & 3, rr = lane >> 2;
  const int n = n0 + (rr < nrows ? rr : nrows - 1);         // idle quads shadow the last channel and write nothing
  const double s = s64[n], z = z64[n], qmax = (double)((1 << bits) - 1);
  for (int b = 0; b < nb; ++b) {
    const int j0 = b * NB;
    const double(*Ep)[SWEEP_ROWS] = Es[(b + 1) & 1];        // errors of block b - 1
    // ---- phase 1 ----
    for (int i = tid; i < NB * NB; i += SWEEP_WAVES * 64) {
      const int jj = i >> 6, cc = i & 63;
      Ub[jj][cc] = X[(int64_t)(K - 1 - j0 - jj) * K + (K - 1 - j0 - cc)];
    }
    if (b > 0 && wave < ROWS) {
      constexpr int RW = (ROWS + SWEEP_WAVES - 1) / SWEEP_WAVES;   // channels per wavefront: wave, wave + 8
      const int c = j0 + lane;
      const double* u = X + (int64_t)(K - 1 - (j0 - NB)) * K + (K - 1 - c);   // U[j0 - 64 + k][c] = u[-k K]
      double w[RW], acc[RW];
#pragma unroll
      for (int r = 0; r < RW; ++r) {
        const int row = wave + r * SWEEP_WAVES;
        w[r] = Wc[(int64_t)(n0 + (row < nrows ? row : nrows - 1)) * K + c];
        acc[r] = 0.0;
      }
#pragma unroll 8
      for (int k = 0; k < NB; ++k) {
        const double uk = u[-(int64_t)k * K];
#pragma unroll
        for (int r = 0; r < RW; ++r) acc[r] = fma(Ep[k][wave + r * SWEEP_WAVES], uk, acc[r]);
      }
#pragma unroll
      for (int r = 0; r < RW; ++r)
        if (wave + r * SWEEP_WAVES < nrows) Wc[(int64_t)(n0 + wave + r * SWEEP_WAVES) * K + c] = w[r] - acc[r];
    }
    __syncthreads();
    // ---- phase 2 ----
    if (wave == 0) {
      double w[NB / 4];
#pragma unroll
      for (int t = 0; t < NB / 4; ++t) w[t] = Wc[(int64_t)n * K + j0 + 4 * t + q];
      sweep_step<0>(w, Ub, q, s, z, qmax, code_s[rr], &Es[b & 1][0][rr]);
      __builtin_amdgcn_wave_barrier();
      if (rr < nrows) {
#pragma unroll
        for (int t = 0; t < NB / 4; ++t) codes[(int64_t)n * K + j0 + 4 * t + q] = code_s[rr][4 * t + q];
      }
    } else if (b > 0 && wave != 4) {
      // Lane k keeps E_{b-1}[k][0..ROWS); a term's error reaches the fma as a scalar operand through v_readlane (LDS stays
      // free for the sweep, whose chain of dependent steps waits on its own LDS reads).  Wavefront 4 shares its SIMD
      // with the sweep and stays out.  CP chunks of 64 columns per pass: 32 sums per lane whatever ROWS is, and one
      // v_readlane pair serves CP terms.
      constexpr int CP = 32 / ROWS;
      const int fw = wave < 4 ? wave - 1 : wave - 2;        // 0..5
      double e[ROWS];
#pragma unroll
      for (int r = 0; r < ROWS; ++r) e[r] = Ep[lane][r];
      for (int c0 = j0 + NB + fw * CP * NB; c0 < K; c0 += (SWEEP_WAVES - 2) * CP * NB) {
        const int c = c0 + lane;
        const double* u = X + (int64_t)(K - 1 - (j0 - NB)) * K + (K - 1 - c);
        // the current values first (rows beyond the last channel re-read the last one and store nothing)
        double w[CP][ROWS], acc[CP][ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
          const double* wp = Wc + (int64_t)(n0 + (r < nrows ? r : nrows - 1)) * K + c;
#pragma unroll
          for (int pc = 0; pc < CP; ++pc) {
            w[pc][r] = c0 + pc * NB < K ? wp[pc * NB] : 0.0;
            acc[pc][r] = 0.0;
          }
        }
#pragma unroll 8
        for (int k = 0; k < NB; ++k) {
          double uk[CP];
#pragma unroll
          for (int pc = 0; pc < CP; ++pc) uk[pc] = c0 + pc * NB < K ? u[-(int64_t)k * K - pc * NB] : 0.0;
#pragma unroll
          for (int r = 0; r < ROWS; ++r) {
            const double ek = lane_value(e[r], k);
#pragma unroll
            for (int pc = 0; pc < CP; ++pc) acc[pc][r] = fma(ek, uk[pc], acc[pc][r]);
          }
        }
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
          if (r < nrows) {
            double* wp = Wc + (int64_t)(n0 + r) * K + c;
#pragma unroll
            for (int pc = 0; pc < CP; ++pc)
              if (c0 + pc * NB < K) wp[pc * NB] = w[pc][r] - acc[pc][r];
          }
      }
    }
    __syncthreads();
  }
}

// ---- codes -> storage format, column sums, row permutation of the gated MLP (same conventions as rq_weight_quant_pack) --
__global__ __launch_bounds__(256) void pack_kernel(const uint8_t* __restrict__ codes, int K, int format, int gate_up_rows,
                                                   const double* __restrict__ s64, const double* __restrict__ z64,
                                                   const float* __restrict__ bias, void* __restrict__ w_out, float* __restrict__ s_w,
                                                   int32_t* __restrict__ z_w, int32_t* __restrict__ colsum_w, float* __restrict__ bias_out) {
  __shared__ int ssum[256];
  const int tid = threadIdx.x, n = blockIdx.x;
  const uint8_t* c = codes + (int64_t)n * K;
  const int z = (int)z64[n];
  int r = n;
  if (gate_up_rows > 0) {
    const int Dm = gate_up_rows, j = n < Dm ? n : n - Dm;
    r = (j / 32) * 64 + (n < Dm ? 0 : 32) + (j % 32);
  }
  int csum = 0;
  if (format == RQ_W_U4) {
    uint8_t* out = static_cast<uint8_t*>(w_out) + (int64_t)r * (K / 2);
    for (int g = tid; g < K / 8; g += 256) {
      const uint8_t* q = c + g * 8;
      const uint32_t pk = (uint32_t)(q[0] | (q[4] << 4)) | ((uint32_t)(q[1] | (q[5] << 4)) << 8) |
                          ((uint32_t)(q[2] | (q[6] << 4)) << 16) | ((uint32_t)(q[3] | (q[7] << 4)) << 24);
      *reinterpret_cast<uint32_t*>(out + g * 4) = pk;
#pragma unroll
      for (int e = 0; e < 8; ++e) csum += (int)q[e] - z;
    }
  } else {
    int8_t* out = static_cast<int8_t*>(w_out) + (int64_t)r * K;
    const int off = format == RQ_W_I8_CENTERED ? 128 : z;
    for (int k = tid; k < K; k += 256) {
      out[k] = (int8_t)((int)c[k] - off);
      csum += (int)c[k] - z;
    }
  }
  ssum[tid] = csum;
  __syncthreads();
  for (int s2 = 128; s2 > 0; s2 >>= 1) {
    if (tid < s2) ssum[tid] += ssum[tid + s2];
    __syncthreads();
  }
  if (tid == 0) {
    s_w[r] = (float)s64[n];
    z_w[r] = z;
    colsum_w[r] = ssum[0];
    if (bias_out) bias_out[r] = bias ? bias[n] : 0.f;
  }
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct Layout {
  size_t at, g, s, ones, zeros, dead, scal, h, l, x, dinv, wc, codes, s64, z64, total;
};
Layout make_layout(int N, int K, int64_t T) {
  const size_t Tpad = (size_t)((T + 63) / 64) * 64, KK = (size_t)K * K;
  Layout o;
  size_t p = 0;
  auto take = [&](size_t bytes) { const size_t at = p; p += align256(bytes); return at; };
  o.at = take((size_t)K * Tpad);
  o.g = take(KK * 4);
  o.s = take((size_t)K * 4);
  o.ones = take((size_t)K * 4);
  o.zeros = take((size_t)K * 4);
  o.dead = take((size_t)K * 4);
  o.scal = take(64);
  o.h = take(KK * 8);
  o.l = take(KK * 8);
  o.x = take(KK * 8);
  o.dinv = take((size_t)(K / NB) * NB * NB * 8);
  o.wc = take((size_t)N * K * 8);
  o.codes = take((size_t)N * K);
  o.s64 = take((size_t)N * 8);
  o.z64 = take((size_t)N * 8);
  o.total = p;
  return o;
}

}  // namespace

size_t rq_gptq_workspace_bytes(int32_t N, int32_t K, int64_t T) {
  if (N <= 0 || K <= 0 || T <= 0) return 0;
  return make_layout(N, K, T).total;
}

rq_status rq_launch_gptq(rq_ctx* ctx, const rq_gptq_desc* d) {
  const int N = d->N, K = d->K, nb = K / NB;
  const int64_t T = d->T, Tpad = (T + 63) / 64 * 64;
  const Layout o = make_layout(N, K, T);
  char* ws = static_cast<char*>(d->workspace);
  int8_t* At = reinterpret_cast<int8_t*>(ws + o.at);
  int32_t* G = reinterpret_cast<int32_t*>(ws + o.g);
  int32_t* S = reinterpret_cast<int32_t*>(ws + o.s);
  float* ones = reinterpret_cast<float*>(ws + o.ones);
  int32_t* zeros = reinterpret_cast<int32_t*>(ws + o.zeros);
  int32_t* dead = reinterpret_cast<int32_t*>(ws + o.dead);
  double* scal = reinterpret_cast<double*>(ws + o.scal);
  double* H = reinterpret_cast<double*>(ws + o.h);
  double* L = reinterpret_cast<double*>(ws + o.l);
  double* X = reinterpret_cast<double*>(ws + o.x);
  double* Dinv = reinterpret_cast<double*>(ws + o.dinv);
  double* Wc = reinterpret_cast<double*>(ws + o.wc);
  uint8_t* codes = reinterpret_cast<uint8_t*>(ws + o.codes);
  double* s64 = reinterpret_cast<double*>(ws + o.s64);
  double* z64 = reinterpret_cast<double*>(ws + o.z64);
  hipStream_t st = ctx->stream;
  const int delta = d->a_off - d->z_a;
  const int64_t KK = (int64_t)K * K;

  // ---- Gram matrix of the stored codes on the matrix cores, column sums, Hessian ----
  hipLaunchKernelGGL(transpose_i8_kernel, dim3((unsigned)(Tpad / 64), (unsigned)(K / 64)), dim3(256), 0, st, d->A, T, K, d->lda, At, Tpad);
  hipLaunchKernelGGL(fill_gram_consts_kernel, dim3((K + 255) / 256), dim3(256), 0, st, ones, zeros, K);
  RQ_HIP(hipGetLastError());
  rq_gemm_desc gd = {};
  gd.M = K; gd.N = K; gd.K = (int32_t)Tpad;
  gd.A = At; gd.lda = Tpad; gd.a_off = 0; gd.z_a = 0; gd.s_a = 1.f;
  gd.B = At; gd.ldb = Tpad; gd.b_format = RQ_W_I8_BAKED; gd.s_b = ones; gd.z_b = zeros; gd.colsum_b = zeros;
  gd.out_acc = G; gd.ldacc = K;
  gd.batch_outer = 1; gd.batch_inner = 1; gd.n_seg = 1;
  rq_status rc = rq_launch_qgemm_weight(ctx, &gd);
  if (rc != RQ_OK) return rc;
  rc = rq_launch_rowsum(ctx, At, K, (int32_t)Tpad, Tpad, S);
  if (rc != RQ_OK) return rc;
  hipLaunchKernelGGL(diag_stats_kernel, dim3(1), dim3(256), 0, st, G, S, K, T, delta, d->percdamp, dead, scal);
  hipLaunchKernelGGL(assemble_kernel, dim3((unsigned)((KK + 255) / 256)), dim3(256), 0, st, G, S, K, T, delta, dead, scal, H);
  RQ_HIP(hipGetLastError());

  // ---- blocked right-looking Cholesky of the index-reversed Hessian: H = L L^T, one launch per block column ----
  {
    static rq_once_per_device once;
    RQ_HIP(rq_allow_dynamic_lds(ctx, once, reinterpret_cast<const void*>(&chol_step_kernel), CHOL_LDS));
  }
  const int num_cu = ctx->num_cu > 0 ? ctx->num_cu : 256;
  for (int kb = 0; kb < nb; ++kb) {
    const int n = nb - kb - 1;
    const int64_t tiles = (int64_t)n * (n + 1) / 2;
    if (tiles <= num_cu) {
      hipLaunchKernelGGL(chol_step_kernel, dim3((unsigned)(n > 0 ? tiles : 1)), dim3(256), CHOL_LDS, st, H, L, Dinv, K, kb, 0);
      RQ_HIP(hipGetLastError());
      continue;
    }
    hipLaunchKernelGGL(chol_step_kernel, dim3(1), dim3(256), CHOL_LDS, st, H, L, Dinv, K, kb, 1);
    RQ_HIP(hipGetLastError());
    const int r0 = (kb + 1) * NB, rest = K - r0;
    const int64_t c0 = (int64_t)kb * NB;
    // panel: L[r0:, kb] = H[r0:, kb] Dinv_kk^T
    GemmF64 g = {};
    g.batch = 1; g.tri = TRI_NONE;
    g.A = H + (int64_t)r0 * K + c0; g.sam = K; g.sak = 1;
    g.B = Dinv + (int64_t)kb * NB * NB; g.sbk = 1; g.sbn = NB;
    g.C = L + (int64_t)r0 * K + c0; g.scm = K; g.scn = 1;
    g.M = rest; g.N = NB; g.Kin = NB; g.alpha = 1.0; g.beta = 0.0;
    if ((rc = gemm_f64(ctx, g)) != RQ_OK) return rc;
    // trailing update: H[r0:, r0:] -= L[r0:, kb] L[r0:, kb]^T
    g.A = L + (int64_t)r0 * K + c0; g.sam = K; g.sak = 1;
    g.B = L + (int64_t)r0 * K + c0; g.sbk = 1; g.sbn = K;
    g.C = H + (int64_t)r0 * K + r0; g.scm = K; g.scn = 1;
    g.M = rest; g.N = rest; g.Kin = NB; g.alpha = -1.0; g.beta = 1.0; g.tri = TRI_C_LOWER;
    if ((rc = gemm_f64(ctx, g)) != RQ_OK) return rc;
  }
  // ---- X = L^-1 by doubling: the 64-blocks on the diagonal are inverted already; two neighbouring inverted diagonal
  //      blocks X11 (s x s) and X22 merge through X21 = -X22 (L21 X11).  All pairs of a level run as one batched GEMM
  //      pair; H, no longer needed, holds L21 X11.  A shorter last pair (K / 64 not a power of two) runs on its own ----
  hipLaunchKernelGGL(init_inverse_kernel, dim3((unsigned)((KK + 255) / 256)), dim3(256), 0, st, X, Dinv, K);
  RQ_HIP(hipGetLastError());
  for (int64_t sz = NB; sz < K; sz *= 2) {
    const int64_t full_pairs = K / (2 * sz);                 // pairs whose second half has the full size
    const int64_t tail_start = full_pairs * 2 * sz;          // a last pair with a shorter second half, if any
    const int64_t tail_second = K - tail_start > sz ? K - tail_start - sz : 0;
    for (int part = 0; part < 2; ++part) {
      const int64_t p0 = part == 0 ? 0 : tail_start, second = part == 0 ? sz : tail_second;
      const int batch = part == 0 ? (int)full_pairs : (tail_second > 0 ? 1 : 0);
      if (batch == 0) continue;
      const int64_t pair_stride = 2 * sz * ((int64_t)K + 1);
      const int64_t o21 = (p0 + sz) * K + p0, o11 = p0 * K + p0, o22 = (p0 + sz) * K + (p0 + sz);
      GemmF64 g = {};
      g.batch = batch;
      g.A = L + o21; g.sam = K; g.sak = 1; g.bsa = pair_stride;
      g.B = X + o11; g.sbk = K; g.sbn = 1; g.bsb = pair_stride;
      g.C = H + o21; g.scm = K; g.scn = 1; g.bsc = pair_stride;
      g.M = second; g.N = (int)sz; g.Kin = (int)sz; g.alpha = 1.0; g.beta = 0.0; g.tri = TRI_B_LOWER;
      if ((rc = gemm_f64(ctx, g)) != RQ_OK) return rc;
      g.A = X + o22; g.sam = K; g.sak = 1; g.bsa = pair_stride;
      g.B = H + o21; g.sbk = K; g.sbn = 1; g.bsb = pair_stride;
      g.C = X + o21; g.scm = K; g.scn = 1; g.bsc = pair_stride;
      g.M = second; g.N = (int)sz; g.Kin = (int)second; g.alpha = -1.0; g.beta = 0.0; g.tri = TRI_A_LOWER;
      if ((rc = gemm_f64(ctx, g)) != RQ_OK) return rc;
    }
  }
  // ---- the sweep ----
  hipLaunchKernelGGL(row_init_kernel, dim3((unsigned)N), dim3(256), 0, st, d->W, K, d->bits, dead, Wc, s64, z64);
  RQ_HIP(hipGetLastError());
  // Output channels per workgroup: the six wavefronts that update the later columns must keep up with the one that sweeps
  // (about 33 us per block).  With 16 channels they do for K <= 1664; longer rows take 8 channels per workgroup (half the
  // update's work per workgroup, a third of its time), unless that would give more workgroups than the chip holds at once.
  const int resident = num_cu * 3;
  if (K <= 1664 || (N + 7) / 8 > resident)
    hipLaunchKernelGGL(sweep_all_kernel<16>, dim3((unsigned)((N + 15) / 16)), dim3(SWEEP_WAVES * 64), 0, st, Wc, X, N, K, d->bits, s64, z64, codes);
  else
    hipLaunchKernelGGL(sweep_all_kernel<8>, dim3((unsigned)((N + 7) / 8)), dim3(SWEEP_WAVES * 64), 0, st, Wc, X, N, K, d->bits, s64, z64, codes);
  RQ_HIP(hipGetLastError());
  hipLaunchKernelGGL(pack_kernel, dim3((unsigned)N), dim3(256), 0, st, codes, K, d->format, d->gate_up_rows, s64, z64, d->bias, d->w_out,
                     d->s_w, d->z_w, d->colsum_w, d->bias_out);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}
