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
#include "rq_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct GemmParams {
  int64_t M;
  int N, K;
  const int8_t* A;
  int64_t lda;
  const uint8_t* B;
  int64_t ldb;
  const float* s_b;
  const int32_t* z_b;
  const int32_t* colsum_b;
  const int32_t* rowsum_a;
  const float* bias;
  float s_a;
  int da;        // a_off - z_a
  int centered;  // weights stored code - 128: needs (128 - z_b[n]) * rowsum_a[m]
  int act;
  const float* residual;
  int64_t ldr;
  int32_t* out_acc;
  int64_t ldacc;
  float* out_f32;
  int64_t ldf;
  int8_t* out_q;
  int64_t ldq;
  int n_seg, seg_len;
  float inv_so[4];
  float zo[4];   // z_o - off_o
  int lo[4], hi[4];
  int tiles_n;
};

__device__ __forceinline__ int swz(int row, int c) {
  return (row >> 1) * 128 + (((((row & 1) << 2) | c) ^ ((row >> 1) & 7)) << 4);
}

// erf by the rational-times-Gaussian formula 7.1.26 of Abramowitz & Stegun (|error| <= 1.5e-7), enough for
// 8-bit re-quantization of GELU outputs; GELU(y) = y * Phi(y), Phi(y) = 1 - r/2 (y >= 0) or r/2 (y < 0).
__device__ __forceinline__ float gelu_f(float y) {
  const float ax = fabsf(y) * 0.70710678118654752f;
  const float t = __frcp_rn(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  p *= t;
  const float e = __builtin_amdgcn_exp2f(ax * ax * -1.4426950408889634f);
  const float hr = 0.5f * p * e;
  const float phi = y >= 0.f ? 1.0f - hr : hr;
  return y * phi;
}

__device__ __forceinline__ float silu_f(float y) {
  return y * __frcp_rn(1.0f + __builtin_amdgcn_exp2f(y * -1.4426950408889634f));
}

template <int BM, int BN, bool W4>
__global__ __launch_bounds__(256, 2) void qgemm_kernel(const GemmParams p) {
  constexpr int WM = BM / 2, WN = BN / 2;        // wavefront tile
  constexpr int TM = WM / 32, TN = WN / 32;      // MFMA tiles per wavefront
  constexpr int A_BYTES = BM * 64, B_BYTES = BN * 64;
  constexpr int A_IT = BM * 4 / 256;             // 16-byte chunks per thread per stage
  constexpr int B_IT = W4 ? (BN * 2 / 256) : (BN * 4 / 256);
  __shared__ __align__(16) int8_t lds[2 * (A_BYTES + B_BYTES)];
  __shared__ __align__(16) float sScale[BN];
  __shared__ __align__(16) float sBias[BN];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int tile_n = blockIdx.x % p.tiles_n;
  const int tile_m = blockIdx.x / p.tiles_n;
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = tile_n * BN;
  const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

  // per-column constants of this tile
  for (int i = tid; i < BN; i += 256) {
    const int n = n0 + i;
    const bool ok = n < p.N;
    sScale[i] = ok ? p.s_a * p.s_b[n] : 0.f;
    sBias[i] = (ok && p.bias) ? p.bias[n] : 0.f;
  }

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
        const int z4 = zb4[i];
        v4i c0, c1;
        int lo, hi;
        lo = rb[i][0] & 0x0F0F0F0F; hi = (rb[i][0] >> 4) & 0x0F0F0F0F;
        c0[0] = ((lo | 0x80808080) - z4) ^ 0x80808080; c0[1] = ((hi | 0x80808080) - z4) ^ 0x80808080;
        lo = rb[i][1] & 0x0F0F0F0F; hi = (rb[i][1] >> 4) & 0x0F0F0F0F;
        c0[2] = ((lo | 0x80808080) - z4) ^ 0x80808080; c0[3] = ((hi | 0x80808080) - z4) ^ 0x80808080;
        lo = rb[i][2] & 0x0F0F0F0F; hi = (rb[i][2] >> 4) & 0x0F0F0F0F;
        c1[0] = ((lo | 0x80808080) - z4) ^ 0x80808080; c1[1] = ((hi | 0x80808080) - z4) ^ 0x80808080;
        lo = rb[i][3] & 0x0F0F0F0F; hi = (rb[i][3] >> 4) & 0x0F0F0F0F;
        c1[2] = ((lo | 0x80808080) - z4) ^ 0x80808080; c1[3] = ((hi | 0x80808080) - z4) ^ 0x80808080;
        *reinterpret_cast<v4i*>(lb + swz(row, 2 * pc)) = c0;
        *reinterpret_cast<v4i*>(lb + swz(row, 2 * pc + 1)) = c1;
      } else {
        *reinterpret_cast<v4i*>(lb + b_lds[i]) = rb[i];
      }
    }
  };

  // accumulators start at the zero-point corrections:
  //   true = sum a'w' + (a_off - z_a) * colsum_w[n] + (128 - z_w[n]) * rowsum_a'[m]   (second term only if centered)
  v16i acc[TN][TM];
  {
    const int lcol = lane & 31, lrow4 = (lane >> 5) * 4;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        int n = n0 + wn0 + j * 32 + 8 * (e >> 2) + lrow4 + (e & 3);
        n = n < p.N ? n : p.N - 1;
        const int cs = (p.da != 0 && p.colsum_b) ? p.da * p.colsum_b[n] : 0;
        const int dw = p.centered ? 128 - p.z_b[n] : 0;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          int64_t m = m0 + wm0 + i * 32 + lcol;
          m = m < p.M ? m : p.M - 1;
          acc[j][i][e] = cs + (p.centered ? dw * p.rowsum_a[m] : 0);
        }
      }
    }
  }

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

  // ---- epilogue: lane holds, for tile (j, i) and e-group g, output channels nb..nb+3 of token m ----
  const int lcol = lane & 31, lrow4 = (lane >> 5) * 4;
  const bool gated = p.act == RQ_ACT_SILU_GATED;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int64_t m = m0 + wm0 + i * 32 + lcol;
    if (m >= p.M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if (gated && (j & 1)) continue;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int nl = wn0 + j * 32 + 8 * g + lrow4;   // column within the tile
        const int n = n0 + nl;
        if (n >= p.N) continue;
        if (p.out_acc) {
          v4i t = {acc[j][i][4 * g], acc[j][i][4 * g + 1], acc[j][i][4 * g + 2], acc[j][i][4 * g + 3]};
          *reinterpret_cast<v4i*>(p.out_acc + m * p.ldacc + n) = t;
        }
        const float4 sc = *reinterpret_cast<const float4*>(&sScale[nl]);
        const float4 bi = *reinterpret_cast<const float4*>(&sBias[nl]);
        float y[4];
        y[0] = fmaf((float)acc[j][i][4 * g + 0], sc.x, bi.x);
        y[1] = fmaf((float)acc[j][i][4 * g + 1], sc.y, bi.y);
        y[2] = fmaf((float)acc[j][i][4 * g + 2], sc.z, bi.z);
        y[3] = fmaf((float)acc[j][i][4 * g + 3], sc.w, bi.w);
        int no = n;   // output column
        if (p.act == RQ_ACT_GELU) {
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] = gelu_f(y[e]);
        } else if (gated) {
          if (j + 1 < TN) {
            const float4 sc2 = *reinterpret_cast<const float4*>(&sScale[nl + 32]);
            const float4 bi2 = *reinterpret_cast<const float4*>(&sBias[nl + 32]);
            const float u0 = fmaf((float)acc[j + 1 < TN ? j + 1 : j][i][4 * g + 0], sc2.x, bi2.x);
            const float u1 = fmaf((float)acc[j + 1 < TN ? j + 1 : j][i][4 * g + 1], sc2.y, bi2.y);
            const float u2 = fmaf((float)acc[j + 1 < TN ? j + 1 : j][i][4 * g + 2], sc2.z, bi2.z);
            const float u3 = fmaf((float)acc[j + 1 < TN ? j + 1 : j][i][4 * g + 3], sc2.w, bi2.w);
            y[0] = silu_f(y[0]) * u0; y[1] = silu_f(y[1]) * u1; y[2] = silu_f(y[2]) * u2; y[3] = silu_f(y[3]) * u3;
          }
          no = (n0 + wn0 + j * 32) / 2 + 8 * g + lrow4;
        }
        if (p.residual) {
          const float4 r = *reinterpret_cast<const float4*>(p.residual + m * p.ldr + no);
          y[0] += r.x; y[1] += r.y; y[2] += r.z; y[3] += r.w;
        }
        if (p.out_f32) *reinterpret_cast<float4*>(p.out_f32 + m * p.ldf + no) = make_float4(y[0], y[1], y[2], y[3]);
        if (p.out_q) {
          const int sg = p.n_seg > 1 ? no / p.seg_len : 0;
          const float is = p.inv_so[sg], zz = p.zo[sg];
          const int lo = p.lo[sg], hi = p.hi[sg];
          int c[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            int k = (int)(__builtin_rintf(y[e] * is) + zz);
            c[e] = k < lo ? lo : (k > hi ? hi : k);
          }
          *reinterpret_cast<int*>(p.out_q + m * p.ldq + no) = rq_pack4(c[0], c[1], c[2], c[3]);
        }
      }
    }
  }
}

template <int BM, int BN, bool W4>
void launch_tile(rq_ctx* ctx, GemmParams& p) {
  const int64_t tiles_m = (p.M + BM - 1) / BM;
  p.tiles_n = (p.N + BN - 1) / BN;
  hipLaunchKernelGGL((qgemm_kernel<BM, BN, W4>), dim3((unsigned)(tiles_m * p.tiles_n)), dim3(256), 0, ctx->stream, p);
}

}  // namespace

static int g_gemm_tile = 0;   // 0: heuristic, 1: 128x128, 2: 256x128

extern "C" rq_status rq_set_gemm_tile(int32_t tile) {
  if (tile < 0 || tile > 2) return rq_fail(nullptr, RQ_ERR_INVALID_ARG, "rq_set_gemm_tile: %d not in 0..2", tile);
  g_gemm_tile = tile;
  return RQ_OK;
}

rq_status rq_launch_qgemm_weight(rq_ctx* ctx, const rq_gemm_desc* d) {
  GemmParams p;
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
    p.inv_so[i] = on ? 1.0f / d->s_o[i] : 0.f;
    p.zo[i] = on ? (float)(d->z_o[i] - d->off_o[i]) : 0.f;
    p.lo[i] = on ? -d->off_o[i] : 0;
    p.hi[i] = on ? (1 << d->bits_o) - 1 - d->off_o[i] : 0;
  }
  const bool w4 = d->b_format == RQ_W_U4;
  // Tile choice: the larger tile halves LDS traffic per MAC; the smaller one fills the chip on narrow outputs.
  const int64_t big_tiles = ((d->M + 255) / 256) * ((d->N + 127) / 128);
  const bool big = g_gemm_tile ? g_gemm_tile == 2 : big_tiles >= 2 * (int64_t)ctx->num_cu;
  if (big) {
    if (w4) launch_tile<256, 128, true>(ctx, p); else launch_tile<256, 128, false>(ctx, p);
  } else {
    if (w4) launch_tile<128, 128, true>(ctx, p); else launch_tile<128, 128, false>(ctx, p);
  }
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}
