// rq_ln_quant: LayerNorm / RMSNorm with the folded affine, fused with the layer-wise uniform quantizer
// (Section "Scale reparameterization for LayerNorm activations"; quantizer of Section "Efficient quantizers").
//
// HBM-bound: 4 B read + 1 B written per element.  A row is held in the registers of LPR lanes (16, 32 or 64 lanes of
// a 64-wide wavefront, so that narrow rows still fill the wavefront); the row statistics are reduced with DPP lane
// exchanges inside 16-lane rows and one or two shuffles across them; the codes leave as one dword (4 codes) per
// lane, contiguous across lanes.  The per-channel constants g = gamma~/s~ and h = beta~/s~ + z~ are computed once
// per workgroup in float64 and staged in LDS as float32.  The row statistics are float64; the quantizer is two float32 fma
// per element; codes of 7 or 8 bits, whose float32 pre-round value carries up to ~5e-5 of a code of error, are decided
// again in float64 wherever that value lies within 2^-11 of a rounding tie (codes then agree with a float64 reference
// except at exact ties); rounding, saturation to 0..255 and byte packing are one v_cvt_pk_u8_f32 per code.  Small launches run one pass per workgroup with
// all workgroups resident; large ones use persistent workgroups that fetch their next rows while quantizing.
#include <vector>

#include "rq_internal.h"

namespace {

template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, true);
  return __hiloint2double(hi, lo);
}

// sum over the LPR lanes of a row group (LPR = 16, 32 or 64); every lane receives the total
template <int LPR>
__device__ __forceinline__ double group_sum(double v) {
  v += dpp_f64<0xB1>(v);    // quad_perm [1,0,3,2]: lane ^ 1
  v += dpp_f64<0x4E>(v);    // quad_perm [2,3,0,1]: lane ^ 2
  v += dpp_f64<0x141>(v);   // row_half_mirror: pairs the two quads of 8 lanes
  v += dpp_f64<0x140>(v);   // row_mirror: pairs the two halves of 16 lanes
  if (LPR >= 32) v += __shfl_xor(v, 16, 64);
  if (LPR >= 64) v += __shfl_xor(v, 32, 64);
  return v;
}

template <int LPR>
__device__ __forceinline__ int group_sum_i(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);
  if (LPR >= 32) v += __shfl_xor(v, 16, 64);
  if (LPR >= 64) v += __shfl_xor(v, 32, 64);
  return v;
}

// 1/sqrt(a) in float64: float32 estimate refined by two Newton steps (relative error ~1e-16)
__device__ __forceinline__ double rsqrt_f64(double a) {
  double r = (double)__builtin_amdgcn_rsqf((float)a);
  r = r * fma(-0.5 * a, r * r, 1.5);
  r = r * fma(-0.5 * a, r * r, 1.5);
  return r;
}

// wavefronts per SIMD the kernel is built for (bounds its registers): rows held in registers grow with NV
constexpr int ln_waves_per_simd(int nv, bool guard, bool persist) {
  return persist ? (nv <= 8 ? 2 : 1) : (nv <= 6 && !guard ? 7 : nv <= 8 ? 4 : nv <= 16 ? 2 : 1);
}
constexpr float TIE_GUARD = 1.0f / 2048.0f;

// The normalization and the quantizer run in float32, the row statistics in float64.  GUARD = false (codes of at most 6
// bits): the pre-round value is below 64, so its float32 error, ~1e-5 of a code, flips far fewer than 1e-4 of the codes.
// GUARD = true (7 or 8 bits): values within TIE_GUARD of a rounding tie are re-evaluated in float64, in the order of the
// definition (normalize, folded affine, divide by the scale as a product with g = gamma~ / s~, add z~).
// PERSIST: workgroups loop over rows and fetch the next rows early; otherwise one pass, fewer registers, more wavefronts.
template <int LPR, int NV, bool GUARD, bool PERSIST>
__global__ __launch_bounds__(256, ln_waves_per_simd(NV, GUARD, PERSIST)) void ln_quant_kernel(const float* __restrict__ x, int64_t ldx, int64_t T, int D, int norm_kind,
                                                       double eps, const float* __restrict__ gamma_t,
                                                       const float* __restrict__ beta_t, double inv_s, double zcode, float qmaxf,
                                                       unsigned off4, int8_t* __restrict__ q, int64_t ldq,
                                                       int32_t* __restrict__ rowsum) {
  extern __shared__ __align__(16) char gh_raw[];  // [D]: {gamma~ / s~, beta~ / s~ + z~} as float2
  float2* const ghf = reinterpret_cast<float2*>(gh_raw);
  constexpr int RPW = 64 / LPR;                   // rows per wavefront
  const int lane = threadIdx.x & 63;
  const int sub = lane % LPR;                     // lane within the row
  const int rsel = lane / LPR;                    // which of the wavefront's rows
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t nwave = (int64_t)gridDim.x * 4;
  const int chunks = D >> 2;

  for (int ch = threadIdx.x; ch < D; ch += 256) {
    const double g = (double)gamma_t[ch] * inv_s, h = (beta_t ? (double)beta_t[ch] * inv_s : 0.0) + zcode;
    ghf[ch] = make_float2((float)g, (float)h);
  }

  float4 cur[NV], nxt[PERSIST ? NV : 1];
  int64_t row = wave * RPW + rsel;
  const int64_t stride = nwave * RPW;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = sub + i * LPR;
    cur[i] = (row < T && c < chunks) ? *reinterpret_cast<const float4*>(x + row * ldx + c * 4) : make_float4(0, 0, 0, 0);
  }
  __syncthreads();
  const double invD = 1.0 / (double)D;
  for (; (row - rsel) < T; row += stride) {       // wavefront-uniform trip count
    const int64_t nrow = row + stride;
    if (PERSIST) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = sub + i * LPR;
        nxt[i] = (nrow < T && c < chunks) ? *reinterpret_cast<const float4*>(x + nrow * ldx + c * 4) : make_float4(0, 0, 0, 0);
      }
    }
    double s1 = 0.0, s2 = 0.0;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const double a = cur[i].x, b = cur[i].y, c = cur[i].z, d = cur[i].w;
      s1 += (a + b) + (c + d);
      s2 = fma(a, a, s2); s2 = fma(b, b, s2); s2 = fma(c, c, s2); s2 = fma(d, d, s2);
    }
    s2 = group_sum<LPR>(s2);
    double mean = 0.0, var = s2 * invD;
    if (norm_kind == RQ_NORM_LAYERNORM) {
      s1 = group_sum<LPR>(s1);
      mean = s1 * invD;
      var = fma(-mean, mean, var);
      var = var < 0.0 ? 0.0 : var;
    }
    const double rstd = rsqrt_f64(var + eps);
    const double nmr = -mean * rstd;
    const float rstd_f = (float)rstd, nmr_f = (float)nmr;
    int rs = 0;
    if (row < T) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = sub + i * LPR;
        if (c < chunks) {
          const float xv[4] = {cur[i].x, cur[i].y, cur[i].z, cur[i].w};
          unsigned w = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float2 g = ghf[c * 4 + e];
            float vf = fmaf(fmaf(xv[e], rstd_f, nmr_f), g.x, g.y);    // the packed convert below rounds to nearest-even
            if (GUARD && fabsf(vf - __builtin_rintf(vf)) > 0.5f - TIE_GUARD) {      // next to a tie: float64 decides
              const int ch = c * 4 + e;
              const double gd = (double)gamma_t[ch] * inv_s, hd = (beta_t ? (double)beta_t[ch] * inv_s : 0.0) + zcode;
              vf = (float)rint(fma(fma((double)xv[e], rstd, nmr), gd, hd));      // an exact integer: the float32 conversion is exact too
            }
            vf = fminf(vf, qmaxf);
            if (e == 0) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 0, w);  // saturates below at 0 and packs the byte
            if (e == 1) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 1, w);
            if (e == 2) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 2, w);
            if (e == 3) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 3, w);
          }
          // stored = code - off per byte, no borrow across bytes: ((w | H) - (o & ~H)) ^ ((w ^ ~o) & H)
          w = ((w | 0x80808080u) - (off4 & 0x7F7F7F7Fu)) ^ ((w ^ ~off4) & 0x80808080u);
          if (rowsum) rs = __builtin_amdgcn_sdot4((int)w, 0x01010101, rs, false);
          *reinterpret_cast<unsigned*>(q + row * ldq + c * 4) = w;
        }
      }
    }
    if (rowsum) {
      rs = group_sum_i<LPR>(rs);
      if (sub == 0 && row < T) rowsum[row] = rs;
    }
    if (!PERSIST) break;
#pragma unroll
    for (int i = 0; i < NV; ++i) cur[i] = nxt[PERSIST ? i : 0];
  }
}

// ---- wide rows, few of them: one workgroup per row ----------------------------------------------------------------------
// With wide rows (D >= 2048) and no more rows than the chip holds workgroups a few times over, the kernel above spends as
// long staging its per-channel constants (D channels per workgroup of 4 rows, behind a barrier) as on the rows.  Here a
// workgroup of 256 lanes owns ONE row: lane t holds the chunks t, t + 256, ... (NV float4), reduces the float64 statistics
// across the four wavefronts through LDS in a fixed order, then fetches gamma~ / beta~ of its own channels (cache hits:
// every workgroup reads the same 2 D floats), forms g = gamma~ / s~ and h = beta~ / s~ + z~ in registers (same float64
// products, same float32 values as the staged table) and quantizes from registers.  Nothing is staged, one barrier, and
// few enough registers that most rows of such a call are resident at once.  (Measured at 2048 x 4096: 23 us with the
// kernel above, 16 us with this one; a variant that walks several rows per workgroup with the constants kept in
// registers and the next row prefetched was slower, 19 us: fewer rows in flight.)
constexpr int row_wgs_per_cu(int nv) { return nv <= 2 ? 8 : nv <= 4 ? 6 : 3; }

template <int NV, bool GUARD>
__global__ __launch_bounds__(256, row_wgs_per_cu(NV)) void ln_quant_row_kernel(const float* __restrict__ x, int64_t ldx, int64_t T, int D, int norm_kind,
                                                           double eps, const float* __restrict__ gamma_t,
                                                           const float* __restrict__ beta_t, double inv_s, double zcode, float qmaxf,
                                                           unsigned off4, int8_t* __restrict__ q, int64_t ldq,
                                                           int32_t* __restrict__ rowsum) {
  __shared__ double part[2][4];
  __shared__ int part_i[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunks = D >> 2;
  const int64_t row = blockIdx.x;
  float4 xv[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = tid + i * 256;
    xv[i] = c < chunks ? *reinterpret_cast<const float4*>(x + row * ldx + c * 4) : make_float4(0, 0, 0, 0);
  }
  double s1 = 0.0, s2 = 0.0;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const double a = xv[i].x, b = xv[i].y, c = xv[i].z, d = xv[i].w;
    s1 += (a + b) + (c + d);
    s2 = fma(a, a, s2); s2 = fma(b, b, s2); s2 = fma(c, c, s2); s2 = fma(d, d, s2);
  }
  s1 = group_sum<64>(s1);
  s2 = group_sum<64>(s2);
  if (lane == 0) { part[0][wave] = s1; part[1][wave] = s2; }
  __syncthreads();
  s1 = (part[0][0] + part[0][1]) + (part[0][2] + part[0][3]);
  s2 = (part[1][0] + part[1][1]) + (part[1][2] + part[1][3]);
  const double invD = 1.0 / (double)D;
  double mean = 0.0, var = s2 * invD;
  if (norm_kind == RQ_NORM_LAYERNORM) {
    mean = s1 * invD;
    var = fma(-mean, mean, var);
    var = var < 0.0 ? 0.0 : var;
  }
  const double rstd = rsqrt_f64(var + eps);
  const double nmr = -mean * rstd;
  const float rstd_f = (float)rstd, nmr_f = (float)nmr;
  int rs = 0;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = tid + i * 256;
    if (c < chunks) {
      const float4 gv = *reinterpret_cast<const float4*>(gamma_t + c * 4);
      const float4 bv = beta_t ? *reinterpret_cast<const float4*>(beta_t + c * 4) : make_float4(0, 0, 0, 0);
      const float xe[4] = {xv[i].x, xv[i].y, xv[i].z, xv[i].w};
      const float ge[4] = {gv.x, gv.y, gv.z, gv.w};
      const float be[4] = {bv.x, bv.y, bv.z, bv.w};
      unsigned w = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const double gd = (double)ge[e] * inv_s, hd = (beta_t ? (double)be[e] * inv_s : 0.0) + zcode;
        float vf = fmaf(fmaf(xe[e], rstd_f, nmr_f), (float)gd, (float)hd);    // the packed convert below rounds to nearest-even
        if (GUARD && fabsf(vf - __builtin_rintf(vf)) > 0.5f - TIE_GUARD)     // next to a tie: float64 decides
          vf = (float)rint(fma(fma((double)xe[e], rstd, nmr), gd, hd));
        vf = fminf(vf, qmaxf);
        if (e == 0) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 0, w);
        if (e == 1) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 1, w);
        if (e == 2) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 2, w);
        if (e == 3) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 3, w);
      }
      w = ((w | 0x80808080u) - (off4 & 0x7F7F7F7Fu)) ^ ((w ^ ~off4) & 0x80808080u);      // stored = code - off per byte
      if (rowsum) rs = __builtin_amdgcn_sdot4((int)w, 0x01010101, rs, false);
      *reinterpret_cast<unsigned*>(q + row * ldq + c * 4) = w;
    }
  }
  if (rowsum) {      // kernel-uniform
    rs = group_sum_i<64>(rs);
    if (lane == 0) part_i[wave] = rs;
    __syncthreads();
    if (tid == 0) rowsum[row] = (part_i[0] + part_i[1]) + (part_i[2] + part_i[3]);
  }
}

template <int NV>
rq_status launch_row(rq_ctx* ctx, const rq_ln_desc* d, double inv_s, double zcode, float qmaxf, unsigned off4) {
  if (d->bits > 6)
    hipLaunchKernelGGL((ln_quant_row_kernel<NV, true>), dim3((unsigned)d->T), dim3(256), 0, ctx->stream, d->x, d->ldx, d->T, d->D,
                       d->norm_kind, d->eps, d->gamma_t, d->beta_t, inv_s, zcode, qmaxf, off4, d->q, d->ldq, d->rowsum);
  else
    hipLaunchKernelGGL((ln_quant_row_kernel<NV, false>), dim3((unsigned)d->T), dim3(256), 0, ctx->stream, d->x, d->ldx, d->T, d->D,
                       d->norm_kind, d->eps, d->gamma_t, d->beta_t, inv_s, zcode, qmaxf, off4, d->q, d->ldq, d->rowsum);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

// ---- many rows: rows travel through LDS without holding registers --------------------------------------------------------
// A kernel this simple is bound by how many bytes it keeps in flight.  The persistent kernel above prefetches its next
// rows into registers, which caps a CU at 8 wavefronts x 8 KB.  Here a wavefront owns one row at a time (64 lanes, NV
// float4 each) and a private two-slot ring in LDS: rows are requested with asynchronous global->LDS loads (each lane's 16
// bytes land at slot + 1 KiB * i + 16 * lane, and the same lane reads them back, so the ring is a per-lane FIFO without
// bank conflicts or barriers), two rows ahead, and cost no registers while they travel: 16 wavefronts per CU x 2 rows.
// Waiting for a row is a count of the wavefront's own younger memory operations (loads return in issue order): the next
// row's NV loads and the previous row's NV code stores may still be in flight, everything older has landed.
constexpr int ring_wgs_per_cu(int nv) { return nv <= 4 ? 4 : nv <= 6 ? 3 : 2; }      // by LDS (table + 8 nv KiB) and registers

template <int NV, bool GUARD>
__global__ __launch_bounds__(256, ring_wgs_per_cu(NV)) void ln_quant_ring_kernel(const float* __restrict__ x, int64_t ldx, int64_t T, int D, int norm_kind,
                                                               double eps, const float* __restrict__ gamma_t,
                                                               const float* __restrict__ beta_t, double inv_s, double zcode, float qmaxf,
                                                               unsigned off4, int8_t* __restrict__ q, int64_t ldq,
                                                               int32_t* __restrict__ rowsum) {
  extern __shared__ __align__(16) char ring_raw[];      // [D] float2 {gamma~ / s~, beta~ / s~ + z~}, then per wavefront 2 slots of NV KiB
  float2* const ghf = reinterpret_cast<float2*>(ring_raw);
  const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int chunks = D >> 2;
  char* const slots = ring_raw + (size_t)D * 8 + (size_t)wv * (2 * NV * 1024);
  for (int ch = threadIdx.x; ch < D; ch += 256) {
    const double g = (double)gamma_t[ch] * inv_s, h = (beta_t ? (double)beta_t[ch] * inv_s : 0.0) + zcode;
    ghf[ch] = make_float2((float)g, (float)h);
  }
  const int64_t stride = (int64_t)gridDim.x * 4;
  int64_t row = (int64_t)blockIdx.x * 4 + wv;
  // request row r into slot k (rows past the end re-read the last row: every request is the same NV loads)
  auto request = [&](int64_t r, int k) {
    const float* src = x + (r < T ? r : T - 1) * ldx;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = lane + i * 64;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + (c < chunks ? c : 0) * 4),
                                       (__attribute__((address_space(3))) void*)(slots + k * (NV * 1024) + i * 1024), 16, 0, 0);
    }
  };
  request(row, 0);
  request(row + stride, 1);
  __syncthreads();      // the constant table
  const double invD = 1.0 / (double)D;
  bool first = true;
  for (int k = 0; row < T; row += stride, k ^= 1) {      // wavefront-uniform
    // younger than this row's loads: the next row's NV loads, and (from the second turn on) the last row's NV code stores
    if (first) __builtin_amdgcn_s_waitcnt((NV & 0xF) | ((NV >> 4) << 14) | 0x0F70);
    else __builtin_amdgcn_s_waitcnt(((2 * NV) & 0xF) | (((2 * NV) >> 4) << 14) | 0x0F70);
    first = false;
    float4 cur[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const float4 v = *reinterpret_cast<const float4*>(slots + k * (NV * 1024) + i * 1024 + lane * 16);
      cur[i] = lane + i * 64 < chunks ? v : make_float4(0, 0, 0, 0);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // the slot is read: it may be refilled
    request(row + 2 * stride, k);
    double s1 = 0.0, s2 = 0.0;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const double a = cur[i].x, b = cur[i].y, c = cur[i].z, d = cur[i].w;
      s1 += (a + b) + (c + d);
      s2 = fma(a, a, s2); s2 = fma(b, b, s2); s2 = fma(c, c, s2); s2 = fma(d, d, s2);
    }
    s2 = group_sum<64>(s2);
    double mean = 0.0, var = s2 * invD;
    if (norm_kind == RQ_NORM_LAYERNORM) {
      s1 = group_sum<64>(s1);
      mean = s1 * invD;
      var = fma(-mean, mean, var);
      var = var < 0.0 ? 0.0 : var;
    }
    const double rstd = rsqrt_f64(var + eps);
    const double nmr = -mean * rstd;
    const float rstd_f = (float)rstd, nmr_f = (float)nmr;
    int rs = 0;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = lane + i * 64;
      const float xv[4] = {cur[i].x, cur[i].y, cur[i].z, cur[i].w};
      unsigned w = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float2 g = ghf[(c < chunks ? c : 0) * 4 + e];
        float vf = fmaf(fmaf(xv[e], rstd_f, nmr_f), g.x, g.y);    // the packed convert below rounds to nearest-even
        if (GUARD && c < chunks && fabsf(vf - __builtin_rintf(vf)) > 0.5f - TIE_GUARD) {      // next to a tie: float64 decides
          const int ch = c * 4 + e;
          const double gd = (double)gamma_t[ch] * inv_s, hd = (beta_t ? (double)beta_t[ch] * inv_s : 0.0) + zcode;
          vf = (float)rint(fma(fma((double)xv[e], rstd, nmr), gd, hd));
        }
        vf = fminf(vf, qmaxf);
        if (e == 0) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 0, w);
        if (e == 1) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 1, w);
        if (e == 2) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 2, w);
        if (e == 3) w = __builtin_amdgcn_cvt_pk_u8_f32(vf, 3, w);
      }
      w = ((w | 0x80808080u) - (off4 & 0x7F7F7F7Fu)) ^ ((w ^ ~off4) & 0x80808080u);      // stored = code - off per byte
      if (c < chunks) {
        if (rowsum) rs = __builtin_amdgcn_sdot4((int)w, 0x01010101, rs, false);
        *reinterpret_cast<unsigned*>(q + row * ldq + c * 4) = w;      // one store instruction per i: the wait above counts on it
      }
    }
    if (rowsum) {
      rs = group_sum_i<64>(rs);
      if (lane == 0) rowsum[row] = rs;
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);      // no request may outlive the workgroup's LDS
}

constexpr int ring_lds_bytes(int D, int nv) { return D * 8 + 4 * 2 * nv * 1024; }

template <int NV>
rq_status launch_ring(rq_ctx* ctx, const rq_ln_desc* d, double inv_s, double zcode, float qmaxf, unsigned off4) {
  const int lds = ring_lds_bytes(d->D, NV);
  int per_cu = (160 * 1024) / lds;
  per_cu = per_cu > ring_wgs_per_cu(NV) ? ring_wgs_per_cu(NV) : (per_cu < 1 ? 1 : per_cu);
  const int64_t blocks = (d->T + 3) / 4;
  const int64_t cap = (int64_t)ctx->num_cu * per_cu;
  const unsigned grid = (unsigned)(blocks < cap ? blocks : cap);
#define RQ_LN_RING(G)                                                                                                              \
  do {                                                                                                                             \
    static rq_once_per_device lds_attr;                                                                                            \
    RQ_HIP(rq_allow_dynamic_lds(ctx, lds_attr, reinterpret_cast<const void*>(&ln_quant_ring_kernel<NV, G>), 8192 * 8 + 64 * 1024)); \
    hipLaunchKernelGGL((ln_quant_ring_kernel<NV, G>), dim3(grid), dim3(256), lds, ctx->stream, d->x, d->ldx, d->T, d->D,           \
                       d->norm_kind, d->eps, d->gamma_t, d->beta_t, inv_s, zcode, qmaxf, off4, d->q, d->ldq, d->rowsum);          \
  } while (0)
  if (d->bits > 6) RQ_LN_RING(true);
  else RQ_LN_RING(false);
#undef RQ_LN_RING
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

template <int LPR, int NV, bool GUARD, bool PERSIST>
rq_status launch_one(rq_ctx* ctx, const rq_ln_desc* d, int64_t blocks, int lds, double inv_s, double zcode, float qmaxf, unsigned off4) {
  static rq_once_per_device lds_attr;
  RQ_HIP(rq_allow_dynamic_lds(ctx, lds_attr, reinterpret_cast<const void*>(&ln_quant_kernel<LPR, NV, GUARD, PERSIST>), 8192 * 8));
  hipLaunchKernelGGL((ln_quant_kernel<LPR, NV, GUARD, PERSIST>), dim3((unsigned)blocks), dim3(256), lds, ctx->stream, d->x, d->ldx, d->T,
                     d->D, d->norm_kind, d->eps, d->gamma_t, d->beta_t, inv_s, zcode, qmaxf, off4, d->q, d->ldq, d->rowsum);
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}

template <int LPR, int NV>
rq_status launch(rq_ctx* ctx, const rq_ln_desc* d, double inv_s, double zcode, float qmaxf, unsigned off4) {
  constexpr int RPW = 64 / LPR;
  const int64_t rows_per_block = 4 * RPW;
  const int64_t blocks = (d->T + rows_per_block - 1) / rows_per_block;
  const bool guard = d->bits > 6;
  const int lds = d->D * 8;
  // one pass per workgroup while every workgroup can be resident at once (7 per CU: the kernel is built for 7 wavefronts
  // per SIMD; LDS permitting);
  // beyond that, persistent workgroups that prefetch their next rows
  const int by_lds = lds > 0 ? (160 * 1024) / lds : 8;
  const int by_regs = ln_waves_per_simd(NV, guard, false);
  const int64_t one_pass_slots = (int64_t)ctx->num_cu * (by_lds < by_regs ? by_lds : by_regs);
  if (blocks <= one_pass_slots) {
    return guard ? launch_one<LPR, NV, true, false>(ctx, d, blocks, lds, inv_s, zcode, qmaxf, off4)
                 : launch_one<LPR, NV, false, false>(ctx, d, blocks, lds, inv_s, zcode, qmaxf, off4);
  }
  const int per_cu = by_lds < 4 ? (by_lds < 1 ? 1 : by_lds) : 4;
  const int64_t cap = (int64_t)ctx->num_cu * per_cu;
  return guard ? launch_one<LPR, NV, true, true>(ctx, d, cap, lds, inv_s, zcode, qmaxf, off4)
               : launch_one<LPR, NV, false, true>(ctx, d, cap, lds, inv_s, zcode, qmaxf, off4);
}

}  // namespace

rq_status rq_launch_ln_quant(rq_ctx* ctx, const rq_ln_desc* d) {
  const int chunks = d->D / 4;
  const double inv_s = 1.0 / (double)d->s_tilde;
  const double zcode = (double)d->z_tilde;
  const float qmaxf = (float)((1 << d->bits) - 1);
  const unsigned off4 = (unsigned)(d->store_off & 0xFF) * 0x01010101u;
  // wide rows, no more of them than the chip holds such workgroups at once (8 per CU) twice over: one workgroup per row
  const bool affine_aligned = reinterpret_cast<uintptr_t>(d->gamma_t) % 16 == 0 && reinterpret_cast<uintptr_t>(d->beta_t) % 16 == 0;
  if (chunks >= 512 && d->T <= (int64_t)ctx->num_cu * 16 && affine_aligned) {      // (its lanes read gamma~ / beta~ as float4)
    const int nvr = (chunks + 255) / 256;
    if (nvr <= 2) return launch_row<2>(ctx, d, inv_s, zcode, qmaxf, off4);
    if (nvr <= 4) return launch_row<4>(ctx, d, inv_s, zcode, qmaxf, off4);
    if (nvr <= 8) return launch_row<8>(ctx, d, inv_s, zcode, qmaxf, off4);
  }
  // many rows of 2 .. 8 KiB: the LDS-ring kernel, once its wavefronts (16 per CU) have at least six rows each -- with
  // fewer the ring never reaches its steady state and the register kernel's all-rows-at-once pass is faster (12 608 x 768:
  // 13.4 us against 15.6 us; 32 896 x 1024: 36.1 against 34.8 us)
  if (chunks >= 128 && chunks <= 512 && d->T >= (int64_t)ctx->num_cu * 96) {
    const int nvr = (chunks + 63) / 64;
    if (nvr <= 2) return launch_ring<2>(ctx, d, inv_s, zcode, qmaxf, off4);
    if (nvr <= 3) return launch_ring<3>(ctx, d, inv_s, zcode, qmaxf, off4);
    if (nvr <= 4) return launch_ring<4>(ctx, d, inv_s, zcode, qmaxf, off4);
    if (nvr <= 6) return launch_ring<6>(ctx, d, inv_s, zcode, qmaxf, off4);
    return launch_ring<8>(ctx, d, inv_s, zcode, qmaxf, off4);
  }
  // lanes per row: the smallest group that keeps a row within 8 float4 per lane
  int lpr = 64;
  for (int cand : {32, 16})
    if ((chunks + cand - 1) / cand <= 8) lpr = cand;
  const int nv = (chunks + lpr - 1) / lpr;
#define RQ_LN_CASE(L, N) \
  if (lpr == L && nv <= N) return launch<L, N>(ctx, d, inv_s, zcode, qmaxf, off4);
  RQ_LN_CASE(16, 1) RQ_LN_CASE(16, 2) RQ_LN_CASE(16, 3) RQ_LN_CASE(16, 4) RQ_LN_CASE(16, 6) RQ_LN_CASE(16, 8)
  RQ_LN_CASE(32, 5) RQ_LN_CASE(32, 6) RQ_LN_CASE(32, 7) RQ_LN_CASE(32, 8)
  RQ_LN_CASE(64, 5) RQ_LN_CASE(64, 6) RQ_LN_CASE(64, 8) RQ_LN_CASE(64, 12) RQ_LN_CASE(64, 16) RQ_LN_CASE(64, 32)
#undef RQ_LN_CASE
  return rq_fail(ctx, RQ_ERR_SHAPE, "rq_ln_quant: D = %d exceeds the supported 8192", d->D);
}
