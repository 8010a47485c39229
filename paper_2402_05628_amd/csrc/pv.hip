// rq_attn_pv: P.V with shift de-quantized log-sqrt2 probabilities
// (Section "Scale reparameterization for Softmax activations": case analysis before Eq. (3.3-2), Eq. (3.3-2)).
//
//   A^[i, j] = s~(code) * 2^floor(-code/2),  s~ = s (even code) | s*sqrt2 (odd code)
//            = s * 2^-k            (even, k = code >> 1)
//            = (s / sqrt2) * 2^-k  (odd,  k = code >> 1)
// The power of two is an integer shift: inside a window of 8 shifts the probability is the int8 value
// -(128 >> (k & 7)) = -2^(7 - k%8), looked up with one byte-permute per 4 codes.  Even and odd codes go to
// separate exact int32 accumulators on the int8 matrix cores (v_mfma_i32_32x32x32_i8); the parity scale is
// applied once per output.  Codes wider than 4 bits span several windows (k >= 8): shifts are then taken relative to
// the row's smallest shift (whose power of two multiplies the finished row), the windows of 8 relative shifts are
// visited one at a time, only if present, each contributing 2^(-8 w) times its exact integer sum, and relative shifts
// of 40 or more (below 2^-40 of the row's largest probability) are dropped.
// V^T is staged per 256 keys in LDS (transposed on the way in) as the ROW operand; the codes go straight from
// global memory into the COLUMN operand (each lane owns 16 consecutive keys of one query row), so a lane ends up
// with 4 consecutive channels of one token.
#include "rq_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct PvParams {
  const uint8_t* codes;
  const int8_t* V;
  int64_t ld, ldv;
  int H, Nq, Nk;
  int causal;
  int wmax;            // last window index: (2^bits - 1) >> 4
  double a_even, a_odd;   // s_log*s_v*(-1/128), s_log*s_v/sqrt2*(-1/128)
  int dv;              // v_off - z_v
  float* out_f32;
  int64_t ldf;
  int8_t* out_q;
  int64_t ldq;
  double inv_so;
  int zo, lo, hi;      // z_o - off_o, clamp bounds of the stored code
  int tiles_i;
  int num_cu;          // causal: every second round of workgroups walks its group's query tiles backwards
};

constexpr int JB = 256;          // keys staged per LDS block
constexpr int VT_PITCH = JB + 16;  // bytes per V^T row (skewed: 68 dwords -> conflict-free 16-byte reads)

// table of -(128 >> k), k = 0..7, as the 8 bytes {lo dword, hi dword} for v_perm_b32
constexpr unsigned TAB_LO = 0xF0E0C080u, TAB_HI = 0xFFFEFCF8u;

__device__ __forceinline__ unsigned byte_eq_mask(unsigned x, unsigned ref4) {
  // 0xFF in every byte of x equal to the matching byte of ref4 (bytes are < 0x80)
  const unsigned d = x ^ ref4;
  const unsigned nz = ((d + 0x7F7F7F7Fu) | d) & 0x80808080u;   // 0x80 where byte != 0
  const unsigned z = (~nz) & 0x80808080u;                      // 0x80 where byte == 0
  return (z >> 7) * 0xFFu;
}

template <int DH, bool WIDE>
__global__ __launch_bounds__(256) void pv_kernel(const PvParams p) {
  constexpr int TC = DH / 32;
  __shared__ __align__(16) int8_t vt[DH * VT_PITCH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int blocks_per_group = (p.tiles_i + 3) / 4;
  const int64_t g = blockIdx.x / blocks_per_group;
  // With a causal mask the work of a workgroup grows with its query tile.  Workgroups b and b + (number of CUs) tend to
  // share a CU, so every second round takes the tiles of its groups in reverse: a long one then sits next to a short one.
  int blk = blockIdx.x % blocks_per_group;
  if (p.causal && ((blockIdx.x / (unsigned)p.num_cu) & 1u)) blk = blocks_per_group - 1 - blk;
  const int it = blk * 4 + wave;
  const bool wave_live = it < p.tiles_i;
  const int64_t b = g / p.H;
  const int h = (int)(g % p.H);
  const int8_t* Vg = p.V + b * p.Nk * p.ldv + h * DH;
  const uint8_t* Cg = p.codes + g * p.Nq * p.ld;
  const int qi = it * 32 + l32;
  const int qi_ld = qi < p.Nq ? (wave_live ? qi : 0) : p.Nq - 1;
  const uint8_t* crow = Cg + (int64_t)qi_ld * p.ld;
  const int limit = p.causal ? (qi_ld + 1 < p.Nk ? qi_ld + 1 : p.Nk) : p.Nk;
  // keys this workgroup needs: up to the last row of its last tile when causal
  int blk_rows_end = (blk * 4 + 4) * 32;
  blk_rows_end = blk_rows_end < p.Nq ? blk_rows_end : p.Nq;
  const int nk_block = p.causal ? (blk_rows_end < p.Nk ? blk_rows_end : p.Nk) : p.Nk;
  int wave_rows_end = (it + 1) * 32;
  wave_rows_end = wave_rows_end < p.Nq ? wave_rows_end : p.Nq;
  const int nk_wave = wave_live ? (p.causal ? (wave_rows_end < p.Nk ? wave_rows_end : p.Nk) : p.Nk) : 0;

  // WIDE (codes wider than 4 bits): shifts are taken relative to the row's smallest one, kmin = min over valid keys of
  // code >> 1, and the power 2^-kmin is applied to the finished row.  Relative shifts of 40 or more (terms below 2^-40 of
  // the row's largest probability; at most 4096 of them) are dropped: their sum is below 4e-9 of the result.  Windows of
  // 8 relative shifts are visited one at a time, only if some row of the wavefront has a key in them.
  constexpr int WINDOWS = 5;
  int kmin = 0;
  unsigned kmin4 = 0;
  unsigned present = 1u;
  if (WIDE && wave_live) {
    int km = 127;
    for (int j0 = half * 16; j0 < nk_wave; j0 += 32) {
      const v4i cw = *reinterpret_cast<const v4i*>(crow + j0);
#pragma unroll
      for (int d4 = 0; d4 < 4; ++d4) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = j0 + d4 * 4 + e;
          const int k = (int)(((unsigned)cw[d4] >> (8 * e + 1)) & 0x7Fu);
          km = (j < limit && k < km) ? k : km;
        }
      }
    }
    const int other = __shfl_xor(km, 32, 64);      // the other half of the wavefront holds the other keys of the same row
    kmin = km < other ? km : other;
    kmin4 = (unsigned)kmin * 0x01010101u;
    unsigned pm = 0;
    for (int j0 = half * 16; j0 < nk_wave; j0 += 32) {
      const v4i cw = *reinterpret_cast<const v4i*>(crow + j0);
#pragma unroll
      for (int d4 = 0; d4 < 4; ++d4) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = j0 + d4 * 4 + e;
          const int kr = (int)(((unsigned)cw[d4] >> (8 * e + 1)) & 0x7Fu) - kmin;
          pm |= (j < limit && kr < 8 * WINDOWS) ? (1u << (kr >> 3)) : 0u;
        }
      }
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) pm |= __shfl_xor(pm, m, 64);
    present = pm;
  }
  present = __builtin_amdgcn_readfirstlane(present);

  // WIDE: per-window exact integer sums are folded into float64 running sums (each window has its own power of
  // two); otherwise one window, and the int32 accumulators simply run over all keys.
  // (float32 is enough: each window's exact integer sum is rounded once, to 2^-24 of itself, far inside the 1e-4 code budget)
  float outE[WIDE ? TC : 1][16], outO[WIDE ? TC : 1][16];
  double psE = 0.0, psO = 0.0;
  v16i E[TC], O[TC];
  int se = 0, so = 0;
#pragma unroll
  for (int c = 0; c < TC; ++c)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      E[c][e] = 0; O[c][e] = 0;
      if (WIDE) { outE[c][e] = 0.f; outO[c][e] = 0.f; }
    }

  for (int jb = 0; jb < nk_block; jb += JB) {
    __syncthreads();
    // ---- stage V^T for keys jb .. jb+JB-1: thread -> (4 keys, 4 channels), byte transpose in registers ----
    for (int id = tid; id < (JB / 4) * (DH / 4); id += 256) {
      const int j4 = id % (JB / 4), c4 = id / (JB / 4);
      unsigned r[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = jb + j4 * 4 + e;
        r[e] = j < p.Nk ? *reinterpret_cast<const unsigned*>(Vg + (int64_t)j * p.ldv + c4 * 4) : 0u;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const unsigned o = ((r[0] >> (8 * e)) & 0xFFu) | (((r[1] >> (8 * e)) & 0xFFu) << 8) |
                           (((r[2] >> (8 * e)) & 0xFFu) << 16) | (((r[3] >> (8 * e)) & 0xFFu) << 24);
        *reinterpret_cast<unsigned*>(vt + (c4 * 4 + e) * VT_PITCH + j4 * 4) = o;
      }
    }
    __syncthreads();
    if (jb >= nk_wave) continue;
    int jend = nk_wave - jb;
    jend = jend < JB ? jend : JB;
    // WIDE: this lane's codes of the whole block, requested together and once for all windows
    v4i cws[WIDE ? JB / 32 : 1];
    if (WIDE) {
#pragma unroll
      for (int t = 0; t < JB / 32; ++t) {
        const int j0 = jb + t * 32 + half * 16;
        cws[t] = (t * 32 < jend && j0 < p.ld) ? *reinterpret_cast<const v4i*>(crow + j0) : v4i{0, 0, 0, 0};
      }
    }
    for (int w = 0; w < (WIDE ? WINDOWS : 1); ++w) {
      if (WIDE && !((present >> w) & 1u)) continue;
      if (WIDE) {
#pragma unroll
        for (int c = 0; c < TC; ++c)
#pragma unroll
          for (int e = 0; e < 16; ++e) { E[c][e] = 0; O[c][e] = 0; }
        se = 0; so = 0;
      }
      const unsigned wref = (unsigned)w * 0x01010101u;
      // one key tile: its 16 codes per lane -> even / odd operands of this window -> the P.V products
      auto key_tile = [&](int js, const v4i& cw) {
        const int j0 = jb + js + half * 16;
        v4i pe, po;
#pragma unroll
        for (int d4 = 0; d4 < 4; ++d4) {
          // validity of the 4 keys j0+4*d4 .. +3 (padding and causal mask)
          int nv = limit - (j0 + d4 * 4);
          nv = nv < 0 ? 0 : (nv > 4 ? 4 : nv);
          const unsigned vm = nv == 4 ? 0xFFFFFFFFu : ((1u << (8 * nv)) - 1u);
          const unsigned c = (unsigned)cw[d4] | (WIDE ? ~vm : 0u);     // WIDE: invalid positions read as the largest code
          // per byte: relative shift (code >> 1) - kmin; no borrow between bytes because every byte is >= kmin
          const unsigned kr = WIDE ? ((c >> 1) & 0x7F7F7F7Fu) - kmin4 : (c >> 1);
          const unsigned sel = kr & 0x07070707u;
          unsigned pall = __builtin_amdgcn_perm(TAB_HI, TAB_LO, sel);
          if (WIDE) pall &= byte_eq_mask((kr >> 3) & 0x1F1F1F1Fu, wref);
          pall &= vm;
          const unsigned odd = (c & 0x01010101u) * 0xFFu;
          po[d4] = (int)(pall & odd);
          pe[d4] = (int)(pall & ~odd);
        }
        if (p.dv != 0) {
#pragma unroll
          for (int d4 = 0; d4 < 4; ++d4) {
            se = __builtin_amdgcn_sdot4(pe[d4], 0x01010101, se, false);
            so = __builtin_amdgcn_sdot4(po[d4], 0x01010101, so, false);
          }
        }
#pragma unroll
        for (int c = 0; c < TC; ++c) {
          const v4i fv = *reinterpret_cast<const v4i*>(vt + (c * 32 + l32) * VT_PITCH + js + half * 16);
          E[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fv, pe, E[c], 0, 0, 0);
          O[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fv, po, O[c], 0, 0, 0);
        }
      };
      if (WIDE) {
#pragma unroll
        for (int t = 0; t < JB / 32; ++t)
          if (t * 32 < jend) key_tile(t * 32, cws[t]);
      } else {
        for (int js = 0; js < jend; js += 32) {
          const int j0 = jb + js + half * 16;
          key_tile(js, j0 < p.ld ? *reinterpret_cast<const v4i*>(crow + j0) : v4i{0, 0, 0, 0});
        }
      }
      if (WIDE) {
        const float wsf = __builtin_ldexpf(1.0f, -8 * w);
        // the zero-point term dv * sum(p) is added to the integer sums BEFORE the conversion, so that the large
        // cancellation between the two happens exactly (all of it fits int32: |E| < 2^27, dv * sum(p) < 2^26)
        int ce = 0, co = 0;
        if (p.dv != 0) {     // uniform; the two halves of the wavefront saw different keys of the same row
          ce = p.dv * (se + __shfl_xor(se, 32, 64));
          co = p.dv * (so + __shfl_xor(so, 32, 64));
        }
#pragma unroll
        for (int c = 0; c < TC; ++c)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            outE[c][e] = fmaf((float)(E[c][e] + ce), wsf, outE[c][e]);
            outO[c][e] = fmaf((float)(O[c][e] + co), wsf, outO[c][e]);
          }
      }
    }
  }
  if (!WIDE) { psE = (double)se; psO = (double)so; }
  if (!wave_live) return;
  if (!WIDE && p.dv != 0) {   // the two halves of the wavefront saw different keys of the same row
    psE += __shfl_xor(psE, 32, 64);
    psO += __shfl_xor(psO, 32, 64);
  }
  if (qi >= p.Nq) return;
  const int64_t tok = b * p.Nq + qi;
  const double rowscale = WIDE ? __builtin_ldexp(1.0, -kmin) : 1.0;
  const double corr = WIDE ? 0.0 : (double)p.dv * (p.a_even * psE + p.a_odd * psO);
#pragma unroll
  for (int c = 0; c < TC; ++c) {
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const int col = h * DH + c * 32 + 8 * gq + half * 4;
      double y[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const double ve = WIDE ? (double)outE[WIDE ? c : 0][4 * gq + e] : (double)E[c][4 * gq + e];
        const double vo = WIDE ? (double)outO[WIDE ? c : 0][4 * gq + e] : (double)O[c][4 * gq + e];
        y[e] = (p.a_even * ve + p.a_odd * vo + corr) * rowscale;
      }
      if (p.out_f32)
        *reinterpret_cast<float4*>(p.out_f32 + tok * p.ldf + col) = make_float4((float)y[0], (float)y[1], (float)y[2], (float)y[3]);
      if (p.out_q) {
        int k[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          int q = (int)rint(y[e] * p.inv_so) + p.zo;
          k[e] = q < p.lo ? p.lo : (q > p.hi ? p.hi : q);
        }
        *reinterpret_cast<int*>(p.out_q + tok * p.ldq + col) = rq_pack4(k[0], k[1], k[2], k[3]);
      }
    }
  }
}

template <int DH>
void launch(rq_ctx* ctx, const PvParams& p, int64_t groups, bool wide) {
  const int blocks_per_group = (p.tiles_i + 3) / 4;
  const dim3 grid((unsigned)(groups * blocks_per_group));
  if (wide) hipLaunchKernelGGL((pv_kernel<DH, true>), grid, dim3(256), 0, ctx->stream, p);
  else hipLaunchKernelGGL((pv_kernel<DH, false>), grid, dim3(256), 0, ctx->stream, p);
}

}  // namespace

rq_status rq_launch_pv(rq_ctx* ctx, const rq_pv_desc* d) {
  PvParams p;
  p.codes = d->codes; p.V = d->V; p.ld = d->ld; p.ldv = d->ldv;
  p.H = d->H; p.Nq = d->Nq; p.Nk = d->Nk;
  p.causal = d->mask == RQ_MASK_CAUSAL;
  p.wmax = ((1 << d->bits_p) - 1) >> 4;
  const double ss = (double)d->s_log * (double)d->s_v;
  p.a_even = -ss / 128.0;
  p.a_odd = -ss / (128.0 * 1.4142135623730951);
  p.dv = d->v_off - d->z_v;
  p.out_f32 = d->out_f32; p.ldf = d->ldf; p.out_q = d->out_q; p.ldq = d->ldq;
  p.inv_so = d->out_q ? 1.0 / (double)d->s_o : 0.0;
  p.zo = d->z_o - d->off_o; p.lo = -d->off_o; p.hi = (1 << d->bits_o) - 1 - d->off_o;
  p.tiles_i = (d->Nq + 31) / 32;
  p.num_cu = ctx->num_cu > 0 ? ctx->num_cu : 256;
  const bool wide = d->bits_p > 4;
  const int64_t groups = d->batch * d->H;
  switch (d->d_head) {
    case 32: launch<32>(ctx, p, groups, wide); break;
    case 64: launch<64>(ctx, p, groups, wide); break;
    case 128: launch<128>(ctx, p, groups, wide); break;
    default: return rq_fail(ctx, RQ_ERR_SHAPE, "rq_attn_pv: d_head = %d must be 32, 64 or 128", d->d_head);
  }
  RQ_HIP(hipGetLastError());
  return RQ_OK;
}
