/*
 * repquant.h -- C ABI of librepquant.so: the inference path of a transformer block after
 * RepQuant's scale reparameterization (arXiv 2402.05628), hand-written HIP for gfx950 (MI355X).
 *
 * Conventions shared by every call
 * --------------------------------
 *  - Plain C: no C++ types, no exceptions cross this boundary.
 *  - Every data pointer is a DEVICE pointer unless a field says "host".  Scalars travel by value.
 *  - The caller owns every buffer; the library never allocates outputs and never frees inputs.
 *    Scratch memory comes from a caller-provided workspace (rq_block_workspace_bytes).
 *  - Calls are asynchronous on the context's stream; nothing here synchronizes unless stated.
 *  - Arguments are validated before any GPU work is issued.  A context created with device < 0 is a
 *    "host-only" context: validation runs as usual and a valid call then returns RQ_ERR_UNSUPPORTED.
 *  - Matrices are row-major.  Leading dimensions (ld*) are in elements.  Weights are [out, in] with
 *    `in` contiguous, so every GEMM here is C[m, n] = sum_k A[m, k] * B[n, k].
 *  - Returns rq_status; rq_last_error() gives the text of the last failure on that context (or of the
 *    last failure of a call that had no context).
 *
 * Integer codes and their storage
 * -------------------------------
 *  The uniform quantizer (Section "Efficient quantizers") produces unsigned codes in [0, 2^b - 1] with
 *  an integer zero-point z.  The matrix cores multiply signed 8-bit integers, so an activation tensor is
 *  stored as int8 `code - off`, where the storage offset `off` is chosen by the producer so that the
 *  value fits (off = z whenever -128 <= -z and 2^b - 1 - z <= 127; off = 128 for 8-bit codes).  Every
 *  descriptor carries both z and off.  The contract of an integer matmul is the TRUE accumulator
 *      acc[m, n] = sum_k (qa[m, k] - z_a) * (qb[n, k] - z_b[n]),
 *  bit-exact; the kernels reach it from the stored operands with rank-1 corrections.
 *
 *  Weight formats (per-output-channel scale s_w[n] and zero-point z_w[n]):
 *    RQ_W_I8_BAKED     int8 [N, K], stored = code - z_w[n]          (b <= 7)
 *    RQ_W_I8_CENTERED  int8 [N, K], stored = code - 128             (b == 8); needs rowsum_a
 *    RQ_W_U4           uint8 [N, K/2], two raw 4-bit codes per byte (z_b[n] in 0..15), in the interleaved order
 *                      produced by rq_weight_quant_pack (see there); z_w[n] is subtracted while the
 *                      nibbles are unpacked in LDS.
 *  colsum_w[n] = sum_k (code[n, k] - z_w[n]) accompanies every format.
 */
#ifndef REPQUANT_H
#define REPQUANT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rq_ctx rq_ctx;

typedef enum {
  RQ_OK = 0,
  RQ_ERR_INVALID_ARG = 1, /* null pointer, bad enum, bad bit-width, non-positive scale, misalignment */
  RQ_ERR_SHAPE = 2,       /* sizes or leading dimensions inconsistent or beyond what the kernels support */
  RQ_ERR_UNSUPPORTED = 3, /* valid request that this build cannot run (e.g. host-only context) */
  RQ_ERR_WORKSPACE = 4,   /* workspace too small */
  RQ_ERR_HIP = 5          /* a HIP runtime call failed; text in rq_last_error */
} rq_status;

enum { RQ_NORM_LAYERNORM = 0, RQ_NORM_RMSNORM = 1 };
enum { RQ_ACT_NONE = 0, RQ_ACT_GELU = 1, RQ_ACT_SILU_GATED = 2 };
enum { RQ_MASK_NONE = 0, RQ_MASK_CAUSAL = 1 };
enum { RQ_W_I8_BAKED = 0, RQ_W_I8_CENTERED = 1, RQ_W_U4 = 2, RQ_B_ACT_I8 = 3 };
/* `flags` of the attention descriptors and of rq_block_params / rq_block_raw.
 * RQ_LOG_ZERO_AT_MAX_CODE: the log quantizer's de-quantizer (Section "Efficient quantizers", x^ = s 2^-q; Eq. (3.3-2)) is
 * silent on whether the saturated code 2^b - 1, which collects every probability below the grid, still carries mass.  By
 * default it is de-quantized literally like any other code; with this flag it de-quantizes to exactly 0 (every other code
 * unchanged).  The codes themselves do not depend on the flag. */
enum { RQ_LOG_ZERO_AT_MAX_CODE = 1 };

/* ---- context ---------------------------------------------------------------------------------- */

/* Creates a context bound to HIP device `device` and stream `hip_stream` (a hipStream_t, or NULL for
 * the default stream).  device < 0 creates a host-only context (validation only).  Host call. */
rq_status rq_create(rq_ctx** ctx, int device, void* hip_stream);
void rq_destroy(rq_ctx* ctx);
/* Host string owned by the library; valid until the next failing call on the same context/thread. */
const char* rq_last_error(const rq_ctx* ctx);
/* Storage offset the library's own producers use for codes with zero-point z at `bits` bits. */
int32_t rq_store_offset(int32_t bits, int32_t z);

/* ---- rq_reparam_fold ---------------------------------------------------------------------------
 * Section "Scale reparameterization for LayerNorm activations": channel-wise (s, z) of a LayerNorm
 * activation become ONE layer-wise pair, with the difference folded into the LayerNorm affine and
 * the next Linear:
 *    s~ = mean(s),  z~ = round(mean(z))  (an integer, so r2 is integral),  r1 = s / s~,  r2 = z - z~,
 *    gamma~ = gamma / r1,  beta~ = (beta + s.r2) / r1,
 *    W~[j, d] = r1[d] W[j, d],  b~[j] = b[j] - sum_d s[d] r2[d] W[j, d].
 * Section "Scale reparameterization for Softmax activations", Eq. (3.3-2): the log-sqrt2 scale s_log
 * becomes the pair {s_log (even codes), s_log*sqrt2 (odd codes)}.
 * All arithmetic is float64; outputs are rounded once to float32.  In-place (W_t == W etc.) is allowed.
 */
typedef struct {
  int32_t D;             /* channels of the LayerNorm activation (= K of the next Linear) */
  int32_t D_out;         /* output channels of the next Linear */
  const float* s_ch;     /* [D] channel scales, > 0 */
  const int32_t* z_ch;   /* [D] channel zero-points */
  const float* gamma;    /* [D] */
  const float* beta;     /* [D] or NULL (= 0) */
  const float* W;        /* [D_out, D] */
  const float* b;        /* [D_out] or NULL (= 0) */
  float s_log;           /* log-sqrt2 scale, > 0 (ignored when s_log_pair is NULL) */
  float* s_tilde;        /* [1] out */
  int32_t* z_tilde;      /* [1] out */
  float* gamma_t;        /* [D] out */
  float* beta_t;         /* [D] out */
  float* W_t;            /* [D_out, D] out */
  float* b_t;            /* [D_out] out */
  float* s_log_pair;     /* [2] out {s_log, s_log*sqrt2} or NULL */
} rq_fold_desc;
rq_status rq_reparam_fold(rq_ctx* ctx, const rq_fold_desc* d);

/* ---- rq_weight_quant_pack (helper) ---------------------------------------------------------------
 * Channel-wise (per output channel) min/max uniform quantization of a float weight matrix
 * (Section "Efficient quantizers", Eq. for s and z; granularity paragraph):
 *    s_w[n] = float32((max_n - min_n) / (2^b - 1)),  z_w[n] = round(-min_n / s_w[n]),
 *    code = clip(round(W / s_w[n]) + z_w[n], 0, 2^b - 1),
 * where min_n = min(row n, 0) and max_n = max(row n, 0): the zero-point is itself a code in [0, 2^b - 1], which the
 * formula gives exactly when the range contains 0, so a row whose weights all share one sign has its range extended
 * to 0 (z_w = 0 or 2^b - 1); a row of zeros gets s_w = 1.  (rq_qgemm subtracts z_w from packed 4-bit codes byte-wise:
 * z_w[n] outside 0..15 is not a valid RQ_W_U4 operand.)
 * bits = 8 -> RQ_W_I8_CENTERED, bits in 2..7 with format RQ_W_I8_BAKED, bits = 4 with RQ_W_U4.
 * RQ_W_U4 layout: row n holds K/2 bytes; within each aligned group of 8 codes k0..k7 the four bytes
 * are (k0 | k4<<4), (k1 | k5<<4), (k2 | k6<<4), (k3 | k7<<4), so that `dword & 0x0F0F0F0F` yields
 * k0..k3 and `(dword >> 4) & 0x0F0F0F0F` yields k4..k7 as bytes.  K must be a multiple of 8.
 * If gate_up_rows > 0 the input rows are [gate(0..Dm-1) ; up(0..Dm-1)] with Dm = gate_up_rows and the
 * output rows are interleaved in groups of 32 (32 gate rows, then the 32 matching up rows), the order
 * the fused SiLU(gate)*up epilogue of rq_qgemm expects; Dm must be a multiple of 32.
 */
typedef struct {
  int32_t N, K;
  int32_t bits;
  int32_t format;        /* RQ_W_* */
  int32_t gate_up_rows;  /* 0, or Dm for the gated-MLP interleave */
  const float* W;        /* [N, K] */
  const float* bias;     /* [N] or NULL; only permuted along with the rows into bias_out */
  void* w_out;           /* int8 [N, K] or uint8 [N, K/2] */
  float* s_w;            /* [N] out */
  int32_t* z_w;          /* [N] out */
  int32_t* colsum_w;     /* [N] out, sum_k (code - z_w) */
  float* bias_out;       /* [N] out or NULL */
} rq_wq_desc;
rq_status rq_weight_quant_pack(rq_ctx* ctx, const rq_wq_desc* d);

/* ---- rq_ln_quant ---------------------------------------------------------------------------------
 * LayerNorm (Eq. for X'_{n,:}) with the folded affine, fused with the layer-wise uniform quantizer:
 *    code = clip(round((xhat * gamma~ + beta~) / s~) + z~, 0, 2^b - 1),  stored as int8 code - store_off.
 * xhat = (x - mean) / sqrt(var + eps) (population variance) or x / sqrt(mean(x^2) + eps) for RMSNorm.
 * The row statistics are float64; the affine and the quantizer are float32 (pre-round error ~1e-5 of a code at up to 6
 * bits), and at 7 or 8 bits every value within 2^-11 of a rounding tie is decided again in float64, so such codes differ from
 * a float64 evaluation only at exact ties.  rowsum[t] = sum_d stored[t, d] (optional).
 * x and q must be 16-byte aligned, D a multiple of 4, ldx a multiple of 4, ldq a multiple of 4.
 */
typedef struct {
  int64_t T;
  int32_t D;
  int32_t norm_kind;
  double eps;
  const float* x;
  int64_t ldx;
  const float* gamma_t;  /* [D] */
  const float* beta_t;   /* [D] or NULL */
  float s_tilde;
  int32_t z_tilde;
  int32_t bits;          /* 2..8 */
  int32_t store_off;
  int8_t* q;             /* [T, D] out */
  int64_t ldq;
  int32_t* rowsum;       /* [T] out or NULL */
} rq_ln_desc;
rq_status rq_ln_quant(rq_ctx* ctx, const rq_ln_desc* d);

/* ---- rq_qgemm --------------------------------------------------------------------------------------
 * Integer matmul with both operands quantized (Section "Transformer blocks", last paragraph; uniform
 * de-quantizer of Section "Efficient quantizers" applied to both operands):
 *    acc[m, n] = sum_k (qa[m, k] - z_a)(qb[n, k] - z_b[n])            exact, int32
 *    y[m, n]   = s_a * s_b[n] * acc[m, n] + bias[n]                   float32
 *    y = act(y);  y += residual[m, n];  out_f32 = y;
 *    out_q = clip(round(y / s_o) + z_o, 0, 2^bits_o - 1) - off_o     (requantized for the next matmul)
 * Weight mode (b_format = RQ_W_*): batch fields must be 1/0.  s_b, z_b, colsum_b are [N] arrays.
 * Activation mode (b_format = RQ_B_ACT_I8, used for Q.K^T): B is int8 `code - b_off` with the scalar
 * pair (*s_b_scalar, z_b_scalar); problems are batched over (outer, inner) with element strides; only
 * out_acc is produced (the Softmax kernel consumes exact accumulators); K in {32, 64, 128, 256};
 * with causal != 0 tiles entirely above the diagonal are not written.
 * RQ_ACT_SILU_GATED: B rows are interleaved gate/up (see rq_weight_quant_pack), N = 2*Dm, outputs
 * have N/2 columns: SiLU(y_gate) * y_up.
 * Requant segments: column n (output column) uses entry n / seg_len of s_o/z_o/off_o (n_seg <= 4);
 * this is how one GEMM emits Q, K and V with their own static scales.
 * rowsum_a[m] = sum_k stored_a[m, k] is required for RQ_W_I8_CENTERED.  With RQ_W_U4 it is optional and, when given, must
 * be those sums as well: the kernel then multiplies the raw 4-bit codes and takes the zero-point term
 * -z_b[n] * rowsum_a[m] from it where that is faster (K >= 2048; same exact accumulators, fewer instructions per weight;
 * rq_ln_quant can emit the sums).
 * A, B 16-byte aligned; lda % 16 == 0; weight mode: K % 64 == 0, N % 4 == 0.
 */
typedef struct {
  int64_t M;
  int32_t N, K;
  const int8_t* A;
  int64_t lda;
  int32_t a_off, z_a;
  float s_a;
  const void* B;
  int64_t ldb;               /* elements (bytes for RQ_W_U4 rows: K/2) */
  int32_t b_format;
  const float* s_b;          /* [N] (weight mode) */
  const int32_t* z_b;        /* [N] (weight mode; may be NULL for RQ_W_I8_BAKED) */
  const int32_t* colsum_b;   /* [N] (weight mode; required when a_off != z_a) */
  const int32_t* rowsum_a;   /* [M] (required for RQ_W_I8_CENTERED; optional for RQ_W_U4, see above) */
  int32_t b_off, z_b_scalar; /* activation mode */
  const float* bias;         /* [N] or NULL */
  int32_t act;               /* RQ_ACT_* */
  const float* residual;     /* [M, N] or NULL */
  int64_t ldr;
  int32_t* out_acc;          /* [M, N] true accumulators, or NULL */
  int64_t ldacc;
  float* out_f32;            /* or NULL */
  int64_t ldf;
  int8_t* out_q;             /* or NULL */
  int64_t ldq;
  int32_t bits_o, n_seg, seg_len;
  float s_o[4];
  int32_t z_o[4];
  int32_t off_o[4];
  /* batching (activation mode) */
  int64_t batch_outer;       /* >= 1 */
  int32_t batch_inner;       /* >= 1 */
  int64_t a_stride_outer, a_stride_inner;
  int64_t b_stride_outer, b_stride_inner;
  int64_t acc_stride_group;  /* elements between consecutive groups (outer*batch_inner + inner) */
  int32_t causal;
} rq_gemm_desc;
rq_status rq_qgemm(rq_ctx* ctx, const rq_gemm_desc* d);
/* Tuning knob of one context (host call; not to be changed while another thread issues calls on the same context):
 * kernel of the weight mode. 0 = choose by shape (the pipelined kernel whenever N % 32 == 0;
 * its 320x128 tile instead of 256x128 for float+residual outputs when that finishes the busiest CU sooner),
 * 1 = simple 128x128, 2 = simple 256x128, 3 = pipelined; 4 .. 7 = pipelined with the 320- / 192- / 128- / 256-row tile
 * wherever the kernel has that tile (320: float + residual output; 192: both outputs; 128 and 256: re-quantized output);
 * 8 = pipelined with 256 x 256 tiles (re-quantized output: any weight storage; float + residual output: packed 4-bit
 * weights; chosen by shape for re-quantized products with M >= 2048 and K >= 2048 that give every CU two such tiles).
 * Adding 256 keeps the zero-point subtraction in the 4-bit unpack even when rowsum_a is given, adding 512 takes the raw
 * nibbles whenever it is given (by default only for K >= 2048, where it pays); same results either way. */
rq_status rq_set_gemm_tile(rq_ctx* ctx, int32_t tile);

/* rq_qgemm (weight mode, float output + residual) and rq_ln_quant of that output in ONE kernel whose workgroups own whole
 * output rows: xbar = GEMM + residual is written to d->out_f32 as usual and its normalized, quantized codes to ln->q
 * without being read back (block equations for X-bar followed by the LayerNorm of the MLP branch).  ln->x is ignored
 * (the input is the GEMM output); ln->T == d->M, ln->D == d->N.  Supported: RQ_W_U4 weights, N in {256, 512, 768}, no
 * activation, out_f32 the only GEMM output, codes of at most 6 bits, ln->rowsum NULL; RQ_ERR_UNSUPPORTED otherwise (the
 * caller then takes the two separate calls, which compute the same values up to the float32 order of summation of the
 * row statistics). */
rq_status rq_qgemm_ln_quant(rq_ctx* ctx, const rq_gemm_desc* d, const rq_ln_desc* ln);

/* ---- rq_softmax_log2_quant --------------------------------------------------------------------------
 * Softmax fused with the log-sqrt2 quantizer in its base-2 form (Eq. (3.3-1), second line):
 *    l[j]  = logit_scale * acc[j] (+ bias[g % H, i, j]);  masked j (causal: j > i) are excluded;
 *    code[j] = clip(round(-2 * log2(softmax(l)[j] / s_log)), 0, 2^b - 1),
 * evaluated as round(2 * (log2(sum_j 2^(l_j log2 e)) - l_j log2 e + log2 s_log)) in one pass over the
 * row held in registers: the probability itself is never formed.  Masked and padding positions
 * (j >= Nk up to ld) receive the largest code.  ld % 4 == 0, acc 16-byte aligned, codes 4-byte aligned.
 */
typedef struct {
  int64_t G;              /* number of (batch, head) groups */
  int32_t H;              /* heads: bias plane = g % H */
  int32_t Nq, Nk;
  int64_t ld;             /* row pitch (elements) of acc and of codes */
  const int32_t* acc;     /* [G, Nq, ld] exact accumulators of Q.K^T */
  double logit_scale;     /* s_q * s_k / sqrt(d_head) */
  const float* bias;      /* [H, Nq, Nk] dense, or NULL */
  int32_t mask;
  float s_log;
  int32_t bits;           /* 2..8 */
  uint8_t* codes;         /* [G, Nq, ld] out */
  int32_t flags;          /* RQ_LOG_*: accepted for symmetry with rq_attn_pv; the codes do not depend on them */
} rq_softmax_desc;
rq_status rq_softmax_log2_quant(rq_ctx* ctx, const rq_softmax_desc* d);

/* ---- rq_qk_softmax_log2_quant -----------------------------------------------------------------------
 * rq_qgemm in activation mode (exact int32 Q.K^T of the stored Q and K codes, attention Eq. of Section
 * "Transformer blocks") and rq_softmax_log2_quant (Eq. (3.3-1), second line) in ONE kernel: the logits are
 * never written.  Same integers and same code arithmetic as the two separate calls.  Rows of at most 288
 * keys keep the accumulators of a 32-query tile against all keys in registers.  Longer rows (up to 65536
 * keys, bias == NULL only) form the accumulators twice: a first sweep over the keys keeps a running integer
 * maximum and a running float32 sum per row, a second sweep emits the codes; only the order in which the
 * sum is accumulated differs from the separate calls.
 * Q, K: token-major device int8 (row b*N + i, column h*d_head + c, row pitch ld_tok bytes), stored as
 * code - off.  codes: [batch*H, N, ld] device, ld % 16 == 0, 16-byte aligned; positions N..ld-1 and masked
 * keys receive the largest code.  d_head in {32, 64, 128}; RQ_ERR_SHAPE if N > 288 with a bias, or N > 65536.
 */
typedef struct {
  int64_t batch;
  int32_t H, N, d_head;
  const int8_t *Q, *K;
  int64_t ld_tok;
  int32_t q_off, z_q, k_off, z_k;
  double logit_scale;     /* s_q * s_k / sqrt(d_head) */
  const float* bias;      /* [H, N, N] dense, or NULL */
  int32_t mask;
  float s_log;
  int32_t bits;           /* 2..8 */
  uint8_t* codes;
  int64_t ld;
} rq_qk_softmax_desc;
rq_status rq_qk_softmax_log2_quant(rq_ctx* ctx, const rq_qk_softmax_desc* d);

/* ---- rq_attn_fused ------------------------------------------------------------------------------------
 * rq_qk_softmax_log2_quant followed by rq_attn_pv in ONE kernel: the codes of a query tile's whole row stay
 * packed in registers and become the operand of the shift de-quantized P.V product (case analysis before
 * Eq. (3.3-2)), so neither the logits nor the codes travel through memory.  Same integers, same code arithmetic, same
 * output arithmetic as the separate calls.  Restrictions: no mask, N <= 288, d_head in {32, 64, 128}; without a bias
 * and with codes of at most 4 bits (one shift window: int8 matrix cores) every such N; with a bias and / or codes of 5
 * or 6 bits, rows of up to 160 keys (attention windows; wide codes take the bfloat16 matrix cores as in rq_attn_pv);
 * otherwise RQ_ERR_SHAPE and the caller takes the separate calls.  (The
 * 257 .. 288-key variants spill registers and are slower than the two separate calls, which rq_block_forward then
 * prefers.)  Q, K, V: token-major device int8 slices of one tensor
 * with row pitch ld_tok (stored code - off).  codes (optional, may be NULL): [batch*H, N, ld] as in
 * rq_qk_softmax_log2_quant.  Outputs as in rq_attn_pv: out_f32 and/or out_q, token-major [batch*N, H*d_head].
 */
typedef struct {
  int64_t batch;
  int32_t H, N, d_head;
  const int8_t *Q, *K, *V;
  int64_t ld_tok;
  int32_t q_off, z_q, k_off, z_k, v_off, z_v;
  double logit_scale;
  float s_log, s_v;
  int32_t bits_p;
  uint8_t* codes; int64_t ld;
  float* out_f32; int64_t ldf;
  int8_t* out_q; int64_t ldq;
  float s_o; int32_t z_o, off_o, bits_o;
  const float* bias;      /* [H, N, N] dense, or NULL */
  int32_t flags;          /* RQ_LOG_ZERO_AT_MAX_CODE or 0 */
} rq_attn_fused_desc;
rq_status rq_attn_fused(rq_ctx* ctx, const rq_attn_fused_desc* d);
/* 1 if rq_attn_fused supports the shape (host, no context needed). */
int32_t rq_attn_fused_supported(int32_t N, int32_t d_head, int32_t bits_p, int32_t has_bias);

/* ---- rq_attn_pv -----------------------------------------------------------------------------------------
 * P.V with shift de-quantized probabilities (case analysis before Eq. (3.3-2) and Eq. (3.3-2)):
 *    A^[i, j] = s~(code) * 2^floor(-code / 2),   s~ = s_log (even code) or s_log * sqrt2 (odd code),
 *    out[i, c] = sum_j A^[i, j] * s_v * (qv[j, c] - z_v),     masked j excluded.
 * The power of two is applied as an integer shift: each probability becomes -(128 >> k) in int8
 * (k = code >> 1 within a window of 8 shifts), the two parities accumulate separately in exact int32
 * on the matrix cores, and the two sums are combined once per output with s_log and s_log/sqrt2.
 * Codes wider than 4 bits span several windows: rows of up to 256 keys visit them one at a time (each window's exact
 * integer sum rounded once to float32); longer rows hand the powers of two (exact in bfloat16 whatever the shift) and
 * code - z_v (exact in bfloat16) to the bfloat16 matrix cores and accumulate in float32.
 * codes [batch*H, Nq, ld]; V is token-major int8 (row b*Nk + j, column h*d_head + c) stored code - v_off.
 * Outputs are token-major [batch*Nq, H*d_head].  d_head in {32, 64, 128}; ld % 16 == 0, ldv % 16 == 0, codes and V
 * 16-byte aligned (whole 16-byte pieces of the key rows are read).
 */
typedef struct {
  int64_t batch;
  int32_t H, Nq, Nk, d_head;
  int64_t ld;
  const uint8_t* codes;
  const int8_t* V;
  int64_t ldv;
  float s_log, s_v;
  int32_t z_v, v_off;
  int32_t bits_p;
  int32_t mask;
  float* out_f32;         /* or NULL */
  int64_t ldf;
  int8_t* out_q;          /* or NULL */
  int64_t ldq;
  float s_o;
  int32_t z_o, off_o, bits_o;
  int32_t flags;          /* RQ_LOG_ZERO_AT_MAX_CODE or 0 */
} rq_pv_desc;
rq_status rq_attn_pv(rq_ctx* ctx, const rq_pv_desc* d);

/* ---- rq_block_forward -------------------------------------------------------------------------------------
 * One transformer block (Eqs. for X-bar and Y, attention Eq.), every matmul operand quantized:
 *    a1 = ln_quant(x);  q,k,v = requant(qgemm(a1, W_qkv));  acc = q.k^T;  codes = softmax_log2_quant(acc);
 *    o = requant(attn_pv(codes, v));  xbar = qgemm(o, W_proj) + x;
 *    a2 = ln_quant(xbar);  h = requant(act(qgemm(a2, W_fc1)));  y = qgemm(h, W_fc2) + xbar.
 * x, y: float32 [batch*seq, D].  Attention groups are (batch item, head); for windowed attention pass
 * batch = images * windows and seq = tokens per window.
 */
typedef struct {
  int32_t N, K, bits, format;
  const void* w;
  const float* s_w;
  const int32_t* z_w;
  const int32_t* colsum_w;
  const float* bias;      /* [N] or NULL */
} rq_qlinear;

/* ---- GPTQ weight reconstruction on the folded weights (Algorithm 1, last step of every layer; Section "Sequential
 * Quantization Pipeline"; the method is the published GPTQ of Frantar et al., 2022) ----------------------------
 * Same outputs, formats and row permutation as rq_weight_quant_pack, and the same per-output-channel min/max grid,
 * but the codes are chosen column by column with second-order error compensation against the layer's calibration
 * inputs: H = A'^T A' + percdamp * mean(diag) * I with A' = stored + a_off - z_a (the integer part of the de-quantized
 * activation codes; the scale cancels), input channels that are always zero get H_jj = 1 and weight 0; with U the upper
 * Cholesky factor of H^-1, for j = 0 .. K-1: q_j = quantize(w_j), err = (w_j - dequant(q_j)) / U_jj,
 * W[:, j+1:] -= err (x) U[j, j+1:].  Float64 arithmetic; the Gram matrix is exact.
 *   W: device float32 [N, K];  A: device int8 [T, lda], the codes the preceding rq_ln_quant / rq_qgemm stored
 *   workspace: device, 256-byte aligned, rq_gptq_workspace_bytes(N, K, T) bytes
 * Errors: RQ_ERR_SHAPE (K not a multiple of 64 or above 8192, T outside 1..131071, lda < K, gate_up_rows),
 * RQ_ERR_INVALID_ARG (NULL / misaligned pointers, bits / format combination as for rq_weight_quant_pack, percdamp),
 * RQ_ERR_WORKSPACE. */
typedef struct {
  int32_t N, K;
  int32_t bits;
  int32_t format;        /* RQ_W_* */
  int32_t gate_up_rows;  /* 0, or Dm for the gated-MLP interleave */
  const float* W;        /* [N, K] */
  const float* bias;     /* [N] or NULL; only permuted along with the rows into bias_out */
  const int8_t* A;       /* [T, lda] stored activation codes */
  int64_t T, lda;
  int32_t a_off, z_a;
  double percdamp;       /* 0.01 in the published method */
  void* w_out;           /* int8 [N, K] or uint8 [N, K/2] */
  float* s_w;            /* [N] out */
  int32_t* z_w;          /* [N] out */
  int32_t* colsum_w;     /* [N] out */
  float* bias_out;       /* [N] out or NULL */
  void* workspace;
  size_t workspace_bytes;
} rq_gptq_desc;
size_t rq_gptq_workspace_bytes(int32_t N, int32_t K, int64_t T);
rq_status rq_gptq_quant_pack(rq_ctx* ctx, const rq_gptq_desc* d);

/* ---- per-channel dual clipping, learnt (Section "Per-channel dual clipping": Eqs. for X'_up and X'_low, the arg-min
 * Eq.; Section "Implementation details": Adam, 100 iterations, learning rate 0.01) ------------------------------
 * For every channel d of X' = norm(x) * gamma + beta  [T, D]:
 *   up = max_n X'[n,d] * Sigmoid(alpha1_d),  lo = min_n X'[n,d] * Sigmoid(alpha2_d),
 *   s = (up - lo) / (2^bits - 1),  z = round(-lo / s),  X'^ = s (clip(round(X'/s) + z, 0, 2^bits - 1) - z),
 * and (alpha1_d, alpha2_d) follow `iters` Adam steps (beta 0.9 / 0.999, eps 1e-8, bias-corrected) on
 * sum_n (X' - X'^)^2 from alpha1 = alpha2 = alpha0, the two roundings differentiated straight-through (derivative 1)
 * and the clip passing the gradient on [0, 2^bits - 1].  Float64 arithmetic throughout.  A channel whose maximum
 * equals its minimum is left at alpha0 with loss 0.
 *   x:          device float32 [T, ldx]; gamma == NULL means x already is X' (norm_kind, eps, beta ignored)
 *   gamma/beta: device float32 [D]; beta may be NULL (= 0)
 *   alpha1, alpha2: device float64 [D], out (required)
 *   clip_up, clip_lo: device float32 [D] or NULL, out: Sigmoid(alpha), the factors rq_block_calibrate takes
 *   up, lo, loss0, loss: device float64 [D] or NULL, out: the contracted bounds, the channel's sum of squares before
 *               the first and after the last step
 *   workspace:  device, at least rq_dual_clip_workspace_bytes(T) bytes, 16-byte aligned; unused when gamma == NULL
 * Errors: RQ_ERR_INVALID_ARG (NULL / misaligned pointers, bits outside 2..16, iters < 0, lr or eps not finite and
 * positive), RQ_ERR_SHAPE (T < 1, D < 1, ldx < D, D % 4 != 0 with gamma given), RQ_ERR_WORKSPACE. */
typedef struct {
  int64_t T;
  int32_t D;
  int64_t ldx;
  const float* x;
  int32_t norm_kind;
  double eps;
  const float* gamma;
  const float* beta;
  int32_t bits;
  int32_t iters;
  double lr;
  double alpha0;
  double* alpha1;
  double* alpha2;
  float* clip_up;
  float* clip_lo;
  double* up;
  double* lo;
  double* loss0;
  double* loss;
  void* workspace;
  size_t workspace_bytes;
  int32_t waves;         /* tuning: wavefronts per channel workgroup, 1..16; 0 chooses by shape.  The result does not
                            depend on it beyond the order of the sums. */
} rq_dual_clip_desc;
size_t rq_dual_clip_workspace_bytes(int64_t T);
rq_status rq_dual_clip_learn(rq_ctx* ctx, const rq_dual_clip_desc* d);

typedef struct {
  int32_t D, H, Dm;
  int32_t norm_kind, act, mask;
  int32_t bits_a, bits_p;
  double eps;
  const float *ln1_gamma_t, *ln1_beta_t;
  float ln1_s; int32_t ln1_z;
  rq_qlinear qkv;         /* N = 3D */
  float s_q, s_k, s_v; int32_t z_q, z_k, z_v;
  const float* rel_bias;  /* [H, seq, seq] or NULL */
  float s_log;
  float s_o; int32_t z_o;
  rq_qlinear proj;        /* N = D, K = D */
  const float *ln2_gamma_t, *ln2_beta_t;
  float ln2_s; int32_t ln2_z;
  rq_qlinear fc1;         /* N = Dm (GELU) or 2*Dm interleaved gate/up (SiLU gated) */
  float s_h; int32_t z_h;
  rq_qlinear fc2;         /* N = D, K = Dm */
  /* ---- options of the plan; 0 (a zero-filled struct) selects the default of each.  rq_block_workspace_bytes and
   * rq_block_forward read the same fields, so a workspace sized for these parameters fits their forward pass. ---- */
  int32_t attn_path;      /* RQ_ATTN_*: how attention runs */
  int32_t proj_ln_fused;  /* != 0: rq_qgemm_ln_quant for the output projection + second LayerNorm where it applies,
                             instead of rq_qgemm followed by rq_ln_quant.  Same float32 residual stream and same codes up
                             to the summation order of the row statistics; saves one read of the residual stream but runs
                             one 64-row tile per compute unit, and measures no faster on the ViT-B shape. */
  int64_t attn_chunk_bytes; /* where codes (and logits) travel through memory, attention runs in chunks of batch items so
                             that one chunk's scratch stays in the last-level cache between its kernels: the chunk budget
                             in bytes, at least 1 MiB; 0 = 64 MiB */
  int32_t flags;          /* RQ_LOG_ZERO_AT_MAX_CODE or 0 */
} rq_block_params;
/* rq_block_params.attn_path.  All three compute the same integers and the same codes (rows beyond 288 keys with
 * RQ_ATTN_QK_SOFTMAX_PV: up to the order in which the float32 row sum is accumulated).
 *   RQ_ATTN_AUTO:          rq_attn_fused where it applies (no mask, short rows; see there), else as RQ_ATTN_QK_SOFTMAX_PV;
 *   RQ_ATTN_QK_SOFTMAX_PV: rq_qk_softmax_log2_quant + rq_attn_pv wherever that call applies, else as RQ_ATTN_THREE_KERNELS;
 *   RQ_ATTN_THREE_KERNELS: rq_qgemm (activation mode) + rq_softmax_log2_quant + rq_attn_pv for every length. */
enum { RQ_ATTN_AUTO = 0, RQ_ATTN_QK_SOFTMAX_PV = 1, RQ_ATTN_THREE_KERNELS = 2 };
size_t rq_block_workspace_bytes(const rq_block_params* p, int64_t batch, int64_t seq);
/* Where the intermediates of rq_block_forward live inside the workspace (byte offsets from its start; host call, no
 * context).  After a forward pass (and a synchronization of the stream) the regions hold: a = the codes of the second
 * LayerNorm [T, D] (the first LayerNorm's codes were there before), qkv = the Q | K | V codes [T, 3D], o = the codes of the
 * attention output [T, D], xbar = the float32 residual stream after attention [T, D], hidden = the codes of the MLP hidden
 * layer [T, Dm], all stored as code - offset; logits (int32 [chunk*H, seq, ld]) and codes (uint8, same shape) hold the last
 * attention chunk and are empty (0 bytes) on the paths that keep them in registers.  batch_chunk = batch items per
 * attention chunk.  rq_block_calibrate_workspace_layout: the same for the calibration's own passes, which always run the
 * three separate attention kernels; `total` then includes the calibration's further scratch. */
typedef struct {
  int64_t batch_chunk, ld;
  size_t a, rowsum, qkv, logits, logits_bytes, codes, codes_bytes, o, xbar, hidden, total;
} rq_block_layout;
rq_status rq_block_workspace_layout(const rq_block_params* p, int64_t batch, int64_t seq, rq_block_layout* out);
rq_status rq_block_forward(rq_ctx* ctx, const rq_block_params* p, const float* x, float* y,
                           int64_t batch, int64_t seq, void* workspace, size_t workspace_bytes);

/* Streams of rq_block_forward (per context; host call, not to be changed while another thread issues calls on the same
 * context).  The context owns a second stream besides the caller's.  Where the whole attention runs as one kernel (no
 * attention scratch) and the batch is large (tokens x D >= 16 Mi elements, at least two batch items), the pass runs the two
 * halves of the batch side by side, one on each stream: the second stream waits for everything enqueued on the caller's
 * stream before the call, and the caller's stream waits for the second one before the call returns, so for the caller the
 * pass still is one piece of work on its stream (under stream capture: a fork and a join inside the captured graph).  Every
 * intermediate is token-major, so each half works in its own rows of the same workspace; the kernels and the output bits
 * are those of one stream.  What it buys: the tail of one half's kernel, with the chip running empty while the last tiles
 * finish, is filled by the other half's (CLIP ViT-L/14, batch 128: 2 - 3 % per pass; small workloads lose as much, hence
 * the size condition).  streams: 1 = always one stream; 2 = as described (default); 3 = two halves whenever the one-kernel
 * attention applies and batch >= 2 (tests).  Per-kernel profiling (rq_profile_enable) keeps the pass on one stream. */
rq_status rq_set_block_streams(rq_ctx* ctx, int32_t streams);

/* rq_block_forward for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same pass, same kernels and same results, with the scratch in a fixed device array
 * inside the library instead of a caller workspace.  The array holds RQ_NOALLOC_SCRATCH_BYTES on every GPU the library is
 * loaded on, until the process ends; its per-device address is resolved in rq_create.  The call allocates nothing and
 * frees nothing.  A shape whose plan (rq_block_workspace_bytes) exceeds the array is refused with RQ_ERR_WORKSPACE and a
 * message that names both sizes.  All calls on one GPU share that GPU's array: two calls that overlap in time on the same
 * GPU (different streams or threads) race; calls on one stream are ordered and need nothing cleared between them (every
 * byte a pass reads, it wrote before).  x and y stay caller buffers as in rq_block_forward. */
#define RQ_NOALLOC_SCRATCH_BYTES (32u << 20)
size_t rq_block_noalloc_scratch_bytes(void);
rq_status rq_block_forward_noalloc(rq_ctx* ctx, const rq_block_params* p, const float* x, float* y, int64_t batch, int64_t seq);

/* ---- block parameters as one flat blob ------------------------------------------------------------------------------
 * The folded and quantized parameters of a block (the result of rq_block_calibrate, or of the caller's own
 * preparation: the output of the reparameterization of Section "Scale reparameterization" and of the weight
 * quantizers) are checkpointed as ONE little-endian byte string, so that the preparation need not run again:
 *    rq_blob_header | arrays, each at the 256-byte aligned offset the header records
 * Array i of RQ_BLOB_ARRAYS: 0..3 = ln1_gamma_t, ln1_beta_t, ln2_gamma_t, ln2_beta_t (float32 [D]); then for each of
 * qkv, proj, fc1, fc2 (k = 0..3): 4+5k = w (int8 [N, K] or packed 4-bit [N, K/2]), 5+5k = s_w (float32 [N]),
 * 6+5k = z_w (int32 [N]), 7+5k = colsum_w (int32 [N]), 8+5k = bias (float32 [N]); 24 = rel_bias (float32, rel_bias_elems).
 * An absent (NULL) array has offset 0 and length 0.  Pointers inside rq_block_params never enter the blob.
 *
 * rq_block_blob_bytes: size of the blob of these parameters (host arithmetic only); 0 if p is NULL or inconsistent.
 * rq_block_blob_save:  copies the device arrays into blob_host (host memory of at least that size; pageable is fine) on
 *                      the context's stream and synchronizes it.  RQ_ERR_WORKSPACE if blob_bytes is too small.
 * rq_block_blob_check: validates a blob in host memory (magic, version, sizes, every offset and length against the shapes
 *                      in the header and against blob_bytes) without touching a device; *arena_bytes receives the device
 *                      memory rq_block_blob_load needs.  RQ_ERR_INVALID_ARG / RQ_ERR_SHAPE with text in rq_last_error(NULL).
 * rq_block_blob_load:  validates likewise, copies the blob to `arena_device` (caller-owned device memory, 256-byte
 *                      aligned, at least *arena_bytes; it must outlive every use of `out`), synchronizes, and fills `out`
 *                      with the scalars of the header and pointers into the arena.
 */
enum { RQ_BLOB_ARRAYS = 25, RQ_BLOB_VERSION = 1 };
typedef struct {
  char magic[8];                 /* "RQBLOCK\0" */
  uint32_t header_bytes;         /* sizeof(rq_blob_header) */
  uint32_t version;              /* RQ_BLOB_VERSION */
  uint64_t total_bytes;          /* header + arrays + padding */
  int32_t D, H, Dm, norm_kind, act, mask, bits_a, bits_p;
  double eps;
  float ln1_s, ln2_s, s_q, s_k, s_v, s_log, s_o, s_h;
  int32_t ln1_z, ln2_z, z_q, z_k, z_v, z_o, z_h;
  int32_t attn_path, proj_ln_fused, flags;
  int64_t attn_chunk_bytes;
  int32_t lin[4][4];             /* N, K, bits, format of qkv, proj, fc1, fc2 */
  int64_t rel_bias_elems;
  uint64_t off[RQ_BLOB_ARRAYS];  /* from the start of the blob */
  uint64_t len[RQ_BLOB_ARRAYS];  /* bytes */
} rq_blob_header;
size_t rq_block_blob_bytes(const rq_block_params* p, int64_t rel_bias_elems);
rq_status rq_block_blob_save(rq_ctx* ctx, const rq_block_params* p, int64_t rel_bias_elems, void* blob_host, size_t blob_bytes);
rq_status rq_block_blob_check(const void* blob_host, size_t blob_bytes, size_t* arena_bytes);
rq_status rq_block_blob_load(rq_ctx* ctx, const void* blob_host, size_t blob_bytes, void* arena_device, size_t arena_bytes,
                             rq_block_params* out);

/* Per-kernel timing of rq_block_forward: when enabled, every kernel launch inside rq_block_forward is
 * bracketed by HIP events on the context's stream.  rq_profile_read synchronizes the stream, writes up to
 * `cap` records (host arrays) accumulated since the last rq_profile_reset and returns their number.
 * step ids: see RQ_STEP_*. */
enum {
  RQ_STEP_LN1 = 0, RQ_STEP_QKV, RQ_STEP_QK, RQ_STEP_SOFTMAX, RQ_STEP_PV, RQ_STEP_PROJ,
  RQ_STEP_LN2, RQ_STEP_FC1, RQ_STEP_FC2, RQ_STEP_AUX, RQ_STEP_COUNT
};
rq_status rq_profile_enable(rq_ctx* ctx, int32_t on);
rq_status rq_profile_reset(rq_ctx* ctx);
int32_t rq_profile_read(rq_ctx* ctx, double* ms_total /* [RQ_STEP_COUNT] */, int64_t* launches /* [RQ_STEP_COUNT] */);

/* ---- calibration helpers (the step before the path; untimed preparation) -----------------------------------
 * rq_rowsum_i8:        rowsum[m] = sum_k A[m, k].
 * rq_ln_channel_minmax: per-channel min and max over all T tokens of LayerNorm(x) * gamma + beta
 *                      (the channel extremes of the Eqs. for X'_up and X'_low), float64 math and output
 *                      (cmin, cmax: device double [D]).
 * rq_minmax_f32:       min and max of a [rows, cols] float32 region -> out2[0], out2[1] (device double).
 * rq_block_calibrate:  Algorithm 1 restricted to one block: walks the block on one calibration batch, layer by
 *                      layer, each layer seeing the quantized layers before it; fills the caller-allocated
 *                      arrays named in rq_block_params and writes the scalar fields.  By default bounds are
 *                      min/max (times the given clip factors) and weights round-to-nearest; rq_block_raw can
 *                      switch on the learnt clipping and GPTQ.
 */
rq_status rq_rowsum_i8(rq_ctx* ctx, const int8_t* A, int64_t M, int32_t K, int64_t lda, int32_t* rowsum);
rq_status rq_ln_channel_minmax(rq_ctx* ctx, const float* x, int64_t T, int32_t D, int64_t ldx, int32_t norm_kind,
                               double eps, const float* gamma, const float* beta, double* cmin, double* cmax);
rq_status rq_minmax_f32(rq_ctx* ctx, const float* v, int64_t rows, int64_t cols, int64_t ld, double* out2);
/* Percentile variant of rq_ln_channel_minmax (Section "Implementation details": the default calibration strategy is
 * "Percentile"; no value is printed, so the fractions are arguments): for every channel of X' = norm(x) * gamma + beta
 * the q_lo-th and q_hi-th fractions of its T values, 0 <= q_lo <= q_hi <= 1, each interpolated linearly between the
 * order statistics floor(q (T - 1)) and the next one (exact selection, float64).  q_lo = 0, q_hi = 1 give min and max.
 * gamma == NULL means x already is X' (norm_kind, eps, beta ignored; any D).  lo, hi: device double [D].
 * workspace: device, 16 * T bytes, 16-byte aligned; unused when gamma == NULL. */
rq_status rq_ln_channel_percentile(rq_ctx* ctx, const float* x, int64_t T, int32_t D, int64_t ldx, int32_t norm_kind,
                                   double eps, const float* gamma, const float* beta, double q_lo, double q_hi,
                                   double* lo, double* hi, void* workspace, size_t workspace_bytes);

typedef struct {
  int32_t D, H, Dm;
  int32_t norm_kind, act, mask;
  int32_t bits_w, bits_a, bits_p;
  double eps;
  const float *ln1_gamma, *ln1_beta, *ln2_gamma, *ln2_beta;     /* [D]; beta may be NULL */
  const float *w_qkv, *b_qkv, *w_proj, *b_proj, *w_fc1, *b_fc1, *w_fc2, *b_fc2; /* biases may be NULL */
  const float *ln1_clip_up, *ln1_clip_lo, *ln2_clip_up, *ln2_clip_lo;           /* [D] or NULL (= 1) */
  const float* rel_bias;
  float s_log;
  /* Algorithm 1's two learning steps (both off when the fields are 0, the state after memset):
   * learn_clip_iters > 0: the clip factors of both LayerNorms are learnt by rq_dual_clip_learn (that many Adam
   *   iterations, learning rate learn_clip_lr, start learn_clip_alpha0) instead of being read from ln*_clip_up/lo;
   * gptq != 0: every Linear is quantized by rq_gptq_quant_pack against the codes it is fed (gptq_percdamp, 0.01 in the
   *   published method) instead of round-to-nearest; needs every K (D and Dm) a multiple of 64 and at most 8192. */
  int32_t learn_clip_iters;
  double learn_clip_lr;
  double learn_clip_alpha0;
  int32_t gptq;
  double gptq_percdamp;
  int64_t attn_chunk_bytes; /* chunk budget of the calibration's own attention passes, as in rq_block_params; 0 = 64 MiB */
  int32_t flags;            /* RQ_LOG_ZERO_AT_MAX_CODE or 0: enters the static scale of the attention output and is
                               copied to out->flags */
} rq_block_raw;

size_t rq_block_calibrate_workspace_bytes(const rq_block_raw* raw, int64_t batch, int64_t seq);
rq_status rq_block_calibrate_workspace_layout(const rq_block_raw* raw, int64_t batch, int64_t seq, rq_block_layout* out);
/* `out` arrives with every array pointer set to caller-allocated device memory of the documented size
 * (ln*_gamma_t/beta_t [D]; each rq_qlinear: w, s_w, z_w, colsum_w, bias); scalar fields are written.
 * Synchronizes the stream (scalars are read back to the host). */
rq_status rq_block_calibrate(rq_ctx* ctx, const rq_block_raw* raw, const float* x, int64_t batch, int64_t seq,
                             rq_block_params* out, void* workspace, size_t workspace_bytes);

#ifdef __cplusplus
}
#endif
#endif /* REPQUANT_H */
