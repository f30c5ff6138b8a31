/*
 * qvggt — W4A4 Dual-Smoothed Fine-Grained Quantization (DSFQ) linear layer for AMD MI355X (gfx950).
 *
 * C ABI of the inference hot path of the quantized linear layer of QuantVGGT
 * (arXiv 2509.21302, Sec. 3.2 "Dual-Smoothed Fine-Grained Quantization"):
 *
 *     Y = dequant( Q_token( X H diag(c)^-1 ) . Q_channel( diag(c) H^T W^T ) ) + b
 *
 * with H a randomised orthonormal Walsh-Hadamard matrix (Sec. 3.2, Pre-Global-Rotation),
 * c the post-rotation smoothing factor (Sec. 3.2, Post-Local-Smooth, Eq. "smooth_factor"),
 * Q the symmetric 4-bit quantizer (Sec. 3.1.2, Eq. "quantization") applied per token to
 * activations and per output channel to weights (Sec. 3.2, Fine-Grained Quantization
 * Granularity), the product taken in integers and dequantised after the sum.
 *
 * General conventions
 *   - Every pointer is a DEVICE pointer owned by the caller unless stated otherwise; the
 *     library allocates nothing and is re-entrant.  The only thing it remembers between calls is
 *     on which devices qvggt_init has run (see there).
 *   - Every call only enqueues kernels on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and returns; buffers must stay valid until the stream has run.
 *     Calls may be recorded into a HIP graph (stream capture) once qvggt_init has run on the device.
 *   - Matrices are dense row-major.  bf16 values are IEEE bfloat16 bit patterns (uint16).
 *   - K (input features, the Hadamard size) must be a power of two in [128, 8192], or one of the sizes
 *     2^n * m with a Paley matrix as the m-point factor (Sec. 3.2, H_d = H_{2^n} (x) H_m): m = 12: 768, 1536, 3072, 6144;
 *     m = 20: 1280, 2560, 5120; m = 28: 1792, 3584 (type I from GF(11), GF(19), type II from GF(13));
 *     N (output features) a multiple of 16; M (tokens) any value >= 0 (M == 0 is a no-op).
 *     All device pointers must be 16-byte aligned.  Inputs must be finite.
 *   - Return value: QVGGT_OK or an error code; arguments are validated on the host
 *     before anything is launched, so a failed call has touched no output.
 *   - Packed 4-bit buffers (Xq, Wq) hold two's-complement codes, two per byte, rows of K/2
 *     bytes.  The position of a code inside its row is the library's choice (a fixed
 *     permutation of 0..K-1 that depends only on K, the same for Xq and Wq, so the integer
 *     dot products are unaffected); qvggt_pack_int4 / qvggt_unpack_int4 convert between this
 *     layout and plain int8 codes in natural order and are the only supported way to read
 *     or write such buffers from outside.  For reference, the permutation is the identity except
 *     for K = 1024, 2048 and 4096, where natural channel e = 128 hb + 32 nt + c (c < 32, nt < 4)
 *     sits at position c (K / 32) + nt + 4 hb', with hb' = hb except at K = 4096, where bits 3 and
 *     4 of hb change places (the order in which the matrix-core rotation kernel holds a token);
 *     position p is the low nibble of byte p / 2 for even p, the high nibble for odd p.
 */
#ifndef QVGGT_H
#define QVGGT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QVGGT_OK = 0,
    QVGGT_ERR_NULL = 1,      /* a required pointer is NULL */
    QVGGT_ERR_SHAPE = 2,     /* M < 0, N < 16 or not a multiple of 16, K not one of the supported sizes */
    QVGGT_ERR_ALIGN = 3,     /* a pointer is not 16-byte aligned */
    QVGGT_ERR_DTYPE = 4,     /* dtype is neither QVGGT_BF16 nor QVGGT_F32 */
    QVGGT_ERR_WORKSPACE = 5, /* workspace smaller than qvggt_workspace_bytes() */
    QVGGT_ERR_ARG = 6,       /* a scalar argument outside its documented range (alpha, p, eps, flags, bits) */
    QVGGT_ERR_HIP = 7        /* a kernel launch failed (hipGetLastError) */
} qvggt_status;

typedef enum { QVGGT_BF16 = 0, QVGGT_F32 = 1 } qvggt_dtype;

/* Human-readable name of a status code (host pointer to a static string). */
const char *qvggt_status_string(int status);

/*
 * Per-device set-up for the calling thread's current device: raises the dynamic-LDS limit of the library's GEMM kernels
 * there (hipFuncSetAttribute; their tiles need up to 160 KB of LDS, more than a launch gets by default).  Enqueues nothing.
 * Every entry point that launches such a kernel runs the same set-up by itself the first time it is used on a device, so
 * calling qvggt_init is optional; call it once per device before recording calls into a HIP graph, so that the capture holds
 * launches only.  Safe to call from several threads and more than once.  QVGGT_OK or QVGGT_ERR_HIP (no usable device).
 */
int qvggt_init(void);

/*
 * Per-channel activation statistic of the smoothing factor, taken in rotated space
 * (Sec. 3.2, Eq. "smooth_factor", numerator):
 *     absmax_rot[j] = max_t | (X_cal H)[t, j] |,   H = diag(signs) . Hhat_K
 * X_cal: [M, K] calibration activations (bf16 or f32).  signs: int8 [K] of +1/-1 applied to
 * the INPUT channels before the transform, or NULL for the plain Hadamard.  absmax_rot: f32 [K],
 * overwritten.  (The paper writes H = Hhat diag(v), which only flips output channels and
 * cancels exactly in the integer product; the input-side form used by the works it follows
 * is the one implemented.)
 */
int qvggt_rotated_col_absmax(const void *X_cal, int x_dtype, int M, int K, const int8_t *signs,
                             float *absmax_rot, void *stream);

/*
 * Offline half (Sec. 3.2: rotate, smooth, quantize per output channel):
 *     Wr = W H;  w_j = max_o |Wr[o, j]|;  c_j = max(a_j, 1e-5)^alpha / max(w_j, 1e-5)^(1 - alpha);
 *     Ws = Wr diag(c);  w_scale[o] = max_j |Ws[o, j]| / 7;  Wq[o, :] = clamp(rne(Ws[o, :] / w_scale[o]), -8, 7)
 * W: [N, K] (bf16 or f32).  act_absmax_rot: f32 [K] from qvggt_rotated_col_absmax (a_j), or NULL
 * for c = 1 (rotation only).  signs: as above, must be the vector later given to
 * qvggt_rotate_smooth_quant.  alpha in [0, 1] (the paper uses 0.5).
 * Outputs: Wq packed [N, K/2] bytes; w_scale f32 [N]; inv_smooth f32 [K] with
 *     inv_smooth[j] = 1 / (sqrt(K) c_j)
 * i.e. the Hadamard normalisation and the smoothing divide folded into one multiplier for
 * the online kernel.  The floor 1e-5 on the statistics guards all-zero channels (the paper is
 * silent there).
 */
int qvggt_prep_weights(const void *W, int w_dtype, int N, int K, const float *act_absmax_rot,
                       const int8_t *signs, float alpha, uint8_t *Wq, float *w_scale,
                       float *inv_smooth, void *stream);

/*
 * Offline half with calibrated parameters handed in (appendix, implementation details: the channel-wise factor and the
 * quantization steps are learnable during calibration; this is what deploys the learned values, the activation side being
 * qvggt_rotate_smooth_quant_static):
 *     Ws = W H diag(c_hat);  Wq[o, :] = clamp(rne(Ws[o, :] / w_step[o]), -2^(bits-1), 2^(bits-1) - 1);  w_scale = w_step
 * c_hat: f32 [K], positive and finite (not checked), or NULL for 1.  w_step: f32 [N], positive, or NULL for each channel's
 * own step max_j |Ws[o, j]| / (2^(bits-1) - 1) as in qvggt_prep_weights.  bits: 4 writes packed Wq [N, K/2] (for
 * qvggt_w4a4_gemm and, through qvggt_codes_to_e2m3, qvggt_e2m3_gemm: that conversion reports codes -8, which it cannot carry,
 * so keep w_step at or above the channel's own step there); 5..8 write int8 Wq [N, K] (for qvggt_i8_gemm).  QVGGT_ERR_ARG for other
 * bits.  Outputs as qvggt_prep_weights; inv_smooth[j] = 1 / (sqrt(K) c_hat[j]).
 */
int qvggt_prep_weights_given(const void *W, int w_dtype, int N, int K, const float *c_hat, const int8_t *signs,
                             const float *w_step, int bits, void *Wq, float *w_scale, float *inv_smooth, void *stream);

/*
 * Online kernel 1 (Sec. 3.2 rotation + smoothing; Sec. 3.1.2 quantizer, per token, dynamic):
 *     z[t, :] = (X[t, :] diag(signs) Hadamard_K) * inv_smooth;   x_scale[t] = max_j |z[t, j]| / 7;
 *     Xq[t, j] = clamp(rne(z[t, j] / x_scale[t]), -8, 7)
 * Hadamard_K is the unnormalised +-1 matrix; its 1/sqrt(K) lives in inv_smooth.
 * X: [M, K] (bf16 or f32).  signs: int8 [K] or NULL.  inv_smooth: f32 [K], or NULL for the
 * plain orthonormal rotation (1/sqrt(K) everywhere).  Outputs: Xq packed [M, K/2] bytes,
 * x_scale f32 [M].  A row of zeros gets scale 0 and codes 0, and so does a row whose step would lie below 2^-126, the
 * smallest normal fp32 number (it could not be inverted in fp32).  Butterflies and scaling are fp32.
 */
int qvggt_rotate_smooth_quant(const void *X, int x_dtype, int M, int K, const int8_t *signs,
                              const float *inv_smooth, uint8_t *Xq, float *x_scale, void *stream);

/*
 * Online kernel 1 with a STATIC quantization step (appendix "More analysis on DSFQ", activation-granularity
 * ablation: static vs dynamic, tensor-wise vs token-wise).  Same rotation and smoothing as
 * qvggt_rotate_smooth_quant, but the step is given by the caller (calibrated offline) instead of being
 * derived from the row:
 *     Xq[t, j] = clamp(rne(z[t, j] / x_step[t * per_token]), -8, 7)
 * so the clamp of the quantizer (Sec. 3.1.2) is live here.  x_step: f32, M values (per_token = 1, token-wise
 * static) or one value for the whole tensor (per_token = 0, tensor-wise); 4-byte aligned; a step below 2^-126
 * (zero and negative values included) gives codes 0.  x_scale f32 [M] receives the step every token was quantized with, i.e. what qvggt_w4a4_gemm
 * takes as x_scale.  Other arguments, layouts and errors as qvggt_rotate_smooth_quant; per_token outside
 * {0, 1} is QVGGT_ERR_ARG.
 */
int qvggt_rotate_smooth_quant_static(const void *X, int x_dtype, int M, int K, const int8_t *signs,
                                     const float *inv_smooth, const float *x_step, int per_token,
                                     uint8_t *Xq, float *x_scale, void *stream);

/*
 * The asymmetric setting (appendix, table of further quantization settings: "QuantVGGT (Asymmetric)", W4A4).  The paper
 * gives no formula; this is the usual affine quantizer on the activations, per token and dynamic like Eq. 3's, while the
 * weights keep their symmetric per-channel grid:
 *     z = X H diag(c)^-1 (as in kernel 1),  lo_t = min(0, min_j z_tj),  hi_t = max(0, max_j z_tj),
 *     x_scale[t] = (hi_t - lo_t) / 15,  x_zero[t] = rne(-lo_t / x_scale[t]) in [0, 15],
 *     u_tj = clamp(rne(z_tj / x_scale[t]) + x_zero[t], 0, 15),          z_tj ~ x_scale[t] * (u_tj - x_zero[t]).
 * Xq holds the signed value u - 8 in each nibble (same layout as qvggt_rotate_smooth_quant), so that the integer product
 * is the symmetric one, and the GEMM adds what is missing from
 *     sum_j (u_tj - zp_t) qw_oj = sum_j (u_tj - 8) qw_oj + (8 - zp_t) * w_codesum[o],     w_codesum[o] = sum_j qw_oj
 * in its epilogue (all terms are integers below 2^24 in magnitude, or multiples of 256 below 2^27: exact in fp32):
 *     Y[t, o] = bf16_rne( (acc[t, o] + (8 - x_zero[t]) * w_codesum[o]) * x_scale[t] * w_scale[o] + bias[o] ).
 * A row of zeros has x_scale = 0, x_zero = 0, u = 0.  x_zero: f32 [M] (integer values).  w_codesum: f32 [N].
 * qvggt_rotate_smooth_quant_asym: K a power of two in [128, 8192]; other arguments and errors as
 * qvggt_rotate_smooth_quant.  qvggt_weight_code_sums: Wq as written by qvggt_prep_weights (any supported K), offline.
 * qvggt_w4a4_gemm_asym: as qvggt_w4a4_gemm without the accumulator dump.
 */
int qvggt_rotate_smooth_quant_asym(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                                   uint8_t *Xq, float *x_scale, float *x_zero, void *stream);
int qvggt_weight_code_sums(const uint8_t *Wq, int N, int K, float *w_codesum, void *stream);
int qvggt_w4a4_gemm_asym(const uint8_t *Xq, const float *x_scale, const float *x_zero, const uint8_t *Wq,
                         const float *w_scale, const float *w_codesum, const void *bias, int M, int N, int K, void *Y,
                         void *stream);

/*
 * Online kernel 1 with the LayerNorm that precedes the layer fused in (VGGT's qkv and fc1 inputs; Sec. 3.2 names the
 * neighbouring normalization layer as the place where per-channel factors can live).  Per token, before the rotation:
 *     y = (x - mean) / sqrt(var + eps) * gamma + beta      (mean, population variance over the K channels, fp32),
 * y rounded to the type of X (bf16 input: round to nearest even, i.e. what a separate bf16 LayerNorm kernel would
 * write; f32 input: no rounding), then exactly qvggt_rotate_smooth_quant on y.  One read of X instead of a
 * normalisation pass (read + write) followed by this kernel's read.
 * gamma, beta: f32 [K] or NULL (1 and 0).  eps >= 0 (QVGGT_ERR_ARG otherwise).  K: a power of two in [128, 4096]
 * (8192 and the sizes 2^n * m are QVGGT_ERR_SHAPE here).  Other arguments, layouts and errors as qvggt_rotate_smooth_quant.
 */
int qvggt_layernorm_rotate_smooth_quant(const void *X, int x_dtype, int M, int K, const float *gamma, const float *beta,
                                        float eps, const int8_t *signs, const float *inv_smooth, uint8_t *Xq,
                                        float *x_scale, void *stream);

/*
 * Online kernel 1 of fc2 with the GELU that precedes it fused in (VGGT's MLP blocks: fc1 -> GELU -> fc2, the linear
 * layers being those of Sec. 3.2).  X is fc1's output as stored; per element, before the rotation:
 *     y = bf16_rne( x * Phi(x) )      (Phi the standard normal distribution function; the exact, erf-based GELU),
 * i.e. what a separate bf16 activation kernel would write, then exactly qvggt_rotate_smooth_quant (Xq: packed codes) or
 * qvggt_rotate_smooth_quant_e2m3 (Xf: E2M3 blocks, below) on y.  One read of fc1's output instead of an activation pass
 * (read + write) followed by this kernel's read.  A bf16 input has 65536 values, so the activation is a table: the kernel
 * looks up the correctly rounded result (2^-20 <= |x| < 2^12 from the table; below that x / 2, above it x or -0, all exact
 * at bf16 precision) instead of evaluating erfc per element.
 * qvggt_gelu_table: fills `table` (device, QVGGT_GELU_TABLE_BYTES bytes, 16-byte aligned, caller-owned; contents are the
 *   library's own format) on the device, in double precision, once; it depends on nothing but the function.  The other
 *   calls take it as gelu_table (required: QVGGT_ERR_NULL without it).
 * bf16 X with K = 1024, 2048 or 4096 only: other K are QVGGT_ERR_SHAPE, f32 X is QVGGT_ERR_DTYPE.  Inputs must be finite.
 * Other arguments, layouts and errors as the entry points named above.
 */
#define QVGGT_GELU_TABLE_BYTES 16384u
size_t qvggt_gelu_table_bytes(void);
int qvggt_gelu_table(void *table, void *stream);
int qvggt_gelu_rotate_smooth_quant(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                                   const void *gelu_table, uint8_t *Xq, float *x_scale, void *stream);
int qvggt_gelu_rotate_smooth_quant_e2m3(const void *X, int x_dtype, int M, int K, const int8_t *signs,
                                        const float *inv_smooth, const void *gelu_table, uint8_t *Xf, float *x_scale,
                                        void *stream);
/* Y = GELU(X) W^T + b on the E2M3 path: qvggt_gelu_rotate_smooth_quant_e2m3 into the workspace, then qvggt_e2m3_gemm, on one
 * stream; arguments, workspace (qvggt_workspace_bytes_e2m3) and errors as qvggt_linear_e2m3 below. */
int qvggt_gelu_linear_e2m3(const void *X, int x_dtype, int M, int N, int K, const int8_t *signs, const float *inv_smooth,
                           const void *gelu_table, const uint8_t *Wf, const float *w_scale, const void *bias, void *Y,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * Online kernel 2 (Sec. 3.2 granularity paragraph: integer sum, dequantise after it):
 *     acc[t, o] = sum_j Xq[t, j] Wq[o, j]   (int32, exact);
 *     Y[t, o]   = bf16_rne( acc[t, o] * x_scale[t] * w_scale[o] + bias[o] )
 * Xq [M, K/2], Wq [N, K/2] packed as written by this library; x_scale f32 [M]; w_scale f32 [N];
 * bias bf16 [N] or NULL; Y bf16 [M, N].  acc_debug: int32 [M, N] receiving the raw accumulators,
 * or NULL (test hook; costs an extra 4 bytes per output when given).
 */
int qvggt_w4a4_gemm(const uint8_t *Xq, const float *x_scale, const uint8_t *Wq, const float *w_scale,
                    const void *bias, int M, int N, int K, void *Y, int32_t *acc_debug, void *stream);

/*
 * Online kernel 2 through the 6-bit floating-point matrix instructions: the same integer sums and the same Y as
 * qvggt_w4a4_gemm, bit for bit, at twice the matrix rate.  A 4-bit code q in [-7, 7] is written as the E2M3 number
 * of value q (1 sign, 2 exponent, 3 mantissa bits); products and sums are integers below 2^24 and exact in the
 * fp32 accumulators.  -8 has no E2M3 value: the dynamic quantizers never produce it (Eq. 3 with absmax / 7 gives
 * codes in [-7, 7]); codes from a static step or the asymmetric setting are stored half a step up (see the
 * _shifted entry points below).
 *
 * "E2M3 blocks": a row is K / 64 units of 48 bytes.  Unit s holds the codes at positions 64 s .. 64 s + 63 of a
 * packed row (library order) as two blobs of 32 six-bit fields, field i of blob h = position 64 s + 32 h + i at
 * bits [6 i, 6 i + 6) of the blob's 24 bytes, stored [blob 0 bytes 0..15][blob 1 bytes 0..15][blob 0 bytes 16..23]
 * [blob 1 bytes 16..23].  Rows are grouped in blocks of 128: unit s of row r starts at byte
 * ((r / 128) * (K / 64) + s) * 6144 + (r % 128) * 48, so a buffer holds ceil(rows / 128) * 128 rows:
 * qvggt_e2m3_bytes(rows, K) bytes (0 for an unsupported K).  The rows past `rows` in the last block are never
 * written and may hold anything (the GEMM reads them and discards what they produce).
 * qvggt_codes_to_e2m3:  packed u8 [rows, K/2] (Xq or Wq as written by this library) -> out, E2M3 blocks; distinct buffers.
 *                       A code -8 cannot be carried over: it is written as -7 and COUNTED in *n_unrepresentable (device uint32,
 *                       4-byte aligned, required: QVGGT_ERR_NULL without it; the call adds to it, so zero it first and read it
 *                       after the stream has run).  A count other than 0 means `out` is not a faithful copy and must not be
 *                       used: such codes (static steps below a row's own, qvggt_prep_weights_given) belong on
 *                       qvggt_w4a4_gemm, or, for activations, in the half-step form of the _shifted entry points.
 * qvggt_e2m3_gemm:      Xf, Wf E2M3 blocks of M and N rows; everything else as qvggt_w4a4_gemm (acc_debug receives
 *                       the exact sums as int32).
 * qvggt_rotate_smooth_quant_e2m3:  online kernel 1 writing E2M3 blocks directly (the same codes and steps as
 *                       qvggt_rotate_smooth_quant; a code 0 may carry a sign bit).  bf16 X with K = 1024, 2048 or 4096 only:
 *                       other K are QVGGT_ERR_SHAPE, f32 X is QVGGT_ERR_DTYPE (use qvggt_rotate_smooth_quant and
 *                       qvggt_codes_to_e2m3 there).
 * qvggt_layernorm_rotate_smooth_quant_e2m3:  qvggt_layernorm_rotate_smooth_quant writing E2M3 blocks; bf16 X and
 *                       K = 1024 only (other K QVGGT_ERR_SHAPE, f32 X QVGGT_ERR_DTYPE).
 * Codes that fill the whole 4-bit range (a static step reaches -8; affine codes u run over 0..15) go to the same
 * instructions shifted by half a step: all sixteen half-integers -7.5 .. 7.5 are E2M3 numbers.
 * qvggt_rotate_smooth_quant_asym_e2m3 / _static_e2m3:  qvggt_rotate_smooth_quant_asym / _static writing E2M3 blocks that
 *                       hold u - 7.5 resp. code + 0.5, the steps in x_scale, and in x_zero (f32 [M]) the zero point resp. 8
 *                       (a signed code is u - 8).  bf16 X, K = 1024, 2048 or 4096 only, as above.
 * qvggt_e2m3_gemm_shifted:  Y[t, o] = bf16_rne( (acc'[t, o] + (7.5 - x_zero[t]) * w_codesum[o]) * x_scale[t] * w_scale[o]
 *                       + bias[o] ) with acc' the sum over the stored half-integers times the weight codes (multiples of 0.5
 *                       below 2^23 and an integer after the correction: exact); w_codesum as in qvggt_w4a4_gemm_asym.
 *                       The same Y, bit for bit, as qvggt_w4a4_gemm_asym resp. qvggt_w4a4_gemm on the same codes.
 * qvggt_linear_e2m3:    both kernels on one stream, as qvggt_linear; Wf = qvggt_codes_to_e2m3 of qvggt_prep_weights'
 *                       Wq; workspace of qvggt_workspace_bytes_e2m3(M, N, K) bytes; same restriction on X and K.
 */
size_t qvggt_e2m3_bytes(int rows, int K);
int qvggt_rotate_smooth_quant_asym_e2m3(const void *X, int x_dtype, int M, int K, const int8_t *signs,
                                        const float *inv_smooth, uint8_t *Xf, float *x_scale, float *x_zero, void *stream);
int qvggt_rotate_smooth_quant_static_e2m3(const void *X, int x_dtype, int M, int K, const int8_t *signs,
                                          const float *inv_smooth, const float *x_step, int per_token, uint8_t *Xf,
                                          float *x_scale, float *x_zero, void *stream);
int qvggt_e2m3_gemm_shifted(const uint8_t *Xf, const float *x_scale, const float *x_zero, const uint8_t *Wf,
                            const float *w_scale, const float *w_codesum, const void *bias, int M, int N, int K, void *Y,
                            void *stream);
int qvggt_layernorm_rotate_smooth_quant_e2m3(const void *X, int x_dtype, int M, int K, const float *gamma,
                                             const float *beta, float eps, const int8_t *signs,
                                             const float *inv_smooth, uint8_t *Xf, float *x_scale, void *stream);
int qvggt_rotate_smooth_quant_e2m3(const void *X, int x_dtype, int M, int K, const int8_t *signs,
                                   const float *inv_smooth, uint8_t *Xf, float *x_scale, void *stream);
size_t qvggt_workspace_bytes_e2m3(int M, int N, int K);
int qvggt_linear_e2m3(const void *X, int x_dtype, int M, int N, int K, const int8_t *signs, const float *inv_smooth,
                      const uint8_t *Wf, const float *w_scale, const void *bias, void *Y, void *workspace,
                      size_t workspace_bytes, void *stream);
int qvggt_codes_to_e2m3(const uint8_t *packed, int rows, int K, uint8_t *out, uint32_t *n_unrepresentable, void *stream);

/*
 * qvggt_linear_e2m3 for callers that cannot provide or allocate a workspace (code under HIP graph capture that may not call
 * hipMalloc, tight serving loops, harnesses that forbid allocation): the activation codes and per-token steps that pass from
 * kernel 1 to the GEMM live in a fixed device array inside the library (QVGGT_OWN_WORKSPACE_BYTES, one copy per device, held
 * until the process ends) instead of a workspace argument.  Same kernels, same Y, bit for bit, as qvggt_linear_e2m3; inputs and
 * outputs are still the caller's.  Calls no allocating routine.  The first use on a device resolves the array's address there
 * (the set-up of qvggt_init: call that first when capturing).  Shapes with qvggt_workspace_bytes_e2m3(M, N, K) >
 * QVGGT_OWN_WORKSPACE_BYTES (more than 12160 tokens at K = 4096, 48896 at K = 1024) are refused with QVGGT_ERR_WORKSPACE before anything
 * is launched.  All calls on one device share that device's array, which keeps the last call's contents (nothing in it has to
 * start from zero): calls that overlap in time on one device, on any streams, race on it and give wrong results; calls queued on
 * one stream are safe.  qvggt_own_workspace_bytes returns the limit.
 */
#define QVGGT_OWN_WORKSPACE_BYTES (36u << 20)
size_t qvggt_own_workspace_bytes(void);
int qvggt_linear_e2m3_own_workspace(const void *X, int x_dtype, int M, int N, int K, const int8_t *signs,
                                    const float *inv_smooth, const uint8_t *Wf, const float *w_scale, const void *bias,
                                    void *Y, void *stream);
int qvggt_e2m3_gemm(const uint8_t *Xf, const float *x_scale, const uint8_t *Wf, const float *w_scale,
                    const void *bias, int M, int N, int K, void *Y, int32_t *acc_debug, void *stream);

/*
 * The 8-bit and 6-bit settings of the same layer (Sec. 4.1 bit settings and the pose / point-map tables at 8/8;
 * appendix "More experiments", the 6/6 rows).  Everything is as in the 4-bit entry points above except the
 * quantizer's range and the storage of the codes:
 *     qmax = 2^(bits-1) - 1;   scale = absmax / qmax;   code = clamp(rne(v / scale), -qmax - 1, qmax)
 * with bits in 4..8 (else QVGGT_ERR_ARG), and codes stored one per byte as int8: Xq int8 [M, K], Wq int8 [N, K].
 * The GEMM only sees int8 codes, so weights and activations may take different widths: the mixed-precision setting
 * of the appendix table of further settings, e.g. qvggt_prep_weights_i8 with bits = 4 and qvggt_linear_i8 with
 * bits = 8 (4-bit weights, 8-bit activations; which widths the paper mixes it does not say).
 * The position of a code inside its row is again the library's fixed permutation (the same for Xq and Wq);
 * qvggt_layout_int8 converts to and from natural order.  Sums stay in int32: |acc| <= 128 * 128 * 8192 = 2^27.
 *
 * qvggt_prep_weights_i8:         offline half, as qvggt_prep_weights.
 * qvggt_rotate_smooth_quant_i8:  online kernel 1, per token, dynamic, as qvggt_rotate_smooth_quant.
 * qvggt_i8_gemm:                 online kernel 2, as qvggt_w4a4_gemm (acc_debug receives the exact sums).
 * qvggt_linear_i8:               both on one stream; workspace of qvggt_workspace_bytes_i8(M, N, K) bytes.
 * qvggt_layout_int8:             src int8 [rows, K] -> dst int8 [rows, K] (distinct buffers); to_library = 1: natural
 *                                order -> library order, 0: the inverse; other values are QVGGT_ERR_ARG.
 */
int qvggt_prep_weights_i8(const void *W, int w_dtype, int N, int K, const float *act_absmax_rot,
                          const int8_t *signs, float alpha, int bits, int8_t *Wq, float *w_scale,
                          float *inv_smooth, void *stream);
int qvggt_rotate_smooth_quant_i8(const void *X, int x_dtype, int M, int K, const int8_t *signs,
                                 const float *inv_smooth, int bits, int8_t *Xq, float *x_scale, void *stream);
int qvggt_i8_gemm(const int8_t *Xq, const float *x_scale, const int8_t *Wq, const float *w_scale,
                  const void *bias, int M, int N, int K, void *Y, int32_t *acc_debug, void *stream);
int qvggt_linear_i8(const void *X, int x_dtype, int M, int N, int K, const int8_t *signs,
                    const float *inv_smooth, int bits, const int8_t *Wq, const float *w_scale, const void *bias,
                    void *Y, void *workspace, size_t workspace_bytes, void *stream);
size_t qvggt_workspace_bytes_i8(int M, int N, int K);
int qvggt_layout_int8(const int8_t *src, int rows, int K, int8_t *dst, int to_library, void *stream);

/*
 * The int8-code path (8-/6-bit and mixed settings above) with its operands in "int8 blocks", the layout in which every
 * global -> LDS transfer of the GEMM is contiguous in memory: rows grouped in blocks of 128 with the K-tiles of 64 codes
 * outermost, K-tile kt of row r at byte ((r / 128) * (K / 64) + kt) * 8192 + (r % 128) * 64, and inside it the 16-byte
 * chunk ch of the row's codes (library order) in slot ch ^ ((r % 16) >> 2).  A buffer holds ceil(rows / 128) * 128 rows:
 * qvggt_i8b_bytes(rows, K) bytes (0 for an unsupported K); the rows past `rows` are never written and may hold anything.  Same codes, same sums,
 * same Y as the qvggt_*_i8 entry points, bit for bit.
 * qvggt_int8_to_blocks:           int8 [rows, K] in library order (Xq or Wq of the _i8 entry points) -> int8 blocks.
 * qvggt_rotate_smooth_quant_i8b:  qvggt_rotate_smooth_quant_i8 writing int8 blocks; bf16 X, K = 1024, 2048 or 4096 only
 *                                 (other K QVGGT_ERR_SHAPE, f32 X QVGGT_ERR_DTYPE).
 * qvggt_i8b_gemm:                 qvggt_i8_gemm on int8 blocks.
 * qvggt_linear_i8b:               both on one stream; Wb = qvggt_int8_to_blocks of qvggt_prep_weights_i8's Wq; workspace
 *                                 of qvggt_workspace_bytes_i8b(M, N, K) bytes.
 */
size_t qvggt_i8b_bytes(int rows, int K);
int qvggt_int8_to_blocks(const int8_t *src, int rows, int K, int8_t *dst, void *stream);
int qvggt_rotate_smooth_quant_i8b(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                                  int bits, int8_t *Xb, float *x_scale, void *stream);
int qvggt_i8b_gemm(const int8_t *Xb, const float *x_scale, const int8_t *Wb, const float *w_scale, const void *bias, int M,
                   int N, int K, void *Y, int32_t *acc_debug, void *stream);
size_t qvggt_workspace_bytes_i8b(int M, int N, int K);
int qvggt_linear_i8b(const void *X, int x_dtype, int M, int N, int K, const int8_t *signs, const float *inv_smooth, int bits,
                     const int8_t *Wb, const float *w_scale, const void *bias, void *Y, void *workspace,
                     size_t workspace_bytes, void *stream);

/*
 * Whole online path: qvggt_rotate_smooth_quant into the workspace, then qvggt_w4a4_gemm.
 * workspace: device buffer of at least qvggt_workspace_bytes(M, N, K) bytes, 16-byte aligned
 * (holds Xq and x_scale between the two kernels; contents undefined afterwards).
 */
int qvggt_linear(const void *X, int x_dtype, int M, int N, int K, const int8_t *signs,
                 const float *inv_smooth, const uint8_t *Wq, const float *w_scale, const void *bias,
                 void *Y, void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of workspace qvggt_linear needs; 0 if the shape is invalid. */
size_t qvggt_workspace_bytes(int M, int N, int K);

/*
 * Layout converters for packed 4-bit buffers (see "General conventions").
 * qvggt_pack_int4:   codes int8 [rows, K] in natural order, each in [-8, 7] (low 4 bits are
 *                    taken) -> packed [rows, K/2] in the library's layout.
 * qvggt_unpack_int4: the inverse, sign-extending each code to int8.
 */
int qvggt_pack_int4(const int8_t *codes, int rows, int K, uint8_t *packed, void *stream);
int qvggt_unpack_int4(const uint8_t *packed, int rows, int K, int8_t *codes, void *stream);

/*
 * Arithmetic of the calibration-set construction (Sec. 3.3, Noise-Filtered Diverse Sampling).  Offline, outside the
 * inference path; the two calls that read whole activation tensors are HBM-bound reductions, the others handle a pool
 * of a few hundred samples.  Double arithmetic inside, float results.  Choosing the final samples inside each cluster
 * (the uniform draw of Eq. "cluster") is left to the caller.
 *
 * qvggt_nfds_moments (first equation of the noise filter): mean[r] and var[r] (population variance) over the `count`
 *   elements of row r of A [rows, count] (bf16 or f32), one row per (sample, layer) activation.  A row must be a whole
 *   number of 16-byte vectors (count a multiple of 8 for bf16, of 4 for f32).  workspace: device buffer of at least
 *   qvggt_nfds_workspace_bytes(rows, count, dtype) bytes (partial sums; contents undefined afterwards).
 * qvggt_nfds_frame_correlation (frame-aware correlation vector): A [samples, frames, frame_elems] holds the feature of
 *   each sample frame after frame (frame_elems = tokens per frame x channels); corr [samples, frames - 1] receives the
 *   cosine between frame 0 and frame t, t = 1 .. frames - 1.  workspace as above with rows = samples * frames,
 *   count = frame_elems.  A frame of zeros gives NaN, as the definition does.
 * qvggt_nfds_scores (noise score): m, s f32 [D, L] per-sample per-layer moments -> score f32 [D]; the z-scores use the
 *   pool's mean and standard deviation per layer with eps (>= 0) under the root.  D <= 65536, L <= 2048.
 * qvggt_nfds_keep_lowest (Eq. "filter"): keep[i] = 1 for the floor(p * D) samples of lowest score (the percentile
 *   threshold T), else 0; equal scores are ordered by index.  p in [0, 1].
 * qvggt_nfds_kmeans_step (Eq. "cluster"): one Lloyd iteration on c f32 [n, dim] with K centres: labels[i] = index of the
 *   nearest centre of centres_in [K, dim] (squared Euclidean distance, the lower index on a tie), centres_out[k] = mean
 *   of the points labelled k (a centre without points is copied).  The caller iterates and supplies the initial centres.
 *   n <= 65536, dim <= 4096, K <= 256; centres_in and centres_out must differ.
 * Errors: QVGGT_ERR_SHAPE for sizes outside these limits, QVGGT_ERR_ARG for eps / p out of range or aliased centres,
 * otherwise as for the other calls (f32 arrays here only need 4-byte alignment; A and workspace 16 bytes).
 */
size_t qvggt_nfds_workspace_bytes(int rows, long long count, int dtype);
int qvggt_nfds_moments(const void *A, int dtype, int rows, long long count, float *mean, float *var, void *workspace,
                       size_t workspace_bytes, void *stream);
int qvggt_nfds_frame_correlation(const void *A, int dtype, int samples, int frames, long long frame_elems, float *corr,
                                 void *workspace, size_t workspace_bytes, void *stream);
int qvggt_nfds_scores(const float *m, const float *s, int D, int L, double eps, float *score, void *stream);
int qvggt_nfds_keep_lowest(const float *score, int D, double p, uint8_t *keep, void *stream);
int qvggt_nfds_kmeans_step(const float *c, int n, int dim, int K, const float *centres_in, float *centres_out,
                           int32_t *labels, void *stream);

/*
 * Refinement of the smoothing factor and the quantization steps of one layer on a calibration batch (appendix "Experiment
 * Settings": during calibration c_hat and the steps Delta are learnable, learning rates 5e-3 and 5e-2; Sec. 3.1.2, Eq.
 * "loss_ori_overall": the objective is the squared distance between the full-precision and the quantized function over the
 * calibration set).  Offline.  The paper gives no update rule; this library's reading:
 *     z = (X H) / c,  x_hat = step_x * clamp(rne(z / step_x)),     v = (W H) * c,  w_hat[o] = step_w[o] * clamp(rne(v[o] / step_w[o])),
 *     y_q = x_hat . w_hat^T + b,     L = (1 / T) sum_t || y_q[t] - y_ref[t] ||^2     (clamp to [-2^(bits-1), 2^(bits-1) - 1]);
 *   derivatives by the straight-through rules: rounding passes 1; a value whose ROUNDED code leaves the range passes nothing;
 *   d(quantized value) / d(its step) = rne(u) - u inside the range, the clamp bound outside; c_hat moves through both operands
 *   (d v / d c = V, d z / d c = -z / c); with x_step == NULL the activation steps are the dynamic per-token ones, max_j |z| / qmax,
 *   recomputed from each row and held constant in the derivative; with x_step given it is one static step for the tensor and learnable.
 * qvggt_rotate_rows:  R [M, K] f32 = X . H, H = diag(signs) . Hhat_K (orthonormal), natural channel order: what the loss takes as
 *   R = X_cal H and V = W H (computed once per layer; they do not change while c_hat and the steps move).  K a power of two in
 *   [128, 8192].
 * qvggt_calib_loss_grad:  R [T, K], V [N, K], y_ref [T, N] f32 (the full-precision layer's output on the batch, bias included),
 *   bias bf16 [N] or NULL, c_hat f32 [K] and w_step f32 [N] positive, x_step f32 [1] or NULL, bits in 4..8.  Outputs f32: loss [1],
 *   grad_c [K], grad_w_step [N], grad_x_step [1] (given exactly when x_step is: QVGGT_ERR_NULL otherwise).  T, N >= 1, K a
 *   multiple of 4 up to 8192 (QVGGT_ERR_SHAPE).  workspace: qvggt_calib_workspace_bytes(T, N, K) bytes (0 for an invalid shape),
 *   16-byte aligned.  fp32 arithmetic, sums in a fixed order (the same call gives the same bits).
 * qvggt_calib_descent_step:  theta[i] <- max(theta[i] - lr * grad[i], floor), floor > 0 keeping factors and steps positive
 *   (plain gradient descent with the paper's learning rates; which optimiser the paper's pipeline runs it does not say).
 * The refined values are deployed by qvggt_prep_weights_given (c_hat, w_step) and qvggt_rotate_smooth_quant_static (x_step).
 */
int qvggt_rotate_rows(const void *X, int x_dtype, int M, int K, const int8_t *signs, float *R, void *stream);
size_t qvggt_calib_workspace_bytes(int T, int N, int K);
int qvggt_calib_loss_grad(const float *R, const float *V, const float *y_ref, const void *bias, const float *c_hat,
                          const float *w_step, const float *x_step, int T, int N, int K, int bits, float *loss, float *grad_c,
                          float *grad_w_step, float *grad_x_step, void *workspace, size_t workspace_bytes, void *stream);
int qvggt_calib_descent_step(float *theta, const float *grad, int n, float lr, float floor, void *stream);

/*
 * Measurement helper (used by the benchmark, not by the path): a register-only loop of the matrix instruction a GEMM is
 * built on, to state what the matrix pipes of this board sustain when nothing has to be fed to them.  One launch runs
 * 256 blocks x 4 waves x iters x 16 instructions; kind 0: v_mfma_i32_32x32x32_i8 (2 * 32 * 32 * 32 operations each), kind 1:
 * v_mfma_f32_32x32x64_f8f6f4 on E2M3 operands (2 * 32 * 32 * 64 each).  sink: device f32 [65536], overwritten.  QVGGT_ERR_ARG
 * for another kind or iters outside 1 .. 2^24.
 */
int qvggt_mfma_ceiling(int kind, int iters, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QVGGT_H */
