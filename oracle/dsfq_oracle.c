/*
 * CPU oracle of the Dual-Smoothed Fine-Grained Quantization (DSFQ) linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * quantized linear layer computes, written from the paper's definitions; the
 * HIP library is checked against it.  It shares no code with the HIP path and
 * nothing outside tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.
 *
 * All floating point is IEEE double.  Inputs arrive as doubles converted
 * exactly from bf16 / fp32 by the caller.  The Hadamard matrix is materialised
 * densely (O(K^2) per row) because that is the definition; the only
 * parallelism is an optional OpenMP loop over independent rows.
 *
 * Passages followed (paper section / equation):
 *   - symmetric N-bit quantizer ................ Sec. 3.1.2, Eq. "quantization"
 *   - normalised Sylvester Hadamard, random signs . Sec. 3.2 Pre-Global-Rotation
 *   - rotation invariance X W^T = (XH)(WH)^T ..... Sec. 3.2, equation after the Hadamard recursion
 *   - smoothing factor c_hat and its identity ... Sec. 3.2 Post-Local-Smooth, Eq. "smooth_factor"
 *   - per-token activations / per-output-channel weights, integer sum,
 *     dequantisation after the sum ............. Sec. 3.2 Fine-Grained Quantization Granularity
 *
 * Pins (tests/test_oracle_*.py): H H^T = K I in integers, recursion == popcount
 * closed form, rotation and smoothing invariances against a plain matmul,
 * quantizer error bound / symmetry / scale equivariance / hand-worked rows,
 * brute-force integer dot products, bf16 rounding on hand-picked bit patterns.
 * The end-to-end output values have no printed example in the paper: for them
 * parity is pinned only through those per-step properties and the overall
 * error budget ("parity unpinned" for absolute end-to-end values).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_ERR_ARG 1
#define ORC_ERR_OVERFLOW 2
#define ORC_ERR_ALLOC 3

static int is_pow2(int k) { return k >= 1 && (k & (k - 1)) == 0; }

/* ---------------------------------------------------------------- Hadamard
 * Unnormalised Sylvester matrix by the Kronecker recursion
 *   H_1 = [1],  H_2n = [[H_n, H_n], [H_n, -H_n]]  (= H_2 (x) H_n),
 * entries +-1 as int8, row-major K x K.  The paper's orthonormal matrix is this
 * divided by sqrt(K) (each level contributes 1/sqrt 2).
 */
int orc_hadamard_recursive(int K, int8_t *H)
{
    if (!is_pow2(K) || !H) return ORC_ERR_ARG;
    H[0] = 1;
    for (int n = 1; n < K; n *= 2) {
        /* the n x n block is in H[0..n) x [0..n) with row stride K */
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                int8_t h = H[(size_t)i * K + j];
                H[(size_t)i * K + (j + n)] = h;
                H[(size_t)(i + n) * K + j] = h;
                H[(size_t)(i + n) * K + (j + n)] = (int8_t)-h;
            }
    }
    return ORC_OK;
}

/* Closed form of the same matrix: H[i][j] = (-1)^popcount(i & j). */
int orc_hadamard_popcount(int K, int8_t *H)
{
    if (!is_pow2(K) || !H) return ORC_ERR_ARG;
    for (int i = 0; i < K; ++i)
        for (int j = 0; j < K; ++j) {
            unsigned v = (unsigned)i & (unsigned)j, p = 0;
            while (v) { p ^= v & 1u; v >>= 1; }
            H[(size_t)i * K + j] = p ? -1 : 1;
        }
    return ORC_OK;
}

/* ---------------------------------------------------------------- sizes that are not powers of two
 * Sec. 3.2: for d = 2^n m the matrix is H_{2^n} (x) H_m.  The paper does not say which H_m; taken here (the usual
 * choice for m = 12, 20, 28) are Paley's constructions from the quadratic character chi of GF(q):
 *   type I  (q = 3 mod 4, m = q + 1: 12 from q = 11, 20 from q = 19):  H = I + S,
 *           S = [[0, 1 .. 1], [-1 .., Q]],  Q[i][j] = chi(i - j)   (S is skew, S S^T = q I);
 *   type II (q = 1 mod 4, m = 2 (q + 1): 28 from q = 13):  C = [[0, 1 .. 1], [1 .., Q]] (symmetric, C C^T = q I);
 *           every 0 of C becomes [[1, -1], [-1, -1]], every +-1 becomes +-[[1, 1], [1, -1]].
 * chi(x) = 0 for x = 0, 1 if x is a non-zero square mod q, -1 otherwise, by Euler's criterion x^((q-1)/2) mod q.
 */
static int chi_mod(int x, int q)
{
    x %= q;
    if (x < 0) x += q;
    if (x == 0) return 0;
    long long r = 1, b = x;
    for (int e = (q - 1) / 2; e > 0; e >>= 1) {
        if (e & 1) r = r * b % q;
        b = b * b % q;
    }
    return r == 1 ? 1 : -1;
}

int orc_hadamard_paley(int m, int8_t *H)
{
    if (!H) return ORC_ERR_ARG;
    if (m == 12 || m == 20) {
        const int q = m - 1;
        for (int i = 0; i < m; ++i)
            for (int j = 0; j < m; ++j) {
                int s;
                if (i == 0) s = (j == 0) ? 0 : 1;
                else if (j == 0) s = -1;
                else s = chi_mod((i - 1) - (j - 1), q);
                H[i * m + j] = (int8_t)(s + (i == j ? 1 : 0));
            }
        return ORC_OK;
    }
    if (m == 28) {
        const int q = 13, n = 14;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                int c;
                if (i == 0 && j == 0) c = 0;
                else if (i == 0 || j == 0) c = 1;
                else c = chi_mod((i - 1) - (j - 1), q);
                /* 2 x 2 block of entry (i, j) */
                int b00, b01, b10, b11;
                if (c == 0) { b00 = 1; b01 = -1; b10 = -1; b11 = -1; }
                else { b00 = c; b01 = c; b10 = c; b11 = -c; }
                H[(2 * i) * m + 2 * j] = (int8_t)b00;
                H[(2 * i) * m + 2 * j + 1] = (int8_t)b01;
                H[(2 * i + 1) * m + 2 * j] = (int8_t)b10;
                H[(2 * i + 1) * m + 2 * j + 1] = (int8_t)b11;
            }
        return ORC_OK;
    }
    return ORC_ERR_ARG;
}

/* K = 2^n m with m in {1, 12, 20, 28}: returns m (0 if K has no such form); K is a power of two when m == 1 */
static int paley_factor(int K)
{
    if (K < 1) return 0;
    if (is_pow2(K)) return 1;
    int odd = K;
    while ((odd & 1) == 0) odd >>= 1;
    if (odd != 3 && odd != 5 && odd != 7) return 0;
    const int m = 4 * odd;
    return (K % m == 0 && is_pow2(K / m)) ? m : 0;
}

/* Unnormalised K x K matrix H_{2^n} (x) H_m, index e = a m + b (a the 2^n part): H[e][e'] = H2n[a][a'] Hm[b][b']. */
int orc_hadamard_general(int K, int8_t *H)
{
    const int m = paley_factor(K);
    if (m == 0 || !H) return ORC_ERR_ARG;
    if (m == 1) return orc_hadamard_recursive(K, H);
    const int n2 = K / m;
    int8_t *A = (int8_t *)malloc((size_t)n2 * n2), *B = (int8_t *)malloc((size_t)m * m);
    if (!A || !B) { free(A); free(B); return ORC_ERR_ALLOC; }
    orc_hadamard_recursive(n2, A);
    orc_hadamard_paley(m, B);
    for (int a = 0; a < n2; ++a)
        for (int b = 0; b < m; ++b)
            for (int a2 = 0; a2 < n2; ++a2)
                for (int b2 = 0; b2 < m; ++b2)
                    H[(size_t)(a * m + b) * K + (a2 * m + b2)] = (int8_t)(A[a * n2 + a2] * B[b * m + b2]);
    free(A);
    free(B);
    return ORC_OK;
}

/* ---------------------------------------------------------------- rotation
 * Xr = X . H with the randomised orthonormal Hadamard.  Two sign conventions
 * are supported because the paper's text and the works it follows differ:
 *   pre[i]  (may be NULL): H = diag(pre) . Hhat   -- signs flip input channels
 *   post[j] (may be NULL): H = Hhat . diag(post)  -- the paper's literal formula
 * Xr[t][j] = post[j] / sqrt(K) * sum_i X[t][i] * pre[i] * H_K[i][j].
 */
int orc_rotate(const double *X, int rows, int K, const int8_t *pre, const int8_t *post, double *Xr)
{
    if (!X || !Xr || rows < 0 || paley_factor(K) == 0) return ORC_ERR_ARG;
    int8_t *H = (int8_t *)malloc((size_t)K * K);
    if (!H) return ORC_ERR_ALLOC;
    orc_hadamard_general(K, H);
    const double norm = sqrt((double)K);
#pragma omp parallel for schedule(static)
    for (int t = 0; t < rows; ++t) {
        const double *x = X + (size_t)t * K;
        double *y = Xr + (size_t)t * K;
        for (int j = 0; j < K; ++j) y[j] = 0.0;
        for (int i = 0; i < K; ++i) {            /* y[j] = sum_i x_i H[i][j], i ascending */
            const double xi = pre ? x[i] * (double)pre[i] : x[i];
            const int8_t *h = H + (size_t)i * K;
            for (int j = 0; j < K; ++j) y[j] += xi * (double)h[j];
        }
        for (int j = 0; j < K; ++j) {
            double s = y[j] / norm;
            y[j] = post ? s * (double)post[j] : s;
        }
    }
    free(H);
    return ORC_OK;
}

/* ---------------------------------------------------------------- smoothing
 * out[j] = max over rows of |A[r][j]| : the per-channel statistic of the
 * smoothing factor, taken in rotated space.
 */
int orc_col_absmax(const double *A, int rows, int K, double *out)
{
    if (!A || !out || rows < 0 || K < 1) return ORC_ERR_ARG;
    for (int j = 0; j < K; ++j) out[j] = 0.0;
    for (int r = 0; r < rows; ++r)
        for (int j = 0; j < K; ++j) {
            double v = fabs(A[(size_t)r * K + j]);
            if (v > out[j]) out[j] = v;
        }
    return ORC_OK;
}

/* c_hat[j] = a[j]^alpha / w[j]^(1-alpha); a, w are clamped from below by
 * `floor_` first (the paper is silent on zero statistics). */
int orc_smooth_factor(const double *a, const double *w, int K, double alpha, double floor_, double *c)
{
    if (!a || !w || !c || K < 1 || !(alpha >= 0.0 && alpha <= 1.0)) return ORC_ERR_ARG;
    for (int j = 0; j < K; ++j) {
        double aj = a[j] > floor_ ? a[j] : floor_;
        double wj = w[j] > floor_ ? w[j] : floor_;
        c[j] = pow(aj, alpha) / pow(wj, 1.0 - alpha);
    }
    return ORC_OK;
}

/* A[r][j] *= c[j] (inverse == 0) or A[r][j] /= c[j] (inverse != 0), in place. */
int orc_scale_columns(double *A, int rows, int K, const double *c, int inverse)
{
    if (!A || !c || rows < 0 || K < 1) return ORC_ERR_ARG;
    for (int r = 0; r < rows; ++r)
        for (int j = 0; j < K; ++j) {
            if (inverse) A[(size_t)r * K + j] /= c[j];
            else A[(size_t)r * K + j] *= c[j];
        }
    return ORC_OK;
}

/* ---------------------------------------------------------------- quantizer
 * Symmetric `bits`-bit quantizer applied to each row separately (a row is a
 * token for activations, an output channel for weights):
 *   delta[r] = max_j |A[r][j]| / (2^(bits-1) - 1)
 *   q[r][j]  = clamp(round(A[r][j] / delta[r]), -2^(bits-1), 2^(bits-1) - 1)
 * round = round-half-to-even (nearbyint in the default rounding mode).  A row
 * of zeros gets delta 0 and codes 0, and so does a row whose step would lie
 * below ORC_MIN_STEP = 2^-126, the smallest normal single-precision number:
 * the steps are handed on as single-precision numbers, and a step that is not
 * a normal one there cannot be divided by (the paper is silent on both cases).
 */
#define ORC_MIN_STEP 0x1p-126
int orc_quantize_rows(const double *A, int rows, int K, int bits, double *delta, int8_t *q)
{
    if (!A || !delta || !q || rows < 0 || K < 1 || bits < 2 || bits > 8) return ORC_ERR_ARG;
    const double qmax = (double)((1 << (bits - 1)) - 1), qmin = -(double)(1 << (bits - 1));
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const double *a = A + (size_t)r * K;
        double m = 0.0;
        for (int j = 0; j < K; ++j) { double v = fabs(a[j]); if (v > m) m = v; }
        double d = m / qmax;
        if (d < ORC_MIN_STEP) d = 0.0;
        delta[r] = d;
        for (int j = 0; j < K; ++j) {
            double v = (d > 0.0) ? nearbyint(a[j] / d) : 0.0;
            if (v < qmin) v = qmin;
            if (v > qmax) v = qmax;
            q[(size_t)r * K + j] = (int8_t)v;
        }
    }
    return ORC_OK;
}

/* Same quantizer with a given (static) step: used for the clamp's live case.  A step below ORC_MIN_STEP (zero and negative
 * values included) gives codes 0. */
int orc_quantize_rows_static(const double *A, int rows, int K, int bits, const double *delta, int8_t *q)
{
    if (!A || !delta || !q || rows < 0 || K < 1 || bits < 2 || bits > 8) return ORC_ERR_ARG;
    const double qmax = (double)((1 << (bits - 1)) - 1), qmin = -(double)(1 << (bits - 1));
    for (int r = 0; r < rows; ++r)
        for (int j = 0; j < K; ++j) {
            double d = delta[r];
            double v = (d >= ORC_MIN_STEP) ? nearbyint(A[(size_t)r * K + j] / d) : 0.0;
            if (v < qmin) v = qmin;
            if (v > qmax) v = qmax;
            q[(size_t)r * K + j] = (int8_t)v;
        }
    return ORC_OK;
}

/* ---------------------------------------------------------------- integer GEMM
 * acc[t][o] = sum_j qx[t][j] * qw[o][j], summed in int64 and required to fit int32.
 */
int orc_int_gemm(const int8_t *qx, const int8_t *qw, int M, int N, int K, int32_t *acc)
{
    if (!qx || !qw || !acc || M < 0 || N < 0 || K < 1) return ORC_ERR_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < M; ++t)
        for (int o = 0; o < N; ++o) {
            int64_t s = 0;
            for (int j = 0; j < K; ++j)
                s += (int64_t)qx[(size_t)t * K + j] * (int64_t)qw[(size_t)o * K + j];
            if (s > INT32_MAX || s < INT32_MIN) bad = 1;
            acc[(size_t)t * N + o] = (int32_t)s;
        }
    return bad ? ORC_ERR_OVERFLOW : ORC_OK;
}

/* ---------------------------------------------------------------- bf16
 * double -> bf16 bit pattern, round to nearest, ties to even, done on the
 * double's own bits so that there is a single rounding (no detour through
 * fp32).  Handles zero, subnormal bf16 results, overflow to infinity, inf and
 * NaN.  bf16 = 1 sign, 8 exponent (bias 127), 7 fraction bits.
 */
uint16_t orc_bf16_from_double(double v)
{
    uint64_t u;
    memcpy(&u, &v, 8);
    uint16_t sign = (uint16_t)((u >> 63) << 15);
    int e = (int)((u >> 52) & 0x7FF);
    uint64_t frac = u & 0xFFFFFFFFFFFFFull;
    if (e == 0x7FF) return (uint16_t)(sign | 0x7F80 | (frac ? 0x40 : 0));
    if (e == 0 && frac == 0) return sign;
    if (e == 0) return sign; /* double subnormals are far below the smallest bf16 subnormal */
    int ue = e - 1023;                       /* unbiased exponent of 1.frac */
    uint64_t sig = frac | (1ull << 52);      /* 53-bit significand, value = sig * 2^(ue-52) */
    int shift;                               /* bits dropped from sig */
    int be;                                  /* biased bf16 exponent before rounding carry */
    if (ue >= -126) { shift = 52 - 7; be = ue + 127; }
    else { shift = 52 - 7 + (-126 - ue); be = 0; }   /* subnormal: fewer kept bits */
    if (shift > 62) return sign;             /* below half of the smallest subnormal */
    uint64_t kept = sig >> shift;
    uint64_t rem = sig & ((1ull << shift) - 1);
    uint64_t half = 1ull << (shift - 1);
    if (rem > half || (rem == half && (kept & 1))) kept += 1;
    uint32_t out;
    if (be == 0) out = (uint32_t)kept;       /* a carry into bit 7 lands on exponent 1: correct */
    else out = ((uint32_t)be << 7) + (uint32_t)(kept - 0x80) ; /* kept in [0x80, 0x100]; 0x100 carries into the exponent */
    if (out >= 0x7F80) out = 0x7F80;         /* overflow -> infinity */
    return (uint16_t)(sign | out);
}

void orc_bf16_from_double_array(const double *v, size_t n, uint16_t *out)
{
    for (size_t i = 0; i < n; ++i) out[i] = orc_bf16_from_double(v[i]);
}

double orc_bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* ---------------------------------------------------------------- epilogue
 * y[t][o] = acc[t][o] * dx[t] * dw[o] + bias[o]  (bias may be NULL), then
 * rounded once to bf16.  y_f64 (may be NULL) receives the unrounded value.
 */
int orc_dequant_bias(const int32_t *acc, const double *dx, const double *dw, const double *bias,
                     int M, int N, uint16_t *Y, double *y_f64)
{
    if (!acc || !dx || !dw || !Y || M < 0 || N < 1) return ORC_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < M; ++t)
        for (int o = 0; o < N; ++o) {
            double y = (double)acc[(size_t)t * N + o] * dx[t] * dw[o];
            if (bias) y += bias[o];
            if (y_f64) y_f64[(size_t)t * N + o] = y;
            Y[(size_t)t * N + o] = orc_bf16_from_double(y);
        }
    return ORC_OK;
}

/* ---------------------------------------------------------------- int4 packing
 * Canonical packing of 4-bit two's-complement codes in natural order: byte k of
 * a row holds element 2k in bits 0..3 and element 2k+1 in bits 4..7.  (The
 * paper gives no layout; this is the oracle's own reference packing.)
 */
int orc_pack_int4(const int8_t *q, int rows, int K, uint8_t *packed)
{
    if (!q || !packed || rows < 0 || K < 2 || (K & 1)) return ORC_ERR_ARG;
    for (size_t i = 0; i < (size_t)rows * K / 2; ++i) {
        int lo = q[2 * i], hi = q[2 * i + 1];
        if (lo < -8 || lo > 7 || hi < -8 || hi > 7) return ORC_ERR_OVERFLOW;
        packed[i] = (uint8_t)((lo & 0xF) | ((hi & 0xF) << 4));
    }
    return ORC_OK;
}

int orc_unpack_int4(const uint8_t *packed, int rows, int K, int8_t *q)
{
    if (!q || !packed || rows < 0 || K < 2 || (K & 1)) return ORC_ERR_ARG;
    for (size_t i = 0; i < (size_t)rows * K / 2; ++i) {
        int lo = packed[i] & 0xF, hi = packed[i] >> 4;
        q[2 * i] = (int8_t)(lo >= 8 ? lo - 16 : lo);
        q[2 * i + 1] = (int8_t)(hi >= 8 ? hi - 16 : hi);
    }
    return ORC_OK;
}
