/* Runs every function of the C oracle on exactly sized heap buffers, for a build with AddressSanitizer and
 * UndefinedBehaviorSanitizer (tests/test_sanitizers.py compiles this file together with oracle/dsfq_oracle.c).
 * A read or write one element past a buffer, a signed overflow or a misaligned access aborts the program; the
 * plain checks below only make sure that the calls did their work (round trips, orthogonality). */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int orc_hadamard_recursive(int K, int8_t *H);
int orc_hadamard_popcount(int K, int8_t *H);
int orc_hadamard_paley(int m, int8_t *H);
int orc_hadamard_general(int K, int8_t *H);
int orc_rotate(const double *X, int rows, int K, const int8_t *pre, const int8_t *post, double *Xr);
int orc_col_absmax(const double *A, int rows, int K, double *out);
int orc_smooth_factor(const double *a, const double *w, int K, double alpha, double floor_, double *c);
int orc_scale_columns(double *A, int rows, int K, const double *c, int inverse);
int orc_quantize_rows(const double *A, int rows, int K, int bits, double *delta, int8_t *q);
int orc_quantize_rows_static(const double *A, int rows, int K, int bits, const double *delta, int8_t *q);
int orc_int_gemm(const int8_t *qx, const int8_t *qw, int M, int N, int K, int32_t *acc);
uint16_t orc_bf16_from_double(double v);
void orc_bf16_from_double_array(const double *v, size_t n, uint16_t *out);
double orc_bf16_to_double(uint16_t b);
int orc_dequant_bias(const int32_t *acc, const double *dx, const double *dw, const double *bias, int M, int N,
                     uint16_t *Y, double *y_f64);
int orc_pack_int4(const int8_t *q, int rows, int K, uint8_t *packed);
int orc_unpack_int4(const uint8_t *packed, int rows, int K, int8_t *q);

static int failures = 0;
#define CHECK(cond)                                                                   \
    do {                                                                              \
        if (!(cond)) { fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
    } while (0)

static uint64_t state = 0x9e3779b97f4a7c15ull;
static double uniform(void)   /* splitmix64, in (-1, 1) */
{
    uint64_t z = (state += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    z ^= z >> 31;
    return (double)(z >> 11) / (double)(1ull << 52) - 1.0;
}

static void *exact(size_t bytes) { void *p = malloc(bytes ? bytes : 1); if (!p) abort(); return p; }

static void hadamards(void)
{
    const int sizes[] = {1, 2, 4, 64, 12, 20, 28, 24, 40, 56, 96, 128};
    for (unsigned i = 0; i < sizeof sizes / sizeof *sizes; ++i) {
        const int K = sizes[i];
        int8_t *H = exact((size_t)K * K), *G = exact((size_t)K * K);
        CHECK(orc_hadamard_general(K, H) == 0);
        if ((K & (K - 1)) == 0) {
            CHECK(orc_hadamard_recursive(K, G) == 0 && memcmp(G, H, (size_t)K * K) == 0);
            CHECK(orc_hadamard_popcount(K, G) == 0 && memcmp(G, H, (size_t)K * K) == 0);
        } else if (K == 12 || K == 20 || K == 28) {
            CHECK(orc_hadamard_paley(K, G) == 0 && memcmp(G, H, (size_t)K * K) == 0);
        }
        for (int a = 0; a < K; ++a)
            for (int b = a; b < K; ++b) {
                int dot = 0;
                for (int j = 0; j < K; ++j) dot += H[a * K + j] * H[b * K + j];
                CHECK(dot == (a == b ? K : 0));
            }
        free(H);
        free(G);
    }
    int8_t one;
    CHECK(orc_hadamard_general(36, &one) != 0);    /* refused before anything is written */
    CHECK(orc_hadamard_recursive(3, &one) != 0);
}

static void layer(int M, int N, int K, int bits)
{
    double *X = exact(sizeof(double) * M * K), *W = exact(sizeof(double) * N * K);
    double *Xr = exact(sizeof(double) * M * K), *Wr = exact(sizeof(double) * N * K);
    int8_t *pre = exact(K), *post = exact(K);
    for (int i = 0; i < M * K; ++i) X[i] = uniform() * (i % 37 == 0 ? 40.0 : 1.0);
    for (int i = 0; i < N * K; ++i) W[i] = uniform() * 0.05;
    for (int i = 0; i < K; ++i) { pre[i] = uniform() < 0 ? -1 : 1; post[i] = uniform() < 0 ? -1 : 1; }
    CHECK(orc_rotate(X, M, K, pre, NULL, Xr) == 0);
    CHECK(orc_rotate(W, N, K, pre, post, Wr) == 0);
    CHECK(orc_rotate(W, N, K, pre, NULL, Wr) == 0);
    if (M > 0) {   /* the rotation keeps each row's length */
        double a = 0, b = 0;
        for (int j = 0; j < K; ++j) { a += X[j] * X[j]; b += Xr[j] * Xr[j]; }
        CHECK(fabs(a - b) <= 1e-9 * a);
    }
    double *ax = exact(sizeof(double) * K), *aw = exact(sizeof(double) * K), *c = exact(sizeof(double) * K);
    CHECK(orc_col_absmax(Xr, M, K, ax) == 0 && orc_col_absmax(Wr, N, K, aw) == 0);
    CHECK(orc_smooth_factor(ax, aw, K, 0.5, 1e-5, c) == 0);
    CHECK(orc_scale_columns(Xr, M, K, c, 1) == 0 && orc_scale_columns(Wr, N, K, c, 0) == 0);
    double *dx = exact(sizeof(double) * M), *dw = exact(sizeof(double) * N), *bias = exact(sizeof(double) * N);
    int8_t *qx = exact((size_t)M * K), *qw = exact((size_t)N * K), *qs = exact((size_t)M * K);
    CHECK(orc_quantize_rows(Xr, M, K, bits, dx, qx) == 0 && orc_quantize_rows(Wr, N, K, bits, dw, qw) == 0);
    CHECK(orc_quantize_rows_static(Xr, M, K, bits, dx, qs) == 0);
    CHECK(memcmp(qx, qs, (size_t)M * K) == 0);     /* a row's own step reproduces its codes */
    int32_t *acc = exact(sizeof(int32_t) * M * N);
    CHECK(orc_int_gemm(qx, qw, M, N, K, acc) == 0);
    for (int i = 0; i < N; ++i) bias[i] = uniform();
    uint16_t *Y = exact(sizeof(uint16_t) * M * N);
    double *y64 = exact(sizeof(double) * M * N);
    CHECK(orc_dequant_bias(acc, dx, dw, bias, M, N, Y, y64) == 0);
    CHECK(orc_dequant_bias(acc, dx, dw, NULL, M, N, Y, NULL) == 0);
    if (bits == 4 && K % 2 == 0) {
        uint8_t *packed = exact((size_t)M * K / 2);
        int8_t *back = exact((size_t)M * K);
        CHECK(orc_pack_int4(qx, M, K, packed) == 0 && orc_unpack_int4(packed, M, K, back) == 0);
        CHECK(memcmp(back, qx, (size_t)M * K) == 0);
        free(packed);
        free(back);
    }
    free(X); free(W); free(Xr); free(Wr); free(pre); free(post); free(ax); free(aw); free(c);
    free(dx); free(dw); free(bias); free(qx); free(qw); free(qs); free(acc); free(Y); free(y64);
}

static void bf16(void)
{
    const double v[] = {0.0, -0.0, 1.0, 1.00390625, 1.01171875, -3.3895313892515355e38, 3.4e38, 1e39, -1e39, 1e-45, 9.2e-41,
                        1.1754943508222875e-38, 5e-324, INFINITY, -INFINITY, NAN};
    const size_t n = sizeof v / sizeof *v;
    uint16_t *out = exact(sizeof(uint16_t) * n);
    orc_bf16_from_double_array(v, n, out);
    for (size_t i = 0; i < n; ++i) {
        CHECK(out[i] == orc_bf16_from_double(v[i]));
        const double back = orc_bf16_to_double(out[i]);
        CHECK(isnan(v[i]) ? isnan(back) : orc_bf16_from_double(back) == out[i]);
    }
    for (unsigned b = 0; b < 0x10000u; ++b) {       /* every finite pattern survives the round trip */
        const double d = orc_bf16_to_double((uint16_t)b);
        if (!isnan(d)) CHECK(orc_bf16_from_double(d) == (uint16_t)b);
    }
    free(out);
}

int main(void)
{
    hadamards();
    layer(0, 16, 128, 4);        /* no rows */
    layer(1, 16, 128, 4);
    layer(37, 48, 128, 4);       /* ragged against any tiling */
    layer(5, 16, 96, 4);         /* 2^n * 12 */
    layer(3, 16, 160, 8);        /* 2^n * 20, wide codes */
    layer(9, 32, 448, 6);        /* 2^n * 28 */
    layer(7, 16, 1024, 4);
    bf16();
    printf("oracle driver: %d failed checks\n", failures);
    return failures ? 1 : 0;
}
