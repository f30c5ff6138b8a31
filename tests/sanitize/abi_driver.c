/* Host-side exercise of the C-ABI's argument validation and size arithmetic for a sanitizer build.
 *
 * Built by tests/test_sanitizers.py against a copy of the library whose host code carries AddressSanitizer and
 * UndefinedBehaviorSanitizer instrumentation.  Every call here must be rejected (or answered) on the host before any
 * HIP call, so the program runs on a machine without a GPU; the "device" pointers are aligned addresses that are never
 * dereferenced.  Exit status 0 = every call returned what the header documents; a sanitizer report aborts the program. */
#include <limits.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include "qvggt.h"

static int failures = 0;

#define EXPECT(call, want)                                                                         \
    do {                                                                                           \
        int got_ = (call);                                                                         \
        if (got_ != (want)) {                                                                      \
            fprintf(stderr, "%s:%d: %s returned %d (%s), expected %d\n", __FILE__, __LINE__, #call, \
                    got_, qvggt_status_string(got_), (int)(want));                                 \
            ++failures;                                                                            \
        }                                                                                          \
    } while (0)

int main(void)
{
    /* never dereferenced: validation fails first in every call below */
    void *dev = (void *)(uintptr_t)0x7f0000000000ull;
    void *odd = (void *)((uintptr_t)dev + 4);
    const int M = 300, N = 1024, K = 1024;

    for (int s = -2; s < 12; ++s)
        if (!qvggt_status_string(s) || !qvggt_status_string(s)[0]) { fprintf(stderr, "status %d has no text\n", s); ++failures; }

    /* size arithmetic at the ends of the argument range: no signed overflow, no wrap */
    const int big[] = {0, 1, 127, 128, 129, 137400, 1 << 20, INT_MAX - 255, INT_MAX};
    const int Ks[] = {-1, 0, 64, 128, 1024, 1536, 2048, 4096, 8192, INT_MAX};
    size_t sink = 0;
    for (unsigned a = 0; a < sizeof big / sizeof *big; ++a)
        for (unsigned b = 0; b < sizeof Ks / sizeof *Ks; ++b) {
            sink += qvggt_e2m3_bytes(big[a], Ks[b]);
            sink += qvggt_i8b_bytes(big[a], Ks[b]);
            for (unsigned c = 0; c < sizeof big / sizeof *big; ++c) {
                sink += qvggt_workspace_bytes(big[a], big[c], Ks[b]);
                sink += qvggt_workspace_bytes_e2m3(big[a], big[c], Ks[b]);
                sink += qvggt_workspace_bytes_i8(big[a], big[c], Ks[b]);
                sink += qvggt_workspace_bytes_i8b(big[a], big[c], Ks[b]);
                sink += qvggt_calib_workspace_bytes(big[a], big[c], Ks[b]);
            }
            sink += qvggt_nfds_workspace_bytes(big[a], (long long)Ks[b] * 1000003ll, QVGGT_F32);
            sink += qvggt_nfds_workspace_bytes(big[a], LLONG_MAX, QVGGT_BF16);
        }
    if (qvggt_e2m3_bytes(128, 1024) != 128u * 1024u * 3u / 4u) { fprintf(stderr, "e2m3 bytes of one block\n"); ++failures; }
    if (qvggt_own_workspace_bytes() != QVGGT_OWN_WORKSPACE_BYTES) { fprintf(stderr, "own workspace size\n"); ++failures; }
    if (qvggt_gelu_table_bytes() != QVGGT_GELU_TABLE_BYTES) { fprintf(stderr, "gelu table size\n"); ++failures; }

    /* one wrong argument per call */
    EXPECT(qvggt_rotate_smooth_quant(NULL, QVGGT_BF16, M, K, NULL, NULL, dev, dev, NULL), QVGGT_ERR_NULL);
    EXPECT(qvggt_rotate_smooth_quant(dev, QVGGT_BF16, -1, K, NULL, NULL, dev, dev, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_rotate_smooth_quant(dev, QVGGT_BF16, M, 1000, NULL, NULL, dev, dev, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_rotate_smooth_quant(dev, 7, M, K, NULL, NULL, dev, dev, NULL), QVGGT_ERR_DTYPE);
    EXPECT(qvggt_rotate_smooth_quant(odd, QVGGT_BF16, M, K, NULL, NULL, dev, dev, NULL), QVGGT_ERR_ALIGN);
    EXPECT(qvggt_rotate_smooth_quant_static(dev, QVGGT_BF16, M, K, NULL, NULL, dev, 2, dev, dev, NULL), QVGGT_ERR_ARG);
    EXPECT(qvggt_rotate_smooth_quant_asym(dev, QVGGT_BF16, M, K, NULL, NULL, dev, dev, NULL, NULL), QVGGT_ERR_NULL);
    EXPECT(qvggt_layernorm_rotate_smooth_quant(dev, QVGGT_BF16, M, K, NULL, NULL, -1.0f, NULL, NULL, dev, dev, NULL), QVGGT_ERR_ARG);
    EXPECT(qvggt_layernorm_rotate_smooth_quant(dev, QVGGT_BF16, M, 8192, NULL, NULL, 1e-5f, NULL, NULL, dev, dev, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_gelu_rotate_smooth_quant(dev, QVGGT_BF16, M, K, NULL, NULL, NULL, dev, dev, NULL), QVGGT_ERR_NULL);
    EXPECT(qvggt_gelu_rotate_smooth_quant(dev, QVGGT_F32, M, K, NULL, NULL, dev, dev, dev, NULL), QVGGT_ERR_DTYPE);
    EXPECT(qvggt_gelu_table(NULL, NULL), QVGGT_ERR_NULL);
    EXPECT(qvggt_w4a4_gemm(dev, dev, dev, dev, NULL, M, 24, K, dev, NULL, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_w4a4_gemm(dev, dev, dev, NULL, NULL, M, N, K, dev, NULL, NULL), QVGGT_ERR_NULL);
    EXPECT(qvggt_e2m3_gemm(dev, dev, dev, dev, NULL, M, N, 96, dev, NULL, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_e2m3_gemm(dev, dev, odd, dev, NULL, M, N, K, dev, NULL, NULL), QVGGT_ERR_ALIGN);
    EXPECT(qvggt_linear(dev, QVGGT_BF16, M, N, K, NULL, NULL, dev, dev, NULL, dev, dev, 16, NULL), QVGGT_ERR_WORKSPACE);
    EXPECT(qvggt_linear_e2m3(dev, QVGGT_BF16, M, N, K, NULL, NULL, dev, dev, NULL, dev, dev, 16, NULL), QVGGT_ERR_WORKSPACE);
    EXPECT(qvggt_linear_e2m3(dev, QVGGT_BF16, M, N, K, NULL, NULL, dev, dev, NULL, dev, NULL, (size_t)-1, NULL), QVGGT_ERR_NULL);
    EXPECT(qvggt_linear_i8(dev, QVGGT_BF16, M, N, K, NULL, NULL, 9, dev, dev, NULL, dev, dev, (size_t)-1, NULL), QVGGT_ERR_ARG);
    EXPECT(qvggt_linear_i8b(dev, QVGGT_BF16, M, N, K, NULL, NULL, 8, dev, dev, NULL, dev, dev, 0, NULL), QVGGT_ERR_WORKSPACE);
    EXPECT(qvggt_linear_e2m3_own_workspace(dev, QVGGT_BF16, INT_MAX, N, K, NULL, NULL, dev, dev, NULL, dev, NULL), QVGGT_ERR_WORKSPACE);
    EXPECT(qvggt_linear_e2m3_own_workspace(dev, QVGGT_BF16, M, N, 1000, NULL, NULL, dev, dev, NULL, dev, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_codes_to_e2m3(dev, 0, K, dev, NULL, NULL), QVGGT_ERR_NULL);
    EXPECT(qvggt_codes_to_e2m3(dev, M, 96, dev, dev, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_prep_weights(dev, QVGGT_F32, N, K, dev, NULL, 1.5f, dev, dev, dev, NULL), QVGGT_ERR_ARG);
    EXPECT(qvggt_prep_weights_given(dev, QVGGT_F32, N, K, dev, NULL, dev, 3, dev, dev, dev, NULL), QVGGT_ERR_ARG);
    EXPECT(qvggt_prep_weights_i8(dev, QVGGT_F32, N, K, NULL, NULL, 0.5f, 8, NULL, dev, dev, NULL), QVGGT_ERR_NULL);
    EXPECT(qvggt_rotated_col_absmax(dev, QVGGT_F32, M, 100, NULL, dev, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_pack_int4(dev, M, 7, dev, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_unpack_int4(NULL, M, K, dev, NULL), QVGGT_ERR_NULL);
    EXPECT(qvggt_layout_int8(dev, M, K, dev, 2, NULL), QVGGT_ERR_ARG);
    EXPECT(qvggt_int8_to_blocks(dev, M, 100, dev, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_nfds_moments(dev, QVGGT_F32, 4, 0, dev, dev, dev, (size_t)-1, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_nfds_scores(dev, dev, 8, 4, -1.0, dev, NULL), QVGGT_ERR_ARG);
    EXPECT(qvggt_nfds_keep_lowest(dev, 8, 1.5, dev, NULL), QVGGT_ERR_ARG);
    EXPECT(qvggt_nfds_kmeans_step(dev, 10, 4, 0, dev, dev, dev, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_rotate_rows(dev, QVGGT_F32, M, 96, NULL, dev, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_calib_loss_grad(dev, dev, dev, NULL, dev, dev, dev, 8, 16, 128, 4, dev, dev, dev, dev, dev, 0, NULL), QVGGT_ERR_WORKSPACE);
    EXPECT(qvggt_calib_loss_grad(dev, dev, dev, NULL, dev, dev, dev, 8, 16, 128, 9, dev, dev, dev, dev, dev, (size_t)-1, NULL), QVGGT_ERR_ARG);
    EXPECT(qvggt_calib_descent_step(dev, dev, -1, 0.1f, 0.0f, NULL), QVGGT_ERR_SHAPE);
    EXPECT(qvggt_mfma_ceiling(5, 10, dev, NULL), QVGGT_ERR_ARG);

    printf("abi driver: %d mismatches (sizes checksum %zu)\n", failures, sink);
    return failures ? 1 : 0;
}
