// Online kernel 2: int4 x int4 GEMM with int32 accumulation on the int8 matrix cores and a
// fused dequantise + bias epilogue (paper Sec. 3.2, granularity paragraph: the scales are
// constant along the summed dimension, so the sum stays in integers and is rescaled once).
//
//   acc[t, o] = sum_j Xq[t, j] * Wq[o, j]
//   Y[t, o]   = bf16( acc[t, o] * sx[t] * sw[o] + bias[o] )
//
// Tiles of packed codes are staged in LDS as they are in memory (two codes per byte).  A
// wavefront expands them to int8 in registers right before the MFMA: each code is kept in
// the HIGH nibble of its byte (v & 0xF0F0F0F0 for the odd codes, (v << 4) & 0xF0F0F0F0 for
// the even ones), i.e. as 16 * code with the sign in place, so no sign extension is needed.
// Both operands are expanded the same way, hence the accumulator is exactly 256 * acc
// (|256 * acc| <= 256 * 64 * 8192 = 2^27) and the factor is removed exactly afterwards.
// The even/odd split permutes the codes inside a K-step identically for both operands, which
// leaves every dot product unchanged.
//
// The MFMA takes the weights as its row operand and the activations as its column operand,
// so that a lane ends up with 4 consecutive output channels of one token: 8-byte bf16 stores.
#include "qvggt_common.h"

namespace qvggt {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

namespace gemm {
constexpr int BM = 128;          // tokens per block tile
constexpr int BN = 128;          // output channels per block tile
constexpr int BKB = 64;          // packed bytes per row per K-tile (128 codes)
constexpr int LDS_STRIDE = 72;   // row pitch in LDS: 64 B + 8 B pad keeps 8-byte fragment reads conflict-free
constexpr int THREADS = 256;     // 4 waves as 2 (tokens) x 2 (channels), 64 x 64 per wave
}  // namespace gemm

__device__ inline v4i expand_codes(uint2 p)
{
    v4i r;
    r[0] = (int)(p.x & 0xF0F0F0F0u);
    r[1] = (int)((p.x << 4) & 0xF0F0F0F0u);
    r[2] = (int)(p.y & 0xF0F0F0F0u);
    r[3] = (int)((p.y << 4) & 0xF0F0F0F0u);
    return r;
}

__global__ __launch_bounds__(gemm::THREADS) void w4a4_gemm_kernel(
    const uint8_t *__restrict__ Xq, const float *__restrict__ sx, const uint8_t *__restrict__ Wq,
    const float *__restrict__ sw, const uint16_t *__restrict__ bias, int M, int N, int K,
    uint16_t *__restrict__ Y, int32_t *__restrict__ acc_debug, int tiles_n)
{
    using namespace gemm;
    __shared__ __attribute__((aligned(16))) uint8_t sX[2][BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) uint8_t sW[2][BN * LDS_STRIDE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int KB = K >> 1;             // packed bytes per row
    const int ktiles = KB / BKB;

    // global -> LDS staging: a thread moves 16 bytes of two rows of each operand per K-tile
    const int ld_row = tid >> 2, ld_seg = tid & 3;
    const uint8_t *gX[2], *gW[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        int rm = min(m0 + ld_row + 64 * p, M - 1);   // rows past the end re-read the last row; never stored
        int rn = min(n0 + ld_row + 64 * p, N - 1);
        gX[p] = Xq + (size_t)rm * KB + ld_seg * 16;
        gW[p] = Wq + (size_t)rn * KB + ld_seg * 16;
    }
    uint4 rX[2], rW[2];
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            rX[p] = *reinterpret_cast<const uint4 *>(gX[p] + (size_t)kt * BKB);
            rW[p] = *reinterpret_cast<const uint4 *>(gW[p] + (size_t)kt * BKB);
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int off = (ld_row + 64 * p) * LDS_STRIDE + ld_seg * 16;
            *reinterpret_cast<uint2 *>(&sX[buf][off]) = make_uint2(rX[p].x, rX[p].y);
            *reinterpret_cast<uint2 *>(&sX[buf][off + 8]) = make_uint2(rX[p].z, rX[p].w);
            *reinterpret_cast<uint2 *>(&sW[buf][off]) = make_uint2(rW[p].x, rW[p].y);
            *reinterpret_cast<uint2 *>(&sW[buf][off + 8]) = make_uint2(rW[p].z, rW[p].w);
        }
    };

    v16i acc[2][2];   // [channel sub-tile j][token sub-tile i]
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0;

    load_tile(0);
    store_tile(0);
    __syncthreads();

    // fragment addresses: lane (l % 32) is the row inside a 32-row sub-tile, (l / 32) picks 8 of the 16 bytes of a K-step
    const int frag_off = (lane & 31) * LDS_STRIDE + (lane >> 5) * 8;
    for (int kt = 0; kt < ktiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < ktiles) load_tile(kt + 1);
#pragma unroll
        for (int ks = 0; ks < BKB / 16; ++ks) {
            v4i fw[2], fx[2];
#pragma unroll
            for (int j = 0; j < 2; ++j)
                fw[j] = expand_codes(*reinterpret_cast<const uint2 *>(&sW[buf][(wn * 64 + j * 32) * LDS_STRIDE + frag_off + ks * 16]));
#pragma unroll
            for (int i = 0; i < 2; ++i)
                fx[i] = expand_codes(*reinterpret_cast<const uint2 *>(&sX[buf][(wm * 64 + i * 32) * LDS_STRIDE + frag_off + ks * 16]));
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[j], fx[i], acc[j][i], 0, 0, 0);
        }
        if (kt + 1 < ktiles) store_tile(buf ^ 1);
        __syncthreads();
    }

    // epilogue.  32x32 result layout: lane l holds column (l % 32) and rows 8*(r/4) + 4*(l/32) + r%4.
    // Rows are output channels, the column is the token.
    const int c = lane & 31, g = lane >> 5;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int m = m0 + wm * 64 + i * 32 + c;
        if (m >= M) continue;
        const float sxm = sx[m] * (1.0f / 256.0f);
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * 64 + j * 32 + 8 * q + 4 * g;
                if (n >= N) continue;
                const float4 swn = *reinterpret_cast<const float4 *>(sw + n);
                float b0 = 0.f, b1 = 0.f, b2 = 0.f, b3 = 0.f;
                if (bias != nullptr) {
                    uint2 bb = *reinterpret_cast<const uint2 *>(bias + n);
                    b0 = __uint_as_float(bb.x << 16); b1 = __uint_as_float(bb.x & 0xFFFF0000u);
                    b2 = __uint_as_float(bb.y << 16); b3 = __uint_as_float(bb.y & 0xFFFF0000u);
                }
                const int a0 = acc[j][i][4 * q], a1 = acc[j][i][4 * q + 1], a2 = acc[j][i][4 * q + 2], a3 = acc[j][i][4 * q + 3];
                const float y0 = fmaf((float)a0 * sxm, swn.x, b0), y1 = fmaf((float)a1 * sxm, swn.y, b1);
                const float y2 = fmaf((float)a2 * sxm, swn.z, b2), y3 = fmaf((float)a3 * sxm, swn.w, b3);
                *reinterpret_cast<uint2 *>(Y + (size_t)m * N + n) = make_uint2(pack_bf16x2(y0, y1), pack_bf16x2(y2, y3));
                if (acc_debug != nullptr)
                    *reinterpret_cast<int4 *>(acc_debug + (size_t)m * N + n) = make_int4(a0 >> 8, a1 >> 8, a2 >> 8, a3 >> 8);
            }
    }
}

hipError_t run_w4a4_gemm(const uint8_t *Xq, const float *sx, const uint8_t *Wq, const float *sw,
                         const void *bias, int M, int N, int K, void *Y, int32_t *acc_debug, hipStream_t stream)
{
    if (M <= 0) return hipSuccess;
    const int tiles_m = (M + gemm::BM - 1) / gemm::BM, tiles_n = (N + gemm::BN - 1) / gemm::BN;
    w4a4_gemm_kernel<<<tiles_m * tiles_n, gemm::THREADS, 0, stream>>>(
        Xq, sx, Wq, sw, reinterpret_cast<const uint16_t *>(bias), M, N, K, reinterpret_cast<uint16_t *>(Y),
        acc_debug, tiles_n);
    return hipGetLastError();
}

}  // namespace qvggt
