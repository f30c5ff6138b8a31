// One row per wavefront: how a row of K values (K a power of two, 128 .. 8192) is spread over the 64 lanes, loaded, and taken
// through the unnormalised Walsh-Hadamard transform.  Shared by the generic kernel 1 and the calibration-side rotation.
//
// A row of K values lives in K/64 registers per lane; element e = c*(64*V) + lane*V + i sits in register c*V + i, where
// V = min(8, K/64) is the run a lane loads contiguously (16 bytes of bf16 when V = 8, so a wave reads 1 KiB per load
// instruction).  The transform is one butterfly per index bit (the Hadamard matrix is a Kronecker power of H_2, paper Sec. 3.2):
// bits inside i and c are register-to-register, the six lane bits go through cross-lane exchanges.
#pragma once
#include "qvggt_common.h"

namespace qvggt {

template <int K>
struct RowMap {
    static constexpr int V = (K >= 512) ? 8 : K / 64;   // contiguous elements per lane per chunk
    static constexpr int C = K / (64 * V);              // chunks
    static constexpr int R = V * C;                     // registers per lane
};

template <int K, bool F32>
__device__ inline void load_row(const void *X, size_t row, int lane, float (&x)[RowMap<K>::R])
{
    constexpr int V = RowMap<K>::V, C = RowMap<K>::C;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const size_t e0 = row * (size_t)K + (size_t)c * 64 * V + (size_t)lane * V;
        if constexpr (F32) {
            const float *p = reinterpret_cast<const float *>(X) + e0;
            if constexpr (V >= 4) {
#pragma unroll
                for (int q = 0; q < V / 4; ++q) {
                    float4 v = *reinterpret_cast<const float4 *>(p + 4 * q);
                    x[c * V + 4 * q + 0] = v.x; x[c * V + 4 * q + 1] = v.y;
                    x[c * V + 4 * q + 2] = v.z; x[c * V + 4 * q + 3] = v.w;
                }
            } else {
                float2 v = *reinterpret_cast<const float2 *>(p);
                x[c * V] = v.x; x[c * V + 1] = v.y;
            }
        } else {
            const uint16_t *p = reinterpret_cast<const uint16_t *>(X) + e0;
            uint32_t w[V / 2];
            if constexpr (V == 8) {
                uint4 v = *reinterpret_cast<const uint4 *>(p);
                w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
            } else if constexpr (V == 4) {
                uint2 v = *reinterpret_cast<const uint2 *>(p);
                w[0] = v.x; w[1] = v.y;
            } else {
                w[0] = *reinterpret_cast<const uint32_t *>(p);
            }
#pragma unroll
            for (int q = 0; q < V / 2; ++q) {
                x[c * V + 2 * q] = __uint_as_float(w[q] << 16);
                x[c * V + 2 * q + 1] = __uint_as_float(w[q] & 0xFFFF0000u);
            }
        }
    }
}

// In-place unnormalised Walsh-Hadamard transform of a row spread over one wavefront.
template <int K>
__device__ inline void fwht_row(float (&x)[RowMap<K>::R], int lane)
{
    constexpr int V = RowMap<K>::V, R = RowMap<K>::R;
    // index bits inside the lane's contiguous run
#pragma unroll
    for (int h = 1; h < V; h <<= 1)
#pragma unroll
        for (int r = 0; r < R; ++r)
            if ((r & h) == 0) { float a = x[r], b = x[r + h]; x[r] = a + b; x[r + h] = a - b; }
    // the six lane bits
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
        const bool upper = (lane & m) != 0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float p = __shfl_xor(x[r], m);
            x[r] = upper ? p - x[r] : x[r] + p;
        }
    }
    // chunk bits
#pragma unroll
    for (int h = V; h < R; h <<= 1)
#pragma unroll
        for (int r = 0; r < R; ++r)
            if ((r & h) == 0) { float a = x[r], b = x[r + h]; x[r] = a + b; x[r + h] = a - b; }
}

}  // namespace qvggt
