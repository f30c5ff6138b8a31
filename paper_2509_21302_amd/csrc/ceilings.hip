// Measurement helper of the benchmark: register-only loops of the matrix instructions the two GEMMs are built on, so that a
// run can state, beside the published peak, what the matrix pipes deliver on this board when nothing has to be fed to them
// (one wave per SIMD, sixteen independent 32x32 accumulators, operands that stay in registers).  No memory traffic.
#include "qvggt_common.h"

namespace qvggt {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

// KIND 0: v_mfma_i32_32x32x32_i8 (the packed-code and int8-code GEMMs); KIND 1: v_mfma_f32_32x32x64_f8f6f4 on E2M3 operands
template <int KIND>
__global__ __launch_bounds__(256, 1) void mfma_ceiling_kernel(int iters, float *__restrict__ sink)
{
    // operands: small codes as the GEMMs see them (int8 values 16 * code, resp. E2M3 patterns), different per lane
    const uint32_t seed = threadIdx.x * 2654435761u + blockIdx.x * 40503u;
    float total = 0.0f;
    if constexpr (KIND == 0) {
        v4i A[4], B[4];
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                A[f][e] = (int)((seed >> (f + e)) * 0x9E3779B1u) & (int)0xF0F0F0F0u;
                B[f][e] = (int)((seed >> (f + e + 3)) * 0x85EBCA6Bu) & (int)0xF0F0F0F0u;
            }
        v16i acc[16];
#pragma unroll
        for (int t = 0; t < 16; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int t = 0; t < 16; ++t) acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[t / 4], B[t % 4], acc[t], 0, 0, 0);
        }
#pragma unroll
        for (int t = 0; t < 16; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) total += (float)acc[t][r];
    } else {
        v8i A[4], B[4];
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                A[f][e] = e < 6 ? (int)((seed >> (f + e)) * 0x9E3779B1u) : 0;
                B[f][e] = e < 6 ? (int)((seed >> (f + e + 3)) * 0x85EBCA6Bu) : 0;
            }
        v16f acc[16];
#pragma unroll
        for (int t = 0; t < 16; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int t = 0; t < 16; ++t)
                acc[t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A[t / 4], B[t % 4], acc[t], 2, 2, 0, 0, 0, 0);
        }
#pragma unroll
        for (int t = 0; t < 16; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) total += acc[t][r];
    }
    sink[blockIdx.x * 256 + threadIdx.x] = total;
}

hipError_t run_mfma_ceiling(int kind, int iters, float *sink, hipStream_t stream)
{
    if (kind == 0) mfma_ceiling_kernel<0><<<256, 256, 0, stream>>>(iters, sink);
    else mfma_ceiling_kernel<1><<<256, 256, 0, stream>>>(iters, sink);
    return hipGetLastError();
}

}  // namespace qvggt
