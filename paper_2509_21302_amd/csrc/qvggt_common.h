// Shared device-side helpers of the qvggt HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qvggt {

constexpr int kWave = 64;
constexpr int kMinK = 128;
constexpr int kMaxK = 8192;

// Position of natural element e inside a packed row of K codes.  Two codes share a byte:
// position p lives in byte p / 2, low nibble when p is even.  The same map is used for
// activations and weights, so integer dot products do not depend on it.
__host__ __device__ inline int code_position(int e, int /*K*/) { return e; }
// Inverse of code_position: the natural element stored at position p.
__host__ __device__ inline int code_element(int p, int /*K*/) { return p; }

__device__ inline float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// two floats -> packed bf16 pair (round to nearest even), lo in bits 0..15
__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
    bf2 p;
    p[0] = (__bf16)lo;
    p[1] = (__bf16)hi;
    return *reinterpret_cast<uint32_t *>(&p);
}

__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) v = fmaxf(v, __shfl_xor(v, m));
    return v;
}

}  // namespace qvggt
