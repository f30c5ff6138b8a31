// Shared device-side helpers of the qvggt HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qvggt {

constexpr int kWave = 64;
constexpr int kMinK = 128;
constexpr int kMaxK = 8192;
// A quantization step below the smallest normal fp32 number (2^-126) counts as 0: the row gets step 0 and codes 0 (a dynamic
// step), or codes 0 (a given one).  Such a step could not be inverted in fp32 (7 / absmax would overflow).
constexpr float kMinStep = 1.17549435e-38f;

// Width argument of the quantizing launchers: 4 = 4-bit codes packed two per byte; kInt8Container + b = b-bit codes
// (4 <= b <= 8) stored one per byte as int8 (so that weights and activations of one int8 GEMM may take different widths)
constexpr int kInt8Container = 32;
inline int code_width(int bits) { return bits >= kInt8Container ? bits - kInt8Container : bits; }

// Position of natural element e inside a packed row of K codes.  Two codes share a byte:
// position p lives in byte p / 2, low nibble when p is even.  The same map is used for
// activations and weights, so integer dot products do not depend on it.
//
// For K = 1024, 2048, 4096 the map is the one the matrix-core rotation kernel produces
// naturally: with e = 128*hb + 32*nt + c (c < 32, nt < 4), position = c*(K/32) + nt + 4*hb',
// where hb' = hb except for K = 4096, which swaps bits 3 and 4 of hb.  Other K keep natural order.
__host__ __device__ inline bool layout_is_permuted(int K) { return K == 1024 || K == 2048 || K == 4096; }

__host__ __device__ inline int swap_bits_3_4(int v) { return (v & ~0x18) | ((v & 8) << 1) | ((v & 16) >> 1); }

__host__ __device__ inline int code_position(int e, int K)
{
    if (!layout_is_permuted(K)) return e;
    int c = e & 31, nt = (e >> 5) & 3, hb = e >> 7;
    if (K == 4096) hb = swap_bits_3_4(hb);
    return c * (K / 32) + nt + 4 * hb;
}
// Inverse of code_position: the natural element stored at position p.
__host__ __device__ inline int code_element(int p, int K)
{
    if (!layout_is_permuted(K)) return p;
    int c = p / (K / 32), l = p % (K / 32);
    int nt = l & 3, hb = l >> 2;
    if (K == 4096) hb = swap_bits_3_4(hb);
    return 128 * hb + 32 * nt + c;
}

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

// Lanes of one wave hand data to each other through a wave-private LDS area.  LDS operations of a wave execute in order, so
// no instruction has to separate the writes from the reads; the compiler, however, must be told that a lane is about to
// read what other lanes wrote (it may otherwise treat such a read as a repeat of an earlier one).
__device__ inline void lanes_exchange_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Maximum over groups of lanes without going through LDS: four DPP steps inside a row of 16 lanes (quad permutes, then
// mirrors: after each step every lane of the group holds the group's maximum), then the gfx950 row swaps across rows.
template <int CTRL>
__device__ inline float dpp_max_step(float v)
{
    const int p = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false);
    return fmaxf(v, __int_as_float(p));
}
__device__ inline float max_over_16_lanes(float v)
{
    v = dpp_max_step<0xB1>(v);     // quad_perm [1, 0, 3, 2]
    v = dpp_max_step<0x4E>(v);     // quad_perm [2, 3, 0, 1]
    v = dpp_max_step<0x141>(v);    // row_half_mirror
    v = dpp_max_step<0x140>(v);    // row_mirror
    return v;
}
__device__ inline float max_over_32_lanes(float v)   // lanes 0..31 and lanes 32..63 separately
{
    v = max_over_16_lanes(v);
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float max_over_64_lanes(float v)
{
    v = max_over_32_lanes(v);
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Sum over all 64 lanes, the same butterflies with an add (every lane ends with the total).
template <int CTRL>
__device__ inline float dpp_add_step(float v)
{
    const int p = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false);
    return v + __int_as_float(p);
}
__device__ inline float sum_over_64_lanes(float v)
{
    v = dpp_add_step<0xB1>(v);
    v = dpp_add_step<0x4E>(v);
    v = dpp_add_step<0x141>(v);
    v = dpp_add_step<0x140>(v);
    const auto r16 = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(r16[0]) + __uint_as_float(r16[1]);
    const auto r32 = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r32[0]) + __uint_as_float(r32[1]);
}

// LayerNorm in front of the rotation (optional): y = (x - mean) / sqrt(var + eps) * gamma + beta over the K channels of a token.
// gamma / beta may be nullptr (1 / 0).  on == 0: no normalisation.
struct LnParams {
    const float *gamma;
    const float *beta;
    float eps;
    int on;
};

// Kernels that need more dynamic LDS than a launch gets by default.  Each source file that has such kernels lists them in a
// static LdsKernels object (filled when the library is loaded; no HIP call is made then).  prepare_device() raises the limit of
// every listed kernel on the calling thread's current device the first time it runs there (and resolves the address of the
// library's own workspace on that device); later calls are one atomic load.  Thread-safe; qvggt_init() is its public form.
struct LdsKernel {
    const void *fn;
    int lds_bytes;
};
void register_lds_kernels(const LdsKernel *list, int n);
struct LdsKernels {
    template <int N>
    explicit LdsKernels(const LdsKernel (&list)[N]) { register_lds_kernels(list, N); }
};
hipError_t prepare_device(int *device = nullptr);

__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) v = fmaxf(v, __shfl_xor(v, m));
    return v;
}

}  // namespace qvggt
