// Online kernel 1 and its offline twins for input sizes that are not powers of two: K = 2^n * m with m = 12, 20 or 28
// (paper Sec. 3.2: H_K = H_{2^n} (x) H_m).  H_m is Paley's Hadamard matrix (type I from GF(11) and GF(19), type II from
// GF(13)); its entries are computed at compile time from the quadratic residues, so the m-point stage is straight-line
// adds and subtracts.  Element e = a * m + b (a < 2^n, b < m); a wavefront owns a row, lane l holds the m values of every
// a = l + 64 * c: the m-point transform is inside a lane, the six low bits of a go through cross-lane exchanges, the
// remaining bits are register-to-register butterflies.  Codes are written in natural order (element e -> position e).
// This is the general path: dense m x m stages cost m vector ALU ops per element, it is not tuned like the power-of-two
// kernels and VGGT-1B itself has no layer that needs it.
#include "qvggt_common.h"

#include <algorithm>
#include <type_traits>
#include <utility>

namespace qvggt {

namespace gen {

// ---- Paley's matrices, entry (r, c) in {+1, -1}, from the squares of GF(q) found by enumeration
template <int Q>
constexpr bool is_square_mod(int x)
{
    x %= Q;
    if (x < 0) x += Q;
    for (int k = 1; k < Q; ++k)
        if ((k * k) % Q == x) return true;
    return false;
}

template <int MM>
constexpr int paley_entry(int r, int c)
{
    static_assert(MM == 12 || MM == 20 || MM == 28, "Paley matrices of order 12, 20 and 28");
    if constexpr (MM == 28) {
        // type II, q = 13: symmetric conference matrix of order 14 blown up by 2 x 2 blocks
        const int i = r / 2, j = c / 2, u = r % 2, v = c % 2;
        if (i == j) return (u == 0 && v == 0) ? 1 : -1;                       // the zero diagonal becomes [[1, -1], [-1, -1]]
        const int cc = (i == 0 || j == 0) ? 1 : (is_square_mod<13>(i - j) ? 1 : -1);
        return (u == 1 && v == 1) ? -cc : cc;                                 // +-1 becomes +-[[1, 1], [1, -1]]
    } else {
        // type I, q = MM - 1: identity plus the skew matrix bordered by +1 (first row) and -1 (first column)
        if (r == c) return 1;
        if (r == 0) return 1;
        if (c == 0) return -1;
        return is_square_mod<MM - 1>(r - c) ? 1 : -1;
    }
}

template <class F, int... Is>
__device__ inline void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ inline void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

enum Mode { kQuantize = 0, kColAbsMax = 1 };

}  // namespace gen

// mul_mode 0: mul[j] used as given (inv_smooth, or 1/sqrt(K) when mul == nullptr); 1: 1 / (K * mul[j]) (weights)
// CB: bits a stored code occupies (4 or 8); qmax: largest code; step: static quantization step or nullptr
template <int N2, int MM, bool F32, int MODE, int CB>
__global__ __launch_bounds__(256) void rotate_rows_general_kernel(const void *__restrict__ X, int rows,
                                                                  const int8_t *__restrict__ signs,
                                                                  const float *__restrict__ mul, int mul_mode,
                                                                  uint8_t *__restrict__ packed, float *__restrict__ scale,
                                                                  unsigned int *__restrict__ col_absmax_bits,
                                                                  const float *__restrict__ step, int step_stride, float qmax)
{
    constexpr int K = N2 * MM, C = N2 / 64, R = C * MM;
    static_assert(N2 >= 64 && (N2 & (N2 - 1)) == 0, "the power-of-two factor covers the 64 lanes");
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int nwaves = gridDim.x * (blockDim.x >> 6);

    // per-lane constants: register r = c * MM + b holds element e = (lane + 64 c) * MM + b
    float cm[R];
    uint32_t neg[(R + 31) / 32];         // one sign bit per register
#pragma unroll
    for (int w = 0; w < (R + 31) / 32; ++w) neg[w] = 0;
    const float rs = 1.0f / sqrtf((float)K);
    // loads first (all in flight together), arithmetic afterwards
    if (signs != nullptr) {
        int8_t sb[R];
#pragma unroll
        for (int r = 0; r < R; ++r) sb[r] = signs[(lane + 64 * (r / MM)) * MM + (r % MM)];
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (sb[r] < 0) neg[r >> 5] |= 1u << (r & 31);
    }
    if (mul != nullptr) {
#pragma unroll
        for (int r = 0; r < R; ++r) cm[r] = mul[(lane + 64 * (r / MM)) * MM + (r % MM)];
        if (mul_mode) {
#pragma unroll
            for (int r = 0; r < R; ++r) cm[r] = 1.0f / ((float)K * cm[r]);
        }
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r) cm[r] = rs;
    }

    float colmax[MODE == gen::kColAbsMax ? R : 1];
#pragma unroll
    for (int r = 0; r < (MODE == gen::kColAbsMax ? R : 1); ++r) colmax[r] = 0.0f;
    for (int row = wave; row < rows; row += nwaves) {
        float x[R];
        // a lane's MM values of one a are contiguous: 8-byte (bf16) or 16-byte (f32) pieces of four values
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const size_t e0 = (size_t)row * K + (size_t)(lane + 64 * c) * MM;
#pragma unroll
            for (int q = 0; q < MM / 4; ++q) {
                if constexpr (F32) {
                    const float4 v = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(X) + e0 + 4 * q);
                    x[c * MM + 4 * q] = v.x; x[c * MM + 4 * q + 1] = v.y; x[c * MM + 4 * q + 2] = v.z; x[c * MM + 4 * q + 3] = v.w;
                } else {
                    const uint2 v = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(X) + e0 + 4 * q);
                    x[c * MM + 4 * q] = __uint_as_float(v.x << 16); x[c * MM + 4 * q + 1] = __uint_as_float(v.x & 0xFFFF0000u);
                    x[c * MM + 4 * q + 2] = __uint_as_float(v.y << 16); x[c * MM + 4 * q + 3] = __uint_as_float(v.y & 0xFFFF0000u);
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
            if ((neg[r >> 5] >> (r & 31)) & 1u) x[r] = -x[r];

        // H_m inside every group of MM registers: y[b'] = sum_b x[b] H[b][b'], signs known at compile time
#pragma unroll
        for (int c = 0; c < C; ++c) {
            float y[MM];
            gen::static_for<MM>([&](auto bp_c) {
                constexpr int bp = decltype(bp_c)::value;
                float acc = 0.0f;
                gen::static_for<MM>([&](auto b_c) {
                    constexpr int b = decltype(b_c)::value;
                    if constexpr (gen::paley_entry<MM>(b, bp) > 0) acc += x[c * MM + b];
                    else acc -= x[c * MM + b];
                });
                y[bp] = acc;
            });
#pragma unroll
            for (int b = 0; b < MM; ++b) x[c * MM + b] = y[b];
        }
        // H_{2^n} over a = lane + 64 c: the six lane bits, then the bits of c
#pragma unroll
        for (int m = 1; m < kWave; m <<= 1) {
            const bool upper = (lane & m) != 0;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float p = __shfl_xor(x[r], m);
                x[r] = upper ? p - x[r] : x[r] + p;
            }
        }
#pragma unroll
        for (int h = 1; h < C; h <<= 1)
#pragma unroll
            for (int c = 0; c < C; ++c)
                if ((c & h) == 0) {
#pragma unroll
                    for (int b = 0; b < MM; ++b) {
                        const float a = x[c * MM + b], d = x[(c + h) * MM + b];
                        x[c * MM + b] = a + d;
                        x[(c + h) * MM + b] = a - d;
                    }
                }

        float amax = 0.0f;
#pragma unroll
        for (int r = 0; r < R; ++r) { x[r] *= cm[r]; amax = fmaxf(amax, fabsf(x[r])); }

        if constexpr (MODE == gen::kColAbsMax) {
            // the wave keeps a running maximum over its rows; one atomic per column after the loop
#pragma unroll
            for (int r = 0; r < R; ++r) colmax[r] = fmaxf(colmax[r], fabsf(x[r]));
        } else {
            float inv, delta;
            if (step != nullptr) {
                delta = step[(size_t)row * step_stride];
                inv = delta >= kMinStep ? 1.0f / delta : 0.0f;
            } else {
                amax = wave_max(amax);
                const bool live = amax >= qmax * kMinStep;
                delta = live ? amax / qmax : 0.0f;
                inv = live ? qmax / amax : 0.0f;
            }
            if (lane == 0) scale[row] = delta;
            const int q_hi = (int)qmax, q_lo = -q_hi - 1;
            uint8_t *out = packed + (size_t)row * (K * CB / 8);
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int g = 0; g < MM / 4; ++g) {
                    uint32_t word = 0;          // four codes: two bytes of nibbles, or four bytes
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        int qv = (int)__builtin_rintf(x[c * MM + 4 * g + i] * inv);
                        qv = min(q_hi, max(q_lo, qv));
                        word |= (uint32_t)(qv & ((1 << CB) - 1)) << (CB * i);
                    }
                    const size_t pos = (size_t)(lane + 64 * c) * MM + 4 * g;      // position of the first of the four codes
                    if constexpr (CB == 4) *reinterpret_cast<uint16_t *>(out + pos / 2) = (uint16_t)word;
                    else *reinterpret_cast<uint32_t *>(out + pos) = word;
                }
        }
    }
    if constexpr (MODE == gen::kColAbsMax) {
        if (wave < rows) {
            // non-negative floats order like their bit patterns
#pragma unroll
            for (int r = 0; r < R; ++r)
                atomicMax(&col_absmax_bits[(lane + 64 * (r / MM)) * MM + (r % MM)], __float_as_uint(colmax[r]));
        }
    }
}


// K = N2 * MM for the sizes this file instantiates
bool general_size_supported(int K)
{
    switch (K) {
        case 768: case 1536: case 3072: case 6144: case 1280: case 2560: case 5120: case 1792: case 3584: return true;
        default: return false;
    }
}

template <int N2, int MM>
static hipError_t launch_general(const void *X, bool f32, int rows, const int8_t *signs, const float *mul, int mul_mode,
                                 uint8_t *packed, float *scale, unsigned int *colmax, const float *step, int step_stride,
                                 int bits, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    int blocks = (rows + 3) / 4;
    if (blocks > 256 * 8) blocks = 256 * 8;
    if (colmax != nullptr) blocks = std::max(1, std::min((rows + 31) / 32, 256 * 2));   // eight rows or more per wave for the statistic
    const float qmax = (float)((1 << (code_width(bits) - 1)) - 1);
#define QVGGT_GEN(F32_, MODE_, CB_) \
    rotate_rows_general_kernel<N2, MM, F32_, MODE_, CB_><<<blocks, 256, 0, stream>>>(X, rows, signs, mul, mul_mode, packed, scale, colmax, step, step_stride, qmax)
    if (colmax != nullptr) {
        if (f32) QVGGT_GEN(true, gen::kColAbsMax, 4); else QVGGT_GEN(false, gen::kColAbsMax, 4);
    } else if (bits == 4) {
        if (f32) QVGGT_GEN(true, gen::kQuantize, 4); else QVGGT_GEN(false, gen::kQuantize, 4);
    } else {
        if (f32) QVGGT_GEN(true, gen::kQuantize, 8); else QVGGT_GEN(false, gen::kQuantize, 8);
    }
#undef QVGGT_GEN
    return hipGetLastError();
}

// colmax != nullptr: column absmax statistic (packed, scale unused); otherwise quantize with `bits`
hipError_t run_rotate_rows_general(const void *X, bool f32, int rows, int K, const int8_t *signs, const float *mul, int mul_mode,
                                   uint8_t *packed, float *scale, unsigned int *colmax, const float *step, int step_stride,
                                   int bits, hipStream_t stream)
{
#define QVGGT_CASE(KK, N2, MM) \
    case KK: return launch_general<N2, MM>(X, f32, rows, signs, mul, mul_mode, packed, scale, colmax, step, step_stride, bits, stream);
    switch (K) {
        QVGGT_CASE(768, 64, 12)
        QVGGT_CASE(1536, 128, 12)
        QVGGT_CASE(3072, 256, 12)
        QVGGT_CASE(6144, 512, 12)
        QVGGT_CASE(1280, 64, 20)
        QVGGT_CASE(2560, 128, 20)
        QVGGT_CASE(5120, 256, 20)
        QVGGT_CASE(1792, 64, 28)
        QVGGT_CASE(3584, 128, 28)
        default: return hipErrorInvalidValue;
    }
#undef QVGGT_CASE
}

}  // namespace qvggt
