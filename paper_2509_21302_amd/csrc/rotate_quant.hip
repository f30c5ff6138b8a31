// Online kernel 1 and its offline twins: randomised Walsh-Hadamard rotation of rows,
// per-channel multiply, then either per-row quantization (activations per token, weights
// per output channel; 4-bit codes packed two per byte, or wider codes as int8) or a
// per-channel absmax (smoothing statistics).
//
// One wavefront owns one row at a time.  A row of K values lives in K/64 registers per
// lane; element e = c*(64*V) + lane*V + i sits in register c*V + i, where V = min(8, K/64)
// is the run a lane loads contiguously (16 bytes of bf16 when V = 8, so a wave reads 1 KiB
// per load instruction).  The transform is one butterfly per index bit (the Hadamard matrix
// is a Kronecker power of H_2, paper Sec. 3.2): bits inside i and c are register-to-register,
// the six lane bits go through cross-lane exchanges.
#include "qvggt_common.h"
#include "rotate_rows.h"

namespace qvggt {

enum RowMode { kQuantize = 0, kColAbsMax = 1 };

// mul_mode 0: mul[j] used as given (inv_smooth, or 1/sqrt(K) when mul == nullptr)
// mul_mode 1: 1 / (K * mul[j])   (weights: c_j / sqrt(K) recovered from inv_smooth)
// CB: bits a stored code occupies (4: two per byte; 8: one int8 each).  qmax: largest code, 2^(bits-1) - 1.
// LN: a LayerNorm of the row precedes everything else (quantize mode, K <= 4096: beyond that the row no longer fits the registers)
// ASYM: affine 4-bit codes over the row's range [min(0, min z), max(0, max z)], zero point to zero[row], nibbles hold u - 8
template <int K, bool F32, int MODE, int CB, bool LN = false, bool ASYM = false>
__global__ __launch_bounds__(256) void rotate_rows_kernel(const void *__restrict__ X, int rows,
                                                          const int8_t *__restrict__ signs,
                                                          const float *__restrict__ mul, int mul_mode,
                                                          uint8_t *__restrict__ packed,
                                                          float *__restrict__ scale,
                                                          unsigned int *__restrict__ col_absmax_bits,
                                                          const float *__restrict__ step, int step_stride, float qmax,
                                                          LnParams ln, float *__restrict__ zero = nullptr)
{
    constexpr int V = RowMap<K>::V, C = RowMap<K>::C, R = RowMap<K>::R;
    constexpr bool kPermuted = (K == 1024 || K == 2048 || K == 4096) && MODE == kQuantize;
    __shared__ __attribute__((aligned(16))) uint8_t lds_stage[kPermuted ? 4 * K : 16];
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int nwaves = gridDim.x * (blockDim.x >> 6);

    // per-lane constants: sign bits (one bit per register) and channel multipliers
    uint32_t neg[(R + 31) / 32];
#pragma unroll
    for (int w = 0; w < (R + 31) / 32; ++w) neg[w] = 0;
    float cm[R];
    const float rs = 1.0f / sqrtf((float)K);
    // loads first (all in flight together), arithmetic afterwards: the set-up is one memory round trip, not one per element
    if (signs != nullptr) {
        int8_t sb[R];
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int i = 0; i < V; ++i) sb[c * V + i] = signs[c * 64 * V + lane * V + i];
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (sb[r] < 0) neg[r >> 5] |= 1u << (r & 31);
    }
    if (mul != nullptr) {
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int i = 0; i < V; ++i) cm[c * V + i] = mul[c * 64 * V + lane * V + i];
        if (mul_mode) {
#pragma unroll
            for (int r = 0; r < R; ++r) cm[r] = 1.0f / ((float)K * cm[r]);
        }
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r) cm[r] = rs;
    }

    float colmax[MODE == kColAbsMax ? R : 1];
#pragma unroll
    for (int r = 0; r < (MODE == kColAbsMax ? R : 1); ++r) colmax[r] = 0.0f;
    for (int row = wave; row < rows; row += nwaves) {
        float x[R];
        load_row<K, F32>(X, (size_t)row, lane, x);
        if constexpr (LN) {
            // LayerNorm of the token in fp32 (two passes over the registers), result rounded to the input's type as a separate
            // normalisation kernel would hand it on; gamma and beta come through the caches, this is the general path
            float s1 = 0.0f;
#pragma unroll
            for (int r = 0; r < R; ++r) s1 += x[r];
            const float mean = sum_over_64_lanes(s1) * (1.0f / (float)K);
            float s2 = 0.0f;
#pragma unroll
            for (int r = 0; r < R; ++r) { x[r] -= mean; s2 = fmaf(x[r], x[r], s2); }
            const float rstd = 1.0f / sqrtf(sum_over_64_lanes(s2) * (1.0f / (float)K) + ln.eps);
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    const int e = c * 64 * V + lane * V + i, r = c * V + i;
                    float y = x[r] * rstd;
                    const float gm = ln.gamma ? ln.gamma[e] : 1.0f, bt = ln.beta ? ln.beta[e] : 0.0f;
                    y = fmaf(y, gm, bt);
                    if constexpr (!F32) y = bf16_bits_to_float(pack_bf16x2(y, 0.0f) & 0xFFFFu);
                    x[r] = y;
                }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
            if ((neg[r >> 5] >> (r & 31)) & 1u) x[r] = -x[r];
        fwht_row<K>(x, lane);
        float amax = 0.0f, nmin = 0.0f;       // ASYM: max(0, max z) and -min(0, min z)
#pragma unroll
        for (int r = 0; r < R; ++r) {
            x[r] *= cm[r];
            if constexpr (ASYM) { amax = fmaxf(amax, x[r]); nmin = fmaxf(nmin, -x[r]); }
            else amax = fmaxf(amax, fabsf(x[r]));
        }

        if constexpr (MODE == kColAbsMax) {
            // the wave keeps a running maximum over its rows; one atomic per column after the loop
#pragma unroll
            for (int r = 0; r < R; ++r) colmax[r] = fmaxf(colmax[r], fabsf(x[r]));
        } else {
            // dynamic: the step comes from the row's absmax; static: it is given (per token or one for the tensor)
            float inv, delta, off = 0.0f;
            if constexpr (ASYM) {
                const float hi = wave_max(amax), nlo = wave_max(nmin);
                const float range = hi + nlo;
                const bool live = range >= 15.0f * kMinStep;
                delta = live ? range / 15.0f : 0.0f;
                inv = live ? 15.0f / range : 0.0f;
                const float zp = __builtin_rintf(nlo * inv);                  // rne(-lo / step), in [0, 15]
                off = zp - 8.0f;
                if (lane == 0) zero[row] = zp;
            } else if (step != nullptr) {
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
            if constexpr (K == 1024 || K == 2048 || K == 4096) {
                // permuted layout: scatter the codes as bytes into the wave's LDS row at their positions,
                // then every lane packs K/64 consecutive positions
                uint8_t *stage = lds_stage + (threadIdx.x >> 6) * K;
#pragma unroll
                for (int c = 0; c < C; ++c)
#pragma unroll
                    for (int i = 0; i < V; ++i) {
                        int q = (int)__builtin_rintf(ASYM ? fmaf(x[c * V + i], inv, off) : x[c * V + i] * inv);
                        q = min(q_hi, max(q_lo, q));
                        stage[code_position(c * 64 * V + lane * V + i, K)] = (uint8_t)(CB == 4 ? (q & 0xF) : q);
                    }
                lanes_exchange_fence();
                constexpr int PER_LANE = K / 64;      // positions per lane, a multiple of 16
                if constexpr (CB == 8) {
#pragma unroll
                    for (int b = 0; b < PER_LANE / 16; ++b)
                        *reinterpret_cast<uint4 *>(out + lane * PER_LANE + 16 * b) = *reinterpret_cast<const uint4 *>(stage + lane * PER_LANE + 16 * b);
                } else {
#pragma unroll
                    for (int b = 0; b < PER_LANE / 8; ++b) {
                        const uint2 v = *reinterpret_cast<const uint2 *>(stage + lane * PER_LANE + 8 * b);
                        // bytes hold one code each (low nibble): squeeze 8 bytes into 8 nibbles
                        uint32_t lo = v.x, hi = v.y;
                        lo = (lo | (lo >> 4)) & 0x00FF00FFu; lo = (lo | (lo >> 8)) & 0x0000FFFFu;
                        hi = (hi | (hi >> 4)) & 0x00FF00FFu; hi = (hi | (hi >> 8)) & 0x0000FFFFu;
                        *reinterpret_cast<uint32_t *>(out + lane * (PER_LANE / 2) + 4 * b) = lo | (hi << 16);
                    }
                }
                lanes_exchange_fence();
            } else {
#pragma unroll
            for (int c = 0; c < C; ++c) {
                uint64_t word = 0;
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    int q = (int)__builtin_rintf(ASYM ? fmaf(x[c * V + i], inv, off) : x[c * V + i] * inv);
                    q = min(q_hi, max(q_lo, q));
                    word |= (uint64_t)(q & ((1 << CB) - 1)) << (CB * i);
                }
                // natural order: element e -> code slot e; a lane's V codes are V * CB / 8 consecutive bytes
                const int byte0 = (c * 64 * V + lane * V) * CB / 8;
                if constexpr (V * CB == 64) *reinterpret_cast<uint2 *>(out + byte0) = make_uint2((uint32_t)word, (uint32_t)(word >> 32));
                else if constexpr (V * CB == 32) *reinterpret_cast<uint32_t *>(out + byte0) = (uint32_t)word;
                else if constexpr (V * CB == 16) *reinterpret_cast<uint16_t *>(out + byte0) = (uint16_t)word;
                else out[byte0] = (uint8_t)word;
            }
            }
        }
    }
    if constexpr (MODE == kColAbsMax) {
        if (wave < rows) {
            // non-negative floats order like their bit patterns
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int i = 0; i < V; ++i)
                    atomicMax(&col_absmax_bits[c * 64 * V + lane * V + i], __float_as_uint(colmax[c * V + i]));
        }
    }
}

// ---------------------------------------------------------------------------------------
// small helpers of the offline path

__global__ void fill_u32_kernel(unsigned int *p, int n, unsigned int v)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// in place: buf[j] holds w_j = max_o |W H|[o, j] on entry, inv_smooth[j] = 1 / (sqrt(K) c_j) on exit
__global__ void smooth_factor_kernel(float *buf, const float *__restrict__ act_absmax, int K, float alpha)
{
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= K) return;
    const float floor_ = 1e-5f;
    float a = fmaxf(act_absmax[j], floor_), w = fmaxf(buf[j], floor_);
    float c = powf(a, alpha) / powf(w, 1.0f - alpha);
    buf[j] = 1.0f / (sqrtf((float)K) * c);
}

// a given smoothing factor c[j] -> inv_smooth[j] = 1 / (sqrt(K) c_j)
__global__ void inv_from_factor_kernel(float *buf, const float *__restrict__ c, int K)
{
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < K) buf[j] = 1.0f / (sqrtf((float)K) * c[j]);
}

__global__ void fill_f32_kernel(float *p, int n, float v)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// int8 codes in natural order <-> packed rows in the library layout
__global__ void pack_int4_kernel(const int8_t *__restrict__ codes, size_t rows, int K, uint8_t *__restrict__ packed)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // one output byte each
    if (idx >= rows * (size_t)(K / 2)) return;
    size_t row = idx / (K / 2);
    int byte = (int)(idx % (K / 2));
    int e0 = code_element(2 * byte, K), e1 = code_element(2 * byte + 1, K);
    uint8_t lo = (uint8_t)codes[row * K + e0] & 0xF, hi = (uint8_t)codes[row * K + e1] & 0xF;
    packed[idx] = lo | (hi << 4);
}

__global__ void unpack_int4_kernel(const uint8_t *__restrict__ packed, size_t rows, int K, int8_t *__restrict__ codes)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // one natural element each
    if (idx >= rows * (size_t)K) return;
    size_t row = idx / K;
    int e = (int)(idx % K);
    int p = code_position(e, K);
    uint8_t b = packed[row * (K / 2) + p / 2];
    int nib = (p & 1) ? (b >> 4) : (b & 0xF);
    codes[idx] = (int8_t)(nib >= 8 ? nib - 16 : nib);
}

// int8 codes: natural order <-> the library's position order (the same map as for packed rows, one byte per position)
// sums[o] = sum_j code[o, j] over a row of packed 4-bit codes (any position order): one wave per row
__global__ __launch_bounds__(256) void code_sums_kernel(const uint8_t *__restrict__ packed, int rows, int K, float *__restrict__ sums)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const uint32_t *p = reinterpret_cast<const uint32_t *>(packed + (size_t)row * (K / 2));
    int s = 0;
    for (int i = lane; i < K / 8; i += 64) {
        const uint32_t v = p[i];
#pragma unroll
        for (int n = 0; n < 8; ++n) s += (int)(v << (28 - 4 * n)) >> 28;      // sign-extended nibble n
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) s += __shfl_xor(s, m);
    if (lane == 0) sums[row] = (float)s;                                        // |s| <= 8 K: exact
}

__global__ void layout_int8_kernel(const int8_t *__restrict__ src, size_t rows, int K, int8_t *__restrict__ dst, int to_library)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // one output byte each
    if (idx >= rows * (size_t)K) return;
    size_t row = idx / K;
    int o = (int)(idx % K);
    dst[idx] = src[row * K + (to_library ? code_element(o, K) : code_position(o, K))];
}

// ---------------------------------------------------------------------------------------
// host-side launchers (called from api.hip)

// sizes 2^n * m (m = 12, 20, 28): rotate_quant_general.hip
bool general_size_supported(int K);
hipError_t run_rotate_rows_general(const void *X, bool f32, int rows, int K, const int8_t *signs, const float *mul, int mul_mode,
                                   uint8_t *packed, float *scale, unsigned int *colmax, const float *step, int step_stride,
                                   int bits, hipStream_t stream);

template <int MODE, int CB>
static hipError_t launch_rotate_rows(const void *X, bool f32, int rows, int K, const int8_t *signs,
                                     const float *mul, int mul_mode, uint8_t *packed, float *scale,
                                     unsigned int *colmax, const float *step, int step_stride, float qmax, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    const int waves_per_block = 4;
    int blocks = (rows + waves_per_block - 1) / waves_per_block;
    // up to eight blocks per compute unit; the column statistic takes fewer waves for small inputs so that each folds several
    // rows into its running maximum before touching the shared result
    const int max_blocks = (MODE == kColAbsMax) ? 256 * 2 : 256 * 8;
    if (MODE == kColAbsMax) blocks = (rows + 31) / 32;     // eight rows or more per wave: the atomics at the end are what costs
    if (blocks > max_blocks) blocks = max_blocks;
    if (blocks < 1) blocks = 1;
#define QVGGT_LAUNCH(KK)                                                                                     \
    case KK:                                                                                                 \
        if (f32) rotate_rows_kernel<KK, true, MODE, CB><<<blocks, 256, 0, stream>>>(X, rows, signs, mul, mul_mode, packed, scale, colmax, step, step_stride, qmax, LnParams{nullptr, nullptr, 0.0f, 0}); \
        else rotate_rows_kernel<KK, false, MODE, CB><<<blocks, 256, 0, stream>>>(X, rows, signs, mul, mul_mode, packed, scale, colmax, step, step_stride, qmax, LnParams{nullptr, nullptr, 0.0f, 0});    \
        break;
    switch (K) {
        QVGGT_LAUNCH(128)
        QVGGT_LAUNCH(256)
        QVGGT_LAUNCH(512)
        QVGGT_LAUNCH(1024)
        QVGGT_LAUNCH(2048)
        QVGGT_LAUNCH(4096)
        QVGGT_LAUNCH(8192)
        default: return hipErrorInvalidValue;
    }
#undef QVGGT_LAUNCH
    return hipGetLastError();
}

hipError_t run_rotate_quant_mfma(const void *X, int rows, int K, const int8_t *signs, const float *mul, int mul_mode,
                                 uint8_t *packed, float *scale, const float *step, int step_stride, int bits,
                                 hipStream_t stream);
hipError_t run_rotated_col_absmax_mfma(const void *X, int rows, int K, const int8_t *signs, unsigned int *absmax_bits,
                                       hipStream_t stream);

// bits: 4 (packed nibbles) or 5..8 (int8 codes in [-2^(bits-1), 2^(bits-1) - 1])
hipError_t run_rotate_smooth_quant(const void *X, bool f32, int rows, int K, const int8_t *signs,
                                   const float *mul, int mul_mode, uint8_t *packed, float *scale,
                                   const float *step, int step_stride, int bits, hipStream_t stream)
{
    if (general_size_supported(K))
        return run_rotate_rows_general(X, f32, rows, K, signs, mul, mul_mode, packed, scale, nullptr, step, step_stride, bits, stream);
    const float qmax = (float)((1 << (code_width(bits) - 1)) - 1);
    // bf16 rows of the sizes VGGT-1B uses go to the matrix-core kernel; everything else to the generic one
    if (!f32 && (K == 1024 || K == 2048 || K == 4096))
        return run_rotate_quant_mfma(X, rows, K, signs, mul, mul_mode, packed, scale, step, step_stride, bits, stream);
    if (bits == 4)
        return launch_rotate_rows<kQuantize, 4>(X, f32, rows, K, signs, mul, mul_mode, packed, scale, nullptr, step, step_stride, qmax, stream);
    return launch_rotate_rows<kQuantize, 8>(X, f32, rows, K, signs, mul, mul_mode, packed, scale, nullptr, step, step_stride, qmax, stream);
}

hipError_t run_ln_rotate_quant_mfma(const void *X, int rows, const int8_t *signs, const float *mul, uint8_t *packed, float *scale,
                                    LnParams ln, hipStream_t stream);

// LayerNorm + rotation + smoothing + per-token 4-bit quantization in one kernel (power-of-two K)
hipError_t run_ln_rotate_smooth_quant(const void *X, bool f32, int rows, int K, LnParams ln, const int8_t *signs, const float *mul,
                                      uint8_t *packed, float *scale, hipStream_t stream)
{
    if (!f32 && K == 1024) return run_ln_rotate_quant_mfma(X, rows, signs, mul, packed, scale, ln, stream);
    if (rows <= 0) return hipSuccess;
    int blocks = (rows + 3) / 4;
    if (blocks > 256 * 8) blocks = 256 * 8;
#define QVGGT_LAUNCH_LN(KK)                                                                                                            \
    case KK:                                                                                                                           \
        if (f32) rotate_rows_kernel<KK, true, kQuantize, 4, true><<<blocks, 256, 0, stream>>>(X, rows, signs, mul, 0, packed, scale, nullptr, nullptr, 0, 7.0f, ln); \
        else rotate_rows_kernel<KK, false, kQuantize, 4, true><<<blocks, 256, 0, stream>>>(X, rows, signs, mul, 0, packed, scale, nullptr, nullptr, 0, 7.0f, ln);    \
        break;
    switch (K) {
        QVGGT_LAUNCH_LN(128)
        QVGGT_LAUNCH_LN(256)
        QVGGT_LAUNCH_LN(512)
        QVGGT_LAUNCH_LN(1024)
        QVGGT_LAUNCH_LN(2048)
        QVGGT_LAUNCH_LN(4096)
        default: return hipErrorInvalidValue;
    }
#undef QVGGT_LAUNCH_LN
    return hipGetLastError();
}

hipError_t run_rotate_quant_asym_mfma(const void *X, int rows, int K, const int8_t *signs, const float *mul, uint8_t *packed,
                                      float *scale, float *zero, hipStream_t stream);

// rotation + smoothing + per-token affine 4-bit codes with zero points (power-of-two K)
hipError_t run_rotate_smooth_quant_asym(const void *X, bool f32, int rows, int K, const int8_t *signs, const float *mul,
                                        uint8_t *packed, float *scale, float *zero, hipStream_t stream)
{
    if (!f32 && (K == 1024 || K == 2048 || K == 4096))
        return run_rotate_quant_asym_mfma(X, rows, K, signs, mul, packed, scale, zero, stream);
    if (rows <= 0) return hipSuccess;
    int blocks = (rows + 3) / 4;
    if (blocks > 256 * 8) blocks = 256 * 8;
    const LnParams no_ln{nullptr, nullptr, 0.0f, 0};
#define QVGGT_LAUNCH_ASYM(KK)                                                                                                          \
    case KK:                                                                                                                           \
        if (f32) rotate_rows_kernel<KK, true, kQuantize, 4, false, true><<<blocks, 256, 0, stream>>>(X, rows, signs, mul, 0, packed, scale, nullptr, nullptr, 0, 7.0f, no_ln, zero); \
        else rotate_rows_kernel<KK, false, kQuantize, 4, false, true><<<blocks, 256, 0, stream>>>(X, rows, signs, mul, 0, packed, scale, nullptr, nullptr, 0, 7.0f, no_ln, zero);    \
        break;
    switch (K) {
        QVGGT_LAUNCH_ASYM(128)
        QVGGT_LAUNCH_ASYM(256)
        QVGGT_LAUNCH_ASYM(512)
        QVGGT_LAUNCH_ASYM(1024)
        QVGGT_LAUNCH_ASYM(2048)
        QVGGT_LAUNCH_ASYM(4096)
        QVGGT_LAUNCH_ASYM(8192)
        default: return hipErrorInvalidValue;
    }
#undef QVGGT_LAUNCH_ASYM
    return hipGetLastError();
}

hipError_t run_rotated_col_absmax(const void *X, bool f32, int rows, int K, const int8_t *signs,
                                  float *absmax, hipStream_t stream)
{
    fill_u32_kernel<<<(K + 255) / 256, 256, 0, stream>>>(reinterpret_cast<unsigned int *>(absmax), K, 0u);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (!f32 && (K == 1024 || K == 2048 || K == 4096))
        return run_rotated_col_absmax_mfma(X, rows, K, signs, reinterpret_cast<unsigned int *>(absmax), stream);
    if (general_size_supported(K))
        return run_rotate_rows_general(X, f32, rows, K, signs, nullptr, 0, nullptr, nullptr, reinterpret_cast<unsigned int *>(absmax),
                                       nullptr, 0, 4, stream);
    return launch_rotate_rows<kColAbsMax, 4>(X, f32, rows, K, signs, nullptr, 0, nullptr, nullptr,
                                             reinterpret_cast<unsigned int *>(absmax), nullptr, 0, 7.0f, stream);
}

hipError_t run_smooth_factor(float *buf, const float *act_absmax, int K, float alpha, hipStream_t stream)
{
    smooth_factor_kernel<<<(K + 255) / 256, 256, 0, stream>>>(buf, act_absmax, K, alpha);
    return hipGetLastError();
}

hipError_t run_inv_from_factor(float *buf, const float *c, int K, hipStream_t stream)
{
    inv_from_factor_kernel<<<(K + 255) / 256, 256, 0, stream>>>(buf, c, K);
    return hipGetLastError();
}

hipError_t run_fill_f32(float *p, int n, float v, hipStream_t stream)
{
    fill_f32_kernel<<<(n + 255) / 256, 256, 0, stream>>>(p, n, v);
    return hipGetLastError();
}

hipError_t run_pack_int4(const int8_t *codes, int rows, int K, uint8_t *packed, hipStream_t stream)
{
    size_t n = (size_t)rows * (K / 2);
    if (n == 0) return hipSuccess;
    pack_int4_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(codes, (size_t)rows, K, packed);
    return hipGetLastError();
}

hipError_t run_layout_int8(const int8_t *src, int rows, int K, int8_t *dst, int to_library, hipStream_t stream)
{
    size_t n = (size_t)rows * K;
    if (n == 0) return hipSuccess;
    layout_int8_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(src, (size_t)rows, K, dst, to_library);
    return hipGetLastError();
}

// int8 rows in library order [rows, K] -> int8 blocks (K-tiles of 64 bytes outermost inside 128-row blocks, chunks swizzled)
__global__ __launch_bounds__(256) void int8_to_blocks_kernel(const int8_t *__restrict__ src, size_t rows, int K, uint8_t *__restrict__ dst)
{
    const size_t chunks_per_row = (size_t)K / 16;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * chunks_per_row) return;
    const size_t row = idx / chunks_per_row;
    const int ch = (int)(idx - row * chunks_per_row), kt = ch >> 2, slot = (ch & 3) ^ (int)((row & 15) >> 2);
    const uint4 v = *reinterpret_cast<const uint4 *>(src + row * (size_t)K + (size_t)ch * 16);
    *reinterpret_cast<uint4 *>(dst + ((row / 128) * (size_t)(K / 64) + kt) * 8192 + (row % 128) * 64 + slot * 16) = v;
}

hipError_t run_int8_to_blocks(const int8_t *src, int rows, int K, uint8_t *dst, hipStream_t stream)
{
    const size_t n = (size_t)rows * (K / 16);
    if (n == 0) return hipSuccess;
    int8_to_blocks_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(src, (size_t)rows, K, dst);
    return hipGetLastError();
}

hipError_t run_code_sums(const uint8_t *packed, int rows, int K, float *sums, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    code_sums_kernel<<<(rows + 3) / 4, 256, 0, stream>>>(packed, rows, K, sums);
    return hipGetLastError();
}

hipError_t run_unpack_int4(const uint8_t *packed, int rows, int K, int8_t *codes, hipStream_t stream)
{
    size_t n = (size_t)rows * K;
    if (n == 0) return hipSuccess;
    unpack_int4_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(packed, (size_t)rows, K, codes);
    return hipGetLastError();
}

}  // namespace qvggt
