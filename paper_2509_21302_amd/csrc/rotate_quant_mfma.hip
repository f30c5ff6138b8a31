// Online kernel 1, matrix-core version for bf16 rows of K = 1024, 2048 or 4096 values.
//
// The Hadamard matrix is a Kronecker power (paper Sec. 3.2): H_K = H_{K/128} (x) H_128.  With a
// row viewed as a (K/128) x 128 matrix R ("hi-block" hb, low index n), the transform is
// H_{K/128} . R . H_128.  The right factor is taken on the matrix cores: the bf16 inputs and the
// +-1 entries are exact operands and the sums accumulate in fp32, so R . H_128 has fp32-butterfly
// accuracy at 1/16 of a vector-ALU op per element.  The left factor (3 to 5 butterfly stages over
// hb) is done by the vector ALU on the accumulator registers.  Everything after that (multiply by
// inv_smooth, per-token absmax, round, pack) stays in the same registers.
//
// One wavefront handles a tile of 32 segments of 128 values (= 32 MFMA rows): 4 tokens for K = 1024,
// 2 for 2048, 1 for 4096.  Per tile: coalesced 16-byte global loads -> sign flip on the packed bf16 ->
// wave-private LDS rows (pitch 272 B, conflict-free 16-byte fragment reads) -> 32 MFMA 32x32x16 bf16
// (8 K-steps x 4 column tiles) -> butterflies over hb -> scale, absmax, quantize -> 16/32-byte stores.
// The next tile's global loads are issued before the current tile is processed.
//
// MFMA row m of a tile holds segment (token tk, hi-block hb); the bits of hb go to m bits 0, 1, 3, 4, 2
// (in that order) and the token bits fill the rest.  In the 32x32 result layout a lane owns column
// c = lane % 32 and rows 8*(r/4) + 4*(lane/32) + r%4 for its 16 registers r, so m bits 0, 1, 3, 4 are
// register-index bits (butterflies between registers) and m bit 2 is the lane half.
//
// Packed layout written (the same bijection is applied to weight rows, and qvggt_pack_int4 /
// qvggt_unpack_int4 implement it): element e = 128*hb + 32*nt + c goes to position
//   c * (K/32) + nt + 4*hb'      (hb' = hb, except for K = 4096 where bits 3 and 4 of hb are swapped)
// so that a lane's codes of one token are contiguous.
#include "qvggt_common.h"

#include <algorithm>
#include <cstdlib>

namespace qvggt {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

namespace rq {
constexpr int LDS_PITCH = 272;                 // bytes per 128-value bf16 segment row (256 + 16 pad)
constexpr int LDS_PER_WAVE = 32 * LDS_PITCH;   // 8704
constexpr int WAVES_PER_BLOCK = 4;
constexpr float MAGIC = 12582912.0f + 8.0f;    // 1.5 * 2^23 + 8: adding it leaves (code + 8) in the low mantissa bits
constexpr float MAGIC8 = 12582912.0f + 128.0f; // the same for int8 codes: (code + 128) in the low byte

template <int K>
struct Cfg {
    static constexpr int HB = K / 128;                       // hi-blocks per token
    static constexpr int REM = (K == 1024) ? 3 : (K == 2048) ? 4 : 5;
    static constexpr int TOK = 32 / HB;                      // tokens per tile
    static constexpr int TOK_PER_LANE = (REM == 3) ? 2 : 1;  // tokens a lane sees in its registers
    static constexpr int HB_PER_LANE = (REM == 3) ? 8 : 16;  // hi-blocks per lane and token
    static constexpr int NL = 4 * HB_PER_LANE;               // codes per lane and token
    static constexpr int SIGN_CLASSES = K / 512;             // distinct column chunks a lane loads
};

// GELU(x) = x Phi(x) of a bf16 value, as a bf16 value, by table.  A bf16 input has 65536 possible values, and the exact activation
// rounded to bf16 (what a separate activation kernel would hand on, and what the float64 reference computes) is a function of
// those 16 bits alone: the kernel looks it up instead of evaluating erfc per element.  The table (qvggt_gelu_table, built on
// the device in double precision) covers 2^-20 <= |x| < 2^12, 4096 magnitudes per sign: with d = (bits - 0x3580) mod 2^16 an
// input is covered iff (d & 0x7FFF) < 0x1000, and its entry is (d & 0x0FFF) | ((d >> 3) & 0x1000).  Outside: |x| < 2^-20
// gives x / 2 (the correction 0.4 x^2 is below a quarter ulp there), x >= 2^12 gives x, x <= -2^12 gives -0.
constexpr uint32_t GELU_U0 = 0x3580u;            // bf16 bits of 2^-20
constexpr int GELU_TABLE_ENTRIES = 8192;
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

__device__ inline uint32_t gelu_window(uint32_t w)      // both halves of a packed pair: bits - U0
{
    const us2 a = *reinterpret_cast<const us2 *>(&w), u0 = {(unsigned short)GELU_U0, (unsigned short)GELU_U0};
    const us2 d = a - u0;
    return *reinterpret_cast<const uint32_t *>(&d);
}
// both halves covered by the table (the usual case): two lookups.  Inside the window bits 12..14 of a half are zero, so twice the
// entry number, the byte offset into the table, is (low 12 bits) << 1 | (bit 15) >> 2, formed for both halves at once (what the
// shifts carry across the middle is masked out)
__device__ inline uint32_t gelu_pair_table(uint32_t d, const uint16_t *lut)
{
    const uint32_t off = ((d << 1) & 0x1FFE1FFEu) | ((d >> 2) & 0x20002000u);
    const uint8_t *t = reinterpret_cast<const uint8_t *>(lut);
    return (uint32_t) * reinterpret_cast<const uint16_t *>(t + (off & 0xFFFFu)) | ((uint32_t) * reinterpret_cast<const uint16_t *>(t + (off >> 16)) << 16);
}
// any finite value
__device__ inline uint32_t gelu_one_any(uint32_t bits, const uint16_t *lut)
{
    const uint32_t d = (bits - GELU_U0) & 0xFFFFu;
    if ((d & 0x7FFFu) < 0x1000u) return lut[(d & 0x0FFFu) | ((d >> 3) & 0x1000u)];
    if ((bits & 0x7FFFu) < GELU_U0) {                                   // tiny: x / 2, rounded as a bf16 store would (subnormals included)
        const uint32_t p = pack_bf16x2(0.5f * __uint_as_float(bits << 16), 0.0f);
        return p & 0xFFFFu;
    }
    return (bits & 0x8000u) ? 0x8000u : bits;                             // |x| >= 2^12: x or -0
}

// MFMA row of segment `seg` (= tk * HB + hb) of a tile, without the two lowest hb bits
// (those are m bits 0 and 1 and come from the lane at run time).
template <int K>
__host__ __device__ constexpr int row_of_seg_hi(int seg_hi /* seg >> 2 */)
{
    constexpr int REM = Cfg<K>::REM;
    // seg_hi bits: hb2.. then token bits.  hb2 -> m3, hb3 -> m4, hb4 -> m2; token bits fill what is left, ascending.
    int m = 0;
    if (REM == 3) {            // seg_hi = hb2 | tk0 << 1 | tk1 << 2
        m |= (seg_hi & 1) << 3; m |= ((seg_hi >> 1) & 1) << 2; m |= ((seg_hi >> 2) & 1) << 4;
    } else if (REM == 4) {     // seg_hi = hb2 | hb3 << 1 | tk0 << 2
        m |= (seg_hi & 1) << 3; m |= ((seg_hi >> 1) & 1) << 4; m |= ((seg_hi >> 2) & 1) << 2;
    } else {                   // seg_hi = hb2 | hb3 << 1 | hb4 << 2
        m |= (seg_hi & 1) << 3; m |= ((seg_hi >> 1) & 1) << 4; m |= ((seg_hi >> 2) & 1) << 2;
    }
    return m;
}
}  // namespace rq

// CB: bits a stored code occupies: 4 (packed nibbles, codes in [-8, 7]) or 8 (int8, codes in [-qmax - 1, qmax]);
// CB = 6: 4-bit codes written as E2M3 numbers in the 128-row blocks the 6-bit matrix path reads (dynamic steps only: codes in [-7, 7]);
// CB = 0 is the statistic mode: nothing is quantized or stored, the kernel leaves max_t |X H / sqrt(K)|[t, j] per column j
// in col_absmax_bits (the numerator of the smoothing factor, Sec. 3.2), which must be zero on entry
// LN: a LayerNorm of every token (fp32, result rounded to bf16 as a separate normalisation kernel would hand it on) is
// applied to the loaded values before anything else
// ASYM: affine codes.  The row's range [min(0, min z), max(0, max z)] takes the 16 codes, the zero point goes to zero[row], and
// the nibbles hold u - 8 (u the unsigned code), i.e. the signed values the integer GEMM multiplies
// BLK8 (CB = 8): the int8 codes go out as "int8 blocks", the operand format of the blocked int8 GEMM: K-tile kt (64 codes) of row r at
// ((r / 128) * (K / 64) + kt) * 8192 + (r % 128) * 64, its 16-byte chunk ch in slot ch ^ ((r % 16) >> 2)
// GELU: the activation between fc1 and fc2 applied to every loaded value (fp32, result rounded to bf16 as a separate activation
// kernel would hand it on) before anything else: X is fc1's output as stored, the kernel is fc2's kernel 1
template <int K, int PF, int OCC, bool STATIC, int CB, bool LN = false, bool ASYM = false, bool BLK8 = false, bool GELU = false>
__global__ __launch_bounds__(256, OCC) void rotate_quant_mfma_kernel(const uint16_t *__restrict__ X, int rows,
                                                                   const int8_t *__restrict__ signs,
                                                                   const float *__restrict__ mul, int mul_mode,
                                                                   uint8_t *__restrict__ packed,
                                                                   float *__restrict__ scale,
                                                                   const float *__restrict__ step, int step_stride,
                                                                   float qmax8, unsigned int *__restrict__ col_absmax_bits,
                                                                   LnParams ln = LnParams{nullptr, nullptr, 0.0f, 0},
                                                                   float *__restrict__ zero = nullptr,
                                                                   const uint16_t *__restrict__ gelu_table = nullptr)
{
    constexpr bool STAT = (CB == 0);
    static_assert(!ASYM || ((CB == 4 || CB == 6) && !STATIC), "affine codes: dynamic 4-bit only");
    // CB = 6 with a static step or affine codes: the stored E2M3 number is code + 0.5 resp. u - 7.5 (sixteen half-integers, all
    // representable), and zero[row] receives what the GEMM's correction term needs (8 for a static step: 7.5 - 8 = -0.5)
    using C = rq::Cfg<K>;
    constexpr int REM = C::REM, TOK = C::TOK;
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[rq::WAVES_PER_BLOCK * rq::LDS_PER_WAVE];

    __shared__ __attribute__((aligned(16))) uint16_t gelu_lut[GELU ? rq::GELU_TABLE_ENTRIES : 8];
    if constexpr (GELU) {
        for (int i = threadIdx.x; i < rq::GELU_TABLE_ENTRIES / 8; i += 256)
            reinterpret_cast<uint4 *>(gelu_lut)[i] = reinterpret_cast<const uint4 *>(gelu_table)[i];
        __syncthreads();
    }

    const int lane = threadIdx.x & 63, wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c = lane & 31, g = lane >> 5;
    uint8_t *lds = lds_all + wave_in_block * rq::LDS_PER_WAVE;
    const int wave = blockIdx.x * rq::WAVES_PER_BLOCK + wave_in_block;
    const int nwaves = gridDim.x * rq::WAVES_PER_BLOCK;
    const int ntiles = (rows + TOK - 1) / TOK;

    // ---- per-lane constants -------------------------------------------------------------------
    // sign masks for the packed bf16 pairs this lane loads: load j covers flat elements 512*j + 8*lane .. +8
    // (the eight sign bytes of a load are fetched with one 8-byte load, all loads issued before the first use)
    uint32_t sgn[C::SIGN_CLASSES][4];
#pragma unroll
    for (int q = 0; q < C::SIGN_CLASSES; ++q)
#pragma unroll
        for (int d = 0; d < 4; ++d) sgn[q][d] = 0;
    if (signs != nullptr) {
        uint2 sb[C::SIGN_CLASSES];
#pragma unroll
        for (int q = 0; q < C::SIGN_CLASSES; ++q) sb[q] = *reinterpret_cast<const uint2 *>(signs + 512 * q + 8 * lane);
#pragma unroll
        for (int q = 0; q < C::SIGN_CLASSES; ++q) {
            // bit 7 of a sign byte (set for -1) moves to the sign bit of its bf16: even byte -> bit 15, odd byte -> bit 31
            const uint32_t w[2] = {sb[q].x, sb[q].y};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint32_t two = w[d >> 1] >> (16 * (d & 1));
                sgn[q][d] = ((two & 0x80u) << 8) | ((two & 0x8000u) << 16);
            }
        }
    }
    // B operand: lane (n = c, k-half = g) holds H_128[k][n] for k = 16*ks + 8*g + i.  sign = parity(k & n):
    //   bits 0..3 of k (8*g + i) against c & 15 -> base pattern; bit 4 (ks & 1) against c bit 4; bits 5, 6 (ks >> 1) against nt.
    v8bf Bsel[2][2];
    {
        uint32_t w[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t lo = (__popc((8 * g + 2 * d) & (c & 15)) & 1) ? 0xBF80u : 0x3F80u;
            uint32_t hi = (__popc((8 * g + 2 * d + 1) & (c & 15)) & 1) ? 0xBF80u : 0x3F80u;
            w[d] = lo | (hi << 16);
        }
        const uint32_t flip_odd = (c & 16) ? 0x80008000u : 0u;
#pragma unroll
        for (int odd = 0; odd < 2; ++odd)
#pragma unroll
            for (int neg = 0; neg < 2; ++neg) {
                uint32_t t[4];
#pragma unroll
                for (int d = 0; d < 4; ++d) t[d] = w[d] ^ (odd ? flip_odd : 0u) ^ (neg ? 0x80008000u : 0u);
                Bsel[odd][neg] = *reinterpret_cast<v8bf *>(t);
            }
    }
    // channel multipliers of the lane's values: register r, column tile nt -> element e
    //   hb bits 0..2 = r bits 0..2;  REM 4: hb3 = r bit 3;  REM 5 (after the half swap): hb4 = r bit 3, hb3 = g
    float cm[C::HB_PER_LANE][4];
    {
        const float rs = 1.0f / sqrtf((float)K);
        if (mul != nullptr) {
            // all loads first, then the arithmetic: the loads are in flight together
#pragma unroll
            for (int h = 0; h < C::HB_PER_LANE; ++h)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    int hb = h;
                    if (REM == 5) hb = (h & 7) | (g << 3) | ((h >> 3) << 4);
                    cm[h][nt] = mul[128 * hb + 32 * nt + c];
                }
            if (mul_mode) {
#pragma unroll
                for (int h = 0; h < C::HB_PER_LANE; ++h)
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) cm[h][nt] = 1.0f / ((float)K * cm[h][nt]);
            }
        } else {
#pragma unroll
            for (int h = 0; h < C::HB_PER_LANE; ++h)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) cm[h][nt] = rs;
        }
    }

    // LayerNorm scale / shift of the channels this lane loads: load j of a token's LPT loads covers channels 512 j + 8 lane .. + 8
    constexpr int LPT = 8 / TOK;
    float gam[LN ? LPT : 1][8], bet[LN ? LPT : 1][8];
    if constexpr (LN) {
        static_assert(K == 1024, "the fused LayerNorm keeps 2 * K / 64 scale and shift values per lane: K = 1024 only");
#pragma unroll
        for (int jl = 0; jl < LPT; ++jl)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                gam[jl][i] = ln.gamma ? ln.gamma[512 * jl + 8 * lane + i] : 1.0f;
                bet[jl][i] = ln.beta ? ln.beta[512 * jl + 8 * lane + i] : 0.0f;
            }
    }

    // ---- tile loop ------------------------------------------------------------------------------
    const size_t max_flat = (size_t)rows * K;
    auto tile_ptr = [&](int tile, int j) -> const uint4 * {
        // flat element offset of this lane's 16 bytes of load j; rows past the end re-read the last row
        size_t f = (size_t)tile * TOK * K + (size_t)512 * j + 8 * lane;
        if (f >= max_flat) f = max_flat - K + (f % K);
        return reinterpret_cast<const uint4 *>(X + f);
    };
    // streaming loads: X is read exactly once, and fetched past the caches it leaves room there for what is reused
    auto load16 = [&](const uint4 *p) -> uint4 {
        const v4u v = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(p));
        return make_uint4(v[0], v[1], v[2], v[3]);
    };
    // a tile is 4096 consecutive values; when all its rows exist (a wave-uniform test, false at most for the last tile) the
    // eight loads differ by constants only
    auto load_tile = [&](int t, uint4 (&dst)[8]) {
        if ((t + 1) * TOK <= rows) {
            const uint4 *p = reinterpret_cast<const uint4 *>(X + (size_t)t * 4096) + lane;
#pragma unroll
            for (int j = 0; j < 8; ++j) dst[j] = load16(p + 64 * j);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) dst[j] = load16(tile_ptr(t, j));
        }
    };
    // E2M3 output at K = 4096: a token's 64 units lie 6 KiB apart in the output, 48 bytes each; the four waves of a block take
    // four consecutive tokens and flush them together through LDS, so that memory sees runs of 192 bytes per unit (48-byte
    // pieces cost 190 us more at 137400 tokens).  The block then iterates as one: same trip count, barriers inside the loop.
    static_assert(!BLK8 || CB == 8, "int8 blocks hold int8 codes");
    constexpr bool BLOCK_FLUSH = ((CB == 6 || BLK8) && REM == 5);
    // a unit's (K-tile's) four pieces start FLUSH_PITCH apart: one 16-byte bank group more than they fill, so that the lanes of a
    // write (consecutive units) and of a read spread over the banks
    constexpr int FLUSH_PITCH = (BLK8 ? 256 : 192) + 16;
    __shared__ __attribute__((aligned(16))) uint8_t flush_all[BLOCK_FLUSH ? 64 * FLUSH_PITCH : 16];
    uint4 G[PF][8];
    int tile = wave;
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        if (tile + p * nwaves < ntiles) load_tile(tile + p * nwaves, G[p]);
        else if constexpr (BLOCK_FLUSH) {
#pragma unroll
            for (int j = 0; j < 8; ++j) G[p][j] = make_uint4(0u, 0u, 0u, 0u);
        }
    }
    const int wr_base = ((lane >> 4) * rq::LDS_PITCH) + (lane & 15) * 16;
    const int rd_base = c * rq::LDS_PITCH + g * 16;

    float cmax[STAT ? C::HB_PER_LANE : 1][4];     // statistic mode: running |.| maximum of the lane's columns over its tiles
#pragma unroll
    for (int h = 0; h < (STAT ? C::HB_PER_LANE : 1); ++h)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) cmax[h][nt] = 0.0f;

    for (; (BLOCK_FLUSH ? tile - wave_in_block : tile) < ntiles; tile += nwaves) {
        if constexpr (GELU) {
            // one wave-uniform test per tile: is every value inside the table's window?  (Almost always: outside are exact
            // zeros, |x| < 1e-6 and |x| >= 4096.)  Then two lookups per packed pair; otherwise the general form per value.
            // (a half is inside iff bits 12..14 of its offset from the window's start are zero: OR them all and look once)
            uint32_t D[8][4], any = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                D[j][0] = rq::gelu_window(G[0][j].x); D[j][1] = rq::gelu_window(G[0][j].y);
                D[j][2] = rq::gelu_window(G[0][j].z); D[j][3] = rq::gelu_window(G[0][j].w);
                any = any | D[j][0] | D[j][1];
                any = any | D[j][2] | D[j][3];
            }
            const bool outside = (any & 0x70007000u) != 0u;
            if (__builtin_amdgcn_ballot_w64(outside) == 0) {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    G[0][j] = make_uint4(rq::gelu_pair_table(D[j][0], gelu_lut), rq::gelu_pair_table(D[j][1], gelu_lut),
                                         rq::gelu_pair_table(D[j][2], gelu_lut), rq::gelu_pair_table(D[j][3], gelu_lut));
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    uint32_t w[4] = {G[0][j].x, G[0][j].y, G[0][j].z, G[0][j].w};
#pragma unroll
                    for (int d = 0; d < 4; ++d)
                        w[d] = rq::gelu_one_any(w[d] & 0xFFFFu, gelu_lut) | (rq::gelu_one_any(w[d] >> 16, gelu_lut) << 16);
                    G[0][j] = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
        }
        if constexpr (LN) {
            // every token of the tile: mean, variance (two passes over the registers), normalise, scale / shift, back to bf16
#pragma unroll
            for (int t = 0; t < TOK; ++t) {
                float xv[LPT][8];
                float s1 = 0.0f;
#pragma unroll
                for (int jl = 0; jl < LPT; ++jl) {
                    const uint4 v = G[0][t * LPT + jl];
                    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        xv[jl][2 * d] = __uint_as_float(w[d] << 16);
                        xv[jl][2 * d + 1] = __uint_as_float(w[d] & 0xFFFF0000u);
                        s1 += xv[jl][2 * d] + xv[jl][2 * d + 1];
                    }
                }
                const float mean = sum_over_64_lanes(s1) * (1.0f / (float)K);
                float s2 = 0.0f;
#pragma unroll
                for (int jl = 0; jl < LPT; ++jl)
#pragma unroll
                    for (int i = 0; i < 8; ++i) { xv[jl][i] -= mean; s2 = fmaf(xv[jl][i], xv[jl][i], s2); }
                const float rstd = 1.0f / sqrtf(sum_over_64_lanes(s2) * (1.0f / (float)K) + ln.eps);
#pragma unroll
                for (int jl = 0; jl < LPT; ++jl) {
                    uint32_t w[4];
#pragma unroll
                    for (int d = 0; d < 4; ++d)
                        w[d] = pack_bf16x2(fmaf(xv[jl][2 * d] * rstd, gam[jl][2 * d], bet[jl][2 * d]),
                                           fmaf(xv[jl][2 * d + 1] * rstd, gam[jl][2 * d + 1], bet[jl][2 * d + 1]));
                    G[0][t * LPT + jl] = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
        }
        // stage the tile: flip signs on the packed bf16, write each 16-byte chunk to its MFMA row
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int q = j % C::SIGN_CLASSES;
            uint4 v = G[0][j];
            v.x ^= sgn[q][0]; v.y ^= sgn[q][1]; v.z ^= sgn[q][2]; v.w ^= sgn[q][3];
            // segment index = 4*j + lane/16; its low two bits are lane/16 -> rows m0, m1
            const int row_hi = rq::row_of_seg_hi<K>(j);
            *reinterpret_cast<uint4 *>(lds + row_hi * rq::LDS_PITCH + wr_base) = v;
        }
        lanes_exchange_fence();     // the MFMA operand reads below take what other lanes staged
        // shift the prefetch queue and issue the loads of the tile PF steps ahead
#pragma unroll
        for (int p = 0; p + 1 < PF; ++p)
#pragma unroll
            for (int j = 0; j < 8; ++j) G[p][j] = G[p + 1][j];
        const int next = tile + PF * nwaves;
        if (next < ntiles) load_tile(next, G[PF - 1]);

        // R . H_128 on the matrix cores
        v16f acc[4];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nt][r] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const v8bf a = *reinterpret_cast<const v8bf *>(lds + rd_base + ks * 32);
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                const int neg = __builtin_popcount((ks >> 1) & nt) & 1;
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, Bsel[ks & 1][neg], acc[nt], 0, 0, 0);
            }
        }

        // H_{K/128} over the hi-block index: butterflies between accumulator registers
        constexpr int REG_STAGES = (REM >= 4) ? 4 : 3;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
#pragma unroll
            for (int s = 0; s < REG_STAGES; ++s) {
                const int h = 1 << s;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if ((r & h) == 0) {
                        float a = acc[nt][r], b = acc[nt][r + h];
                        acc[nt][r] = a + b;
                        acc[nt][r + h] = a - b;
                    }
            }
            if constexpr (REM == 5) {
                // hb bit 4 sits on the lane half: swap halves between registers r and r + 8, then the
                // butterfly is between those two registers (register bit 3 now means hb4, the lane half hb3)
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[nt][r]), __float_as_uint(acc[nt][r + 8]), false, false);
                    float a = __uint_as_float(sw[0]), b = __uint_as_float(sw[1]);
                    acc[nt][r] = a + b;
                    acc[nt][r + 8] = a - b;
                }
            }
        }

        if constexpr (STAT) {
            // rows past the end repeat the last row (see tile_ptr), which leaves a maximum unchanged
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) cmax[r % C::HB_PER_LANE][nt] = fmaxf(cmax[r % C::HB_PER_LANE][nt], fabsf(acc[nt][r]));
            continue;
        }
        // scale, absmax per token (STATIC: the quantization step is given, no absmax)
        float amax[C::TOK_PER_LANE], nmin[ASYM ? C::TOK_PER_LANE : 1];      // nmin: -min(0, min z), so both ends reduce with max
#pragma unroll
        for (int t = 0; t < C::TOK_PER_LANE; ++t) amax[t] = 0.0f;
#pragma unroll
        for (int t = 0; t < (ASYM ? C::TOK_PER_LANE : 1); ++t) nmin[t] = 0.0f;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int h = r % C::HB_PER_LANE, t = r / C::HB_PER_LANE;
                acc[nt][r] *= cm[h][nt];
                if constexpr (ASYM) {
                    amax[t] = fmaxf(amax[t], acc[nt][r]);
                    nmin[t] = fmaxf(nmin[t], -acc[nt][r]);
                } else if constexpr (!STATIC) {
                    amax[t] = fmaxf(amax[t], fabsf(acc[nt][r]));
                }
            }
        if constexpr (!STATIC) {
#pragma unroll
            for (int t = 0; t < C::TOK_PER_LANE; ++t) {
                amax[t] = (REM == 5) ? max_over_64_lanes(amax[t]) : max_over_32_lanes(amax[t]);
                if constexpr (ASYM) nmin[t] = (REM == 5) ? max_over_64_lanes(nmin[t]) : max_over_32_lanes(nmin[t]);
            }
        }

        // quantize, pack, store
#pragma unroll
        for (int t = 0; t < C::TOK_PER_LANE; ++t) {
            // token of this lane: REM 3: 2*t + g (m bit 4 = register bit 3, m bit 2 = lane half); REM 4: g; REM 5: 0
            const int tk = (REM == 3) ? (2 * t + g) : (REM == 4 ? g : 0);
            const int row = tile * TOK + tk;
            float inv, delta;
            float magic = rq::MAGIC, zp = 0.0f;
            if constexpr (ASYM) {
                // step (hi - lo) / 15, zero point rne(-lo / step) in [0, 15]; u = rne(z / step) + zp is formed as the low mantissa
                // bits of z * inv + (MAGIC - 8 + zp) (MAGIC carries the + 8 of the symmetric codes) and clamped to [0, 15] there
                const float range = amax[t] + nmin[t];
                const bool live = range >= 15.0f * kMinStep;
                delta = live ? range / 15.0f : 0.0f;
                inv = live ? 15.0f * __builtin_amdgcn_rcpf(range) : 0.0f;
                zp = __builtin_rintf(nmin[t] * inv);
                magic = rq::MAGIC - 8.0f + zp;
            } else if constexpr (STATIC) {
                delta = step[(size_t)min(row, rows - 1) * step_stride];
                inv = delta >= kMinStep ? 1.0f / delta : 0.0f;
            } else {
                // hardware reciprocal (1 ulp) instead of two IEEE divisions: |z| * inv <= qmax (1 + 2^-22) still rounds to qmax
                const float qmax = (CB == 4 || CB == 6) ? 7.0f : qmax8;
                const bool live = amax[t] >= qmax * kMinStep;
                delta = live ? amax[t] / qmax : 0.0f;
                inv = live ? qmax * __builtin_amdgcn_rcpf(amax[t]) : 0.0f;
            }
            if constexpr (CB == 6) {
                // The lane's NL codes are positions P0 .. P0 + NL - 1 of the row, i.e. NL / 32 whole blobs; field f of a blob is local
                // index 32 bb + f = nt + 4 h.  The conversion instruction takes the even fields from its first operand and the odd
                // ones from its second; integers up to 7 are E2M3 numbers, so it is exact.
                typedef float v16f __attribute__((ext_vector_type(16)));
                typedef unsigned int v6u __attribute__((ext_vector_type(6)));
                const int P0 = c * (K / 32) + (REM == 5 ? g * 64 : 0);
#pragma unroll
                for (int bb = 0; bb < C::NL / 32; ++bb) {
                    v16f ev, od;
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        const int h = 8 * bb + k / 2;
                        // rounded exactly as the packed codes are: one fused rounding onto the integer grid of the magic constant
                        const float ze = acc[(2 * k) & 3][t * C::HB_PER_LANE + h], zo = acc[(2 * k + 1) & 3][t * C::HB_PER_LANE + h];
                        if constexpr (ASYM) {
                            ev[k] = (__builtin_amdgcn_fmed3f(fmaf(ze, inv, magic), rq::MAGIC - 8.0f, rq::MAGIC + 7.0f) - rq::MAGIC) + 0.5f;
                            od[k] = (__builtin_amdgcn_fmed3f(fmaf(zo, inv, magic), rq::MAGIC - 8.0f, rq::MAGIC + 7.0f) - rq::MAGIC) + 0.5f;
                        } else if constexpr (STATIC) {
                            ev[k] = ((__builtin_amdgcn_fmed3f(ze * inv, -8.0f, 7.0f) + rq::MAGIC) - rq::MAGIC) + 0.5f;
                            od[k] = ((__builtin_amdgcn_fmed3f(zo * inv, -8.0f, 7.0f) + rq::MAGIC) - rq::MAGIC) + 0.5f;
                        } else {
                            ev[k] = fmaf(ze, inv, rq::MAGIC) - rq::MAGIC;
                            od[k] = fmaf(zo, inv, rq::MAGIC) - rq::MAGIC;
                        }
                    }
                    // The conversion makes several passes over its 32 source registers while it writes its 6 results, so the result
                    // must not share registers with the sources.  The compiler's builtin does not know that (it was seen to place
                    // the result on the last source registers, which corrupted fields 25 .. 31): the early-clobber constraint does.
                    v6u blob;
                    asm volatile("v_cvt_scalef32_2xpk16_fp6_f32 %0, %1, %2, 1.0" : "=&v"(blob) : "v"(ev), "v"(od));
                    if constexpr (REM == 5) {
                        // K = 4096: the lane holds both blobs of unit 2 c + g, i.e. that unit's 48 bytes of this wave's token; they go
                        // to the block's flush area [unit][wave][48 bytes]
                        uint8_t *slot = flush_all + (2 * c + g) * FLUSH_PITCH + wave_in_block * 48;
                        if (bb == 0) {
                            *reinterpret_cast<uint4 *>(slot) = make_uint4(blob[0], blob[1], blob[2], blob[3]);
                            *reinterpret_cast<uint2 *>(slot + 32) = make_uint2(blob[4], blob[5]);
                        } else {
                            *reinterpret_cast<uint4 *>(slot + 16) = make_uint4(blob[0], blob[1], blob[2], blob[3]);
                            *reinterpret_cast<uint2 *>(slot + 40) = make_uint2(blob[4], blob[5]);
                        }
                        continue;
                    }
                    if (row < rows) {
                        const int pb = P0 / 32 + bb;            // blob of the row: unit pb / 2, half pb % 2
                        uint8_t *u = packed + ((size_t)(row / 128) * (K / 64) + (pb >> 1)) * 6144 + (size_t)(row % 128) * 48;
                        *reinterpret_cast<uint4 *>(u + (pb & 1) * 16) = make_uint4(blob[0], blob[1], blob[2], blob[3]);
                        *reinterpret_cast<uint2 *>(u + 32 + (pb & 1) * 8) = make_uint2(blob[4], blob[5]);
                    }
                }
                if constexpr (REM == 5) {
                    __syncthreads();
                    // the block's four tokens are rows row4 .. row4 + 3 of one 128-row block: 192 contiguous bytes per unit
                    const int row4 = tile - wave_in_block;
                    uint8_t *rb = packed + (size_t)(row4 / 128) * (K / 64) * 6144 + (size_t)(row4 % 128) * 48;
#pragma unroll
                    for (int i = 0; i < 3; ++i) {
                        const int j = i * 256 + (int)threadIdx.x, unit = j / 12, within = j - 12 * unit;     // 16-byte chunk j of 768
                        if (row4 + within / 3 < rows)
                        {
                            // whole runs of 192 bytes, written past the caches: the 422 MB of a 137400-token launch would otherwise sit
                            // there as dirty lines while the GEMM that follows runs (measured: that GEMM 365 -> 312 us, this kernel + 4 us);
                            // the direct stores of the smaller K stay cached: their pieces are partial lines and their output fits the
                            // memory-side cache, where the GEMM finds it
                            const uint4 fv = *reinterpret_cast<const uint4 *>(flush_all + unit * FLUSH_PITCH + within * 16);
                            const v4u nv = {fv.x, fv.y, fv.z, fv.w};
                            __builtin_nontemporal_store(nv, reinterpret_cast<v4u *>(rb + (size_t)unit * 6144 + within * 16));
                        }
                    }
                    __syncthreads();
                }
                if (row < rows && c == 0 && (REM != 5 || g == 0)) {
                    scale[row] = delta;
                    if constexpr (ASYM) zero[row] = zp;
                    if constexpr (STATIC) zero[row] = 8.0f;
                }
                continue;
            }
            if constexpr (CB == 8) {
                // four codes per word: byte i of word d is local index 4*d + i = nt + 4*h  ->  nt = i, h = d
                uint32_t words[C::NL / 4];
#pragma unroll
                for (int d = 0; d < C::NL / 4; ++d) {
                    uint32_t wv = 0;
#pragma unroll
                    for (int i = 3; i >= 0; --i) {
                        float f;
                        if constexpr (STATIC) f = __builtin_amdgcn_fmed3f(acc[i][t * C::HB_PER_LANE + d] * inv, -qmax8 - 1.0f, qmax8) + rq::MAGIC8;
                        else f = fmaf(acc[i][t * C::HB_PER_LANE + d], inv, rq::MAGIC8);
                        wv = (wv << 8) + __float_as_uint(f);
                    }
                    constexpr uint32_t BIAS8 = (uint32_t)(0x4B400000ull * 0x01010101ull);
                    words[d] = (wv - BIAS8) ^ 0x80808080u;
                }
                if constexpr (BLK8) {
                    // the lane's NL bytes are positions P0 .. of the row: chunk P / 16 of K-tile P / 64
                    const int P0 = c * (K / 32) + (REM == 5 ? g * 64 : 0);
                    const int swz = (row & 15) >> 2;
                    if constexpr (REM == 5) {
                        // K = 4096: the lane holds K-tile 2 c + g of this wave's token, 64 bytes; the block's four tokens leave together
                        // (flush area [K-tile][wave][64 bytes]) in runs of 256 bytes, see the 6-bit variant
                        uint8_t *slot = flush_all + (P0 / 64) * FLUSH_PITCH + wave_in_block * 64;
#pragma unroll
                        for (int d4 = 0; d4 < 4; ++d4)
                            *reinterpret_cast<uint4 *>(slot + ((d4 ^ swz) * 16)) = make_uint4(words[4 * d4], words[4 * d4 + 1], words[4 * d4 + 2], words[4 * d4 + 3]);
                        __syncthreads();
                        const int row4 = tile - wave_in_block;
                        uint8_t *rb = packed + (size_t)(row4 / 128) * (K / 64) * 8192 + (size_t)(row4 % 128) * 64;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int j = i * 256 + (int)threadIdx.x, kt = j / 16, within = j - 16 * kt;      // 16-byte chunk j of 1024
                            if (row4 + within / 4 < rows) {
                                const uint4 fv = *reinterpret_cast<const uint4 *>(flush_all + kt * FLUSH_PITCH + within * 16);
                                const v4u nv = {fv.x, fv.y, fv.z, fv.w};
                                __builtin_nontemporal_store(nv, reinterpret_cast<v4u *>(rb + (size_t)kt * 8192 + within * 16));     // as the 6-bit variant
                            }
                        }
                        __syncthreads();
                    } else if (row < rows) {
                        uint8_t *rb = packed + (size_t)(row / 128) * (K / 64) * 8192 + (size_t)(row % 128) * 64;
#pragma unroll
                        for (int d4 = 0; d4 < C::NL / 16; ++d4) {
                            const int P = P0 + 16 * d4;
                            *reinterpret_cast<uint4 *>(rb + (size_t)(P / 64) * 8192 + ((((P % 64) / 16) ^ swz) * 16)) =
                                make_uint4(words[4 * d4], words[4 * d4 + 1], words[4 * d4 + 2], words[4 * d4 + 3]);
                        }
                    }
                    if (row < rows && c == 0 && (REM != 5 || g == 0)) scale[row] = delta;
                    continue;
                }
                if (row < rows) {
                    uint8_t *out = packed + (size_t)row * K + (size_t)c * (K / 32) + (REM == 5 ? g * 64 : 0);
#pragma unroll
                    for (int d4 = 0; d4 < C::NL / 16; ++d4)
                        *reinterpret_cast<uint4 *>(out + 16 * d4) = make_uint4(words[4 * d4], words[4 * d4 + 1], words[4 * d4 + 2], words[4 * d4 + 3]);
                    if (c == 0 && (REM != 5 || g == 0)) scale[row] = delta;
                }
                continue;
            }
            uint32_t words[C::NL / 8];
#pragma unroll
            for (int d = 0; d < C::NL / 8; ++d) {
                // nibble i of word d is local index 8*d + i = nt + 4*h  ->  nt = i & 3, h = 2*d + (i >> 2)
                uint32_t wv = 0;
#pragma unroll
                for (int i = 7; i >= 0; --i) {
                    const int nt = i & 3, h = 2 * d + (i >> 2);
                    float f;
                    if constexpr (ASYM) {       // rounding noise at the ends of the range may reach -1 or 16: clamp after the rounding
                        f = __builtin_amdgcn_fmed3f(fmaf(acc[nt][t * C::HB_PER_LANE + h], inv, magic), rq::MAGIC - 8.0f, rq::MAGIC + 7.0f);
                    } else if constexpr (STATIC) {     // a given step does not bound the ratio: clamp to the code range (ties to even below)
                        f = __builtin_amdgcn_fmed3f(acc[nt][t * C::HB_PER_LANE + h] * inv, -8.0f, 7.0f) + rq::MAGIC;
                    } else {
                        f = fmaf(acc[nt][t * C::HB_PER_LANE + h], inv, rq::MAGIC);
                    }
                    wv = (wv << 4) + __float_as_uint(f);
                }
                // remove the eight copies of the magic exponent pattern, then offset-binary -> two's complement
                constexpr uint32_t BIAS = (uint32_t)(0x4B400000ull * 0x11111111ull);
                words[d] = (wv - BIAS) ^ 0x88888888u;
            }
            if (row < rows) {
                uint8_t *out = packed + (size_t)row * (K / 2) + (size_t)c * (K / 64) + (REM == 5 ? g * 32 : 0);
#pragma unroll
                for (int d4 = 0; d4 < C::NL / 32; ++d4)
                    *reinterpret_cast<uint4 *>(out + 16 * d4) = make_uint4(words[4 * d4], words[4 * d4 + 1], words[4 * d4 + 2], words[4 * d4 + 3]);
                if (c == 0 && (REM != 5 || g == 0)) {
                    scale[row] = delta;
                    if constexpr (ASYM) zero[row] = zp;
                }
            }
        }
    }
    if constexpr (STAT) {
        // the block's waves fold their maxima in LDS (non-negative floats order like their bit patterns), then every column
        // costs one global atomic per block
        unsigned int *blk = reinterpret_cast<unsigned int *>(lds_all);
        static_assert(sizeof(lds_all) >= K * sizeof(unsigned int), "the staging area holds one value per column");
        __syncthreads();
        for (int j = threadIdx.x; j < K; j += 256) blk[j] = 0u;
        __syncthreads();
        const float rs = 1.0f / sqrtf((float)K);
#pragma unroll
        for (int h = 0; h < C::HB_PER_LANE; ++h)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                int hb = h;
                if (REM == 5) hb = (h & 7) | (g << 3) | ((h >> 3) << 4);
                atomicMax(&blk[128 * hb + 32 * nt + c], __float_as_uint(cmax[h][nt] * rs));
            }
        __syncthreads();
        for (int j = threadIdx.x; j < K; j += 256) atomicMax(&col_absmax_bits[j], blk[j]);
    }
}

hipError_t run_rotate_quant_mfma(const void *X, int rows, int K, const int8_t *signs, const float *mul, int mul_mode,
                                 uint8_t *packed, float *scale, const float *step, int step_stride, int bits,
                                 hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    const uint16_t *x = reinterpret_cast<const uint16_t *>(X);
    const int tok = 32 / (K / 128);
    const int ntiles = (rows + tok - 1) / tok;
    int blocks = (ntiles + rq::WAVES_PER_BLOCK - 1) / rq::WAVES_PER_BLOCK;
    const int max_blocks = 256 * 2;   // two resident blocks of four waves on each of the 256 compute units
    if (blocks > max_blocks) blocks = max_blocks;
    const float qmax8 = (float)((1 << (code_width(bits) - 1)) - 1);
#define RQ1(KK, PF, OCC, ST, CB) rotate_quant_mfma_kernel<KK, PF, OCC, ST, CB><<<blocks, 256, 0, stream>>>(x, rows, signs, mul, mul_mode, packed, scale, step, step_stride, qmax8, nullptr)
#define RQ(KK, PF, OCC)                                      \
    do {                                                     \
        if (bits == 4) {                                     \
            if (step != nullptr) RQ1(KK, PF, OCC, true, 4);  \
            else RQ1(KK, PF, OCC, false, 4);                 \
        } else {                                             \
            if (step != nullptr) RQ1(KK, PF, OCC, true, 8);  \
            else RQ1(KK, PF, OCC, false, 8);                 \
        }                                                    \
    } while (0)
    switch (K) {
        case 1024: RQ(1024, 1, 2); break;
        case 2048: RQ(2048, 1, 2); break;
        case 4096: RQ(4096, 1, 2); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// rotation + smoothing + per-token affine 4-bit codes (stored as u - 8) with zero points, bf16 rows, K = 1024 / 2048 / 4096
hipError_t run_rotate_quant_asym_mfma(const void *X, int rows, int K, const int8_t *signs, const float *mul, uint8_t *packed,
                                      float *scale, float *zero, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    const uint16_t *x = reinterpret_cast<const uint16_t *>(X);
    const int tok = 32 / (K / 128);
    const int ntiles = (rows + tok - 1) / tok;
    int blocks = (ntiles + rq::WAVES_PER_BLOCK - 1) / rq::WAVES_PER_BLOCK;
    if (blocks > 256 * 2) blocks = 256 * 2;
#define RQA(KK) rotate_quant_mfma_kernel<KK, 1, 2, false, 4, false, true><<<blocks, 256, 0, stream>>>(x, rows, signs, mul, 0, packed, scale, nullptr, 0, 7.0f, nullptr, LnParams{nullptr, nullptr, 0.0f, 0}, zero)
    switch (K) {
        case 1024: RQA(1024); break;
        case 2048: RQA(2048); break;
        case 4096: RQA(4096); break;
        default: return hipErrorInvalidValue;
    }
#undef RQA
    return hipGetLastError();
}

// The activation table: entry e (sign = e >> 12, magnitude bits 0x3580 + (e & 0xFFF)) = bf16(x Phi(x)), evaluated in double
// (Phi(x) = erfc(-x / sqrt 2) / 2, so that the negative tail keeps its relative accuracy) and rounded once, to nearest even,
// subnormal results included.
__global__ __launch_bounds__(256) void gelu_table_kernel(uint16_t *__restrict__ table)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= rq::GELU_TABLE_ENTRIES) return;
    const uint32_t bits = ((uint32_t)(e >> 12) << 15) | (rq::GELU_U0 + (uint32_t)(e & 0xFFF));
    const double x = (double)__uint_as_float(bits << 16);
    const double y = x * (0.5 * erfc(-x * 0.70710678118654752440));
    const double a = fabs(y);
    uint32_t r = 0;
    if (a > 0.0) {
        int ex;
        (void)frexp(a, &ex);                               // a = m 2^ex, 0.5 <= m < 1: the leading bit has weight 2^(ex - 1)
        if (ex - 1 >= -126) {                              // normal bf16: 8 significant bits; a carry out of them bumps the exponent field
            const uint32_t q = (uint32_t)rint(ldexp(a, 7 - (ex - 1)));     // 128 .. 256
            r = ((uint32_t)(ex - 1 + 127) << 7) + (q - 128u);
        } else {
            r = (uint32_t)rint(ldexp(a, 133));             // subnormal: multiples of 2^-133; 128 is the smallest normal
        }
    }
    table[e] = (uint16_t)(r | (signbit(y) ? 0x8000u : 0u));
}

hipError_t run_gelu_table(void *table, hipStream_t stream)
{
    gelu_table_kernel<<<rq::GELU_TABLE_ENTRIES / 256, 256, 0, stream>>>(reinterpret_cast<uint16_t *>(table));
    return hipGetLastError();
}

// GELU + rotation + smoothing + per-token 4-bit codes, packed rows (e2m3 = false) or E2M3 blocks, bf16 rows, K = 1024 / 2048 / 4096
hipError_t run_gelu_rotate_quant_mfma(const void *X, int rows, int K, const int8_t *signs, const float *mul, const void *gelu_table,
                                      uint8_t *out, float *scale, bool e2m3, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    const uint16_t *x = reinterpret_cast<const uint16_t *>(X);
    const int tok = 32 / (K / 128);
    const int ntiles = (rows + tok - 1) / tok;
    int blocks = (ntiles + rq::WAVES_PER_BLOCK - 1) / rq::WAVES_PER_BLOCK;
    if (blocks > 256 * 2) blocks = 256 * 2;
    const LnParams no_ln{nullptr, nullptr, 0.0f, 0};
#define RQG(KK, CB) rotate_quant_mfma_kernel<KK, 1, 2, false, CB, false, false, false, true><<<blocks, 256, 0, stream>>>(x, rows, signs, mul, 0, out, scale, nullptr, 0, 7.0f, nullptr, no_ln, nullptr, reinterpret_cast<const uint16_t *>(gelu_table))
    switch (K) {
        case 1024: if (e2m3) RQG(1024, 6); else RQG(1024, 4); break;
        case 2048: if (e2m3) RQG(2048, 6); else RQG(2048, 4); break;
        case 4096: if (e2m3) RQG(4096, 6); else RQG(4096, 4); break;
        default: return hipErrorInvalidValue;
    }
#undef RQG
    return hipGetLastError();
}

// rotation + smoothing + per-token int8 codes of `bits` bits as int8 blocks (what the blocked int8 GEMM reads), bf16 rows
hipError_t run_rotate_quant_i8b_mfma(const void *X, int rows, int K, const int8_t *signs, const float *mul, uint8_t *out,
                                     float *scale, int bits, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    const uint16_t *x = reinterpret_cast<const uint16_t *>(X);
    const int tok = 32 / (K / 128);
    const int ntiles = (rows + tok - 1) / tok;
    int blocks = (ntiles + rq::WAVES_PER_BLOCK - 1) / rq::WAVES_PER_BLOCK;
    if (blocks > 256 * 2) blocks = 256 * 2;
    const float qmax8 = (float)((1 << (bits - 1)) - 1);
    const LnParams no_ln{nullptr, nullptr, 0.0f, 0};
#define RQB(KK) rotate_quant_mfma_kernel<KK, 1, 2, false, 8, false, false, true><<<blocks, 256, 0, stream>>>(x, rows, signs, mul, 0, out, scale, nullptr, 0, qmax8, nullptr, no_ln, nullptr)
    switch (K) {
        case 1024: RQB(1024); break;
        case 2048: RQB(2048); break;
        case 4096: RQB(4096); break;
        default: return hipErrorInvalidValue;
    }
#undef RQB
    return hipGetLastError();
}

// rotation + smoothing + per-token 4-bit codes as E2M3 blocks (what the 6-bit matrix GEMM reads), bf16 rows, K = 1024 / 2048 / 4096
hipError_t run_rotate_quant_e2m3_mfma(const void *X, int rows, int K, const int8_t *signs, const float *mul, uint8_t *out,
                                      float *scale, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    const uint16_t *x = reinterpret_cast<const uint16_t *>(X);
    const int tok = 32 / (K / 128);
    const int ntiles = (rows + tok - 1) / tok;
    int blocks = (ntiles + rq::WAVES_PER_BLOCK - 1) / rq::WAVES_PER_BLOCK;
    if (blocks > 256 * 2) blocks = 256 * 2;
#define RQE(KK) rotate_quant_mfma_kernel<KK, 1, 2, false, 6><<<blocks, 256, 0, stream>>>(x, rows, signs, mul, 0, out, scale, nullptr, 0, 7.0f, nullptr)
    switch (K) {
        case 1024: RQE(1024); break;
        case 2048: RQE(2048); break;
        case 4096: RQE(4096); break;
        default: return hipErrorInvalidValue;
    }
#undef RQE
    return hipGetLastError();
}

// The variants whose codes fill [-8, 7] or [0, 15], as E2M3 blocks of half-integers (code + 0.5, u - 7.5) plus zero[row]:
// step != nullptr: static step (token-wise, stride 1, or one value, stride 0), zero = 8; otherwise affine codes, zero = zero point
hipError_t run_rotate_quant_e2m3_shifted_mfma(const void *X, int rows, int K, const int8_t *signs, const float *mul, uint8_t *out,
                                              float *scale, float *zero, const float *step, int step_stride, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    const uint16_t *x = reinterpret_cast<const uint16_t *>(X);
    const int tok = 32 / (K / 128);
    const int ntiles = (rows + tok - 1) / tok;
    int blocks = (ntiles + rq::WAVES_PER_BLOCK - 1) / rq::WAVES_PER_BLOCK;
    if (blocks > 256 * 2) blocks = 256 * 2;
    const LnParams no_ln{nullptr, nullptr, 0.0f, 0};
#define RQS(KK)                                                                                                                          \
    do {                                                                                                                                 \
        if (step != nullptr)                                                                                                             \
            rotate_quant_mfma_kernel<KK, 1, 2, true, 6, false, false><<<blocks, 256, 0, stream>>>(x, rows, signs, mul, 0, out, scale, step, step_stride, 7.0f, nullptr, no_ln, zero); \
        else                                                                                                                             \
            rotate_quant_mfma_kernel<KK, 1, 2, false, 6, false, true><<<blocks, 256, 0, stream>>>(x, rows, signs, mul, 0, out, scale, nullptr, 0, 7.0f, nullptr, no_ln, zero);     \
    } while (0)
    switch (K) {
        case 1024: RQS(1024); break;
        case 2048: RQS(2048); break;
        case 4096: RQS(4096); break;
        default: return hipErrorInvalidValue;
    }
#undef RQS
    return hipGetLastError();
}

// LayerNorm + rotation + smoothing + per-token 4-bit quantization of bf16 rows, K = 1024
hipError_t run_ln_rotate_quant_mfma(const void *X, int rows, const int8_t *signs, const float *mul, uint8_t *packed, float *scale,
                                    LnParams ln, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    const int ntiles = (rows + 3) / 4;
    int blocks = (ntiles + rq::WAVES_PER_BLOCK - 1) / rq::WAVES_PER_BLOCK;
    if (blocks > 256 * 2) blocks = 256 * 2;
    rotate_quant_mfma_kernel<1024, 1, 2, false, 4, true><<<blocks, 256, 0, stream>>>(
        reinterpret_cast<const uint16_t *>(X), rows, signs, mul, 0, packed, scale, nullptr, 0, 7.0f, nullptr, ln);
    return hipGetLastError();
}

// the same with the codes written as E2M3 blocks
hipError_t run_ln_rotate_quant_e2m3_mfma(const void *X, int rows, const int8_t *signs, const float *mul, uint8_t *out, float *scale,
                                         LnParams ln, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    const int ntiles = (rows + 3) / 4;
    int blocks = (ntiles + rq::WAVES_PER_BLOCK - 1) / rq::WAVES_PER_BLOCK;
    if (blocks > 256 * 2) blocks = 256 * 2;
    rotate_quant_mfma_kernel<1024, 1, 2, false, 6, true><<<blocks, 256, 0, stream>>>(
        reinterpret_cast<const uint16_t *>(X), rows, signs, mul, 0, out, scale, nullptr, 0, 7.0f, nullptr, ln);
    return hipGetLastError();
}

// Column statistic max_t |X H|[t, j] of bf16 rows, K = 1024 / 2048 / 4096, with the same kernel in statistic mode.
// absmax_bits (K values) must be zero on entry.
hipError_t run_rotated_col_absmax_mfma(const void *X, int rows, int K, const int8_t *signs, unsigned int *absmax_bits,
                                       hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    const uint16_t *x = reinterpret_cast<const uint16_t *>(X);
    const int tok = 32 / (K / 128);
    const int ntiles = (rows + tok - 1) / tok;
    // sixteen tiles or more per wave where there are that many: every wave ends with atomics on all K columns
    int blocks = (ntiles + 16 * rq::WAVES_PER_BLOCK - 1) / (16 * rq::WAVES_PER_BLOCK);
    if (blocks > 256 * 2) blocks = 256 * 2;
#define RQS(KK) rotate_quant_mfma_kernel<KK, 1, 2, false, 0><<<blocks, 256, 0, stream>>>(x, rows, signs, nullptr, 0, nullptr, nullptr, nullptr, 0, 0.0f, absmax_bits)
    switch (K) {
        case 1024: RQS(1024); break;
        case 2048: RQS(2048); break;
        case 4096: RQS(4096); break;
        default: return hipErrorInvalidValue;
    }
#undef RQS
    return hipGetLastError();
}

}  // namespace qvggt
