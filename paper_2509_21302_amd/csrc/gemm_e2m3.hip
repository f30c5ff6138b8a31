// Online kernel 2 on the 6-bit floating-point matrix path: the same integer product
//
//   acc[t, o] = sum_j Xq[t, j] * Wq[o, j]                 (paper Sec. 3.2, granularity paragraph)
//   Y[t, o]   = bf16( acc[t, o] * sx[t] * sw[o] + bias[o] )
//
// with every 4-bit code q in [-7, 7] written as the E2M3 number of the same value (1 sign, 2 exponent, 3 mantissa bits:
// 0, 1, 2, ..., 7 are all representable) and multiplied by v_mfma_f32_32x32x64_f8f6f4 (no block scales).  Products are
// integers of magnitude <= 49 and sums of magnitude <= 49 * 8192 < 2^24, so the fp32 accumulators hold the integer sum
// exactly, in any order of addition: the result is the int32 accumulator of the int8 path, bit for bit.  On gfx950 this
// MFMA retires 64 codes per row in the time the int8 one retires 32, and a lane's operand comes from LDS as it is (no
// expansion in registers).  -8 has no E2M3 value: dynamic absmax steps never produce it (codes lie in [-7, 7]); codes that
// fill the whole range (static steps, affine codes) are stored half a step up, as the half-integers -7.5 .. 7.5, all of which
// are E2M3 numbers, and the epilogue adds the term that makes up for the shift (SHIFTED below).
//
// Operand format ("E2M3 blocks").  A row of K codes is K / 64 units of 48 bytes.  Unit s holds the codes at positions
// 64 s .. 64 s + 63 of the library's code order as two blobs of 32 six-bit fields (field i of blob h = position 64 s + 32 h + i,
// at bits [6 i, 6 i + 6) of the blob's 192 bits), laid out [blob 0 bytes 0..15][blob 1 bytes 0..15][blob 0 bytes 16..23]
// [blob 1 bytes 16..23]: lane (row = lane % 32, h = lane / 32) of a fragment takes its blob with one 16-byte and one 8-byte
// LDS read.  Both operands use the same order inside a unit, which is all a dot product needs.  In memory the rows are
// grouped in blocks of 128: unit s of row r lies at ((r / 128) * (K / 64) + s) * 6144 + (r % 128) * 48, so that what a tile
// needs of one unit is 6 KiB contiguous per 128 rows.  (The matrix rate needs 24 KiB per compute unit every ~530 cycles; row-major
// rows deliver 48-byte pieces of 128-byte lines and measured 3.2 times slower through the same path than contiguous KiBs.)
//
// Data movement: persistent blocks, XCD-contiguous tile ranges, operands from global memory straight into an LDS ring
// (global_load_lds_dwordx4, 1 KiB contiguous per wave instruction, here also contiguous in memory), one unit (one MFMA K-step)
// per ring stage.  A stage is the memory image of the tile's rows of that unit: token rows, then channel rows, 48 bytes each, which
// need no swizzle for the 16-byte reads (16 consecutive rows start in 16 different 16-byte bank groups: 3 is odd).  Its 1 KiB pieces
// are dealt to the waves in turn (piece n to wave n % 4), so any tile whose rows are multiples of 128 divides.
//
// Tiles: 256 x 256 per block, one block per compute unit, four waves of 128 x 128 (256 accumulator registers each): the least
// operand traffic per MFMA that the register file allows; 128 x 128 blocks, two per compute unit, for problems of less than a round.
// (256 x 128 blocks, two per compute unit, so that one block's epilogue runs under the other's K loop, were built and measured:
// the K loop is not limited by the matrix pipes but by what feeds them, and 1.5 times the LDS traffic per MFMA ate the overlap.)
// The epilogue: accumulators from AGPRs, scale + bias, bf16, rows through a wave-private LDS tile, non-temporal 128-byte line
// stores.
#include "qvggt_common.h"

#include <algorithm>
#include <cstdlib>
#include <type_traits>
#include <utility>

namespace qvggt {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

namespace {

constexpr int U_BYTES = 48;        // bytes per row per unit: 64 codes of 6 bits
constexpr int RB = 128;            // rows per block of the operand format
constexpr int RB_BYTES = RB * U_BYTES;   // one unit of one block: 6 KiB contiguous
constexpr int RB_PIECES = RB_BYTES / 1024;
// Scale operands of the matrix builtin.  Constant zeros make the compiler emit the instruction form without block scales
// (v_mfma_f32_32x32x64_f8f6f4: products as they are), one instruction per MFMA instead of two; 0x7F7F7F7F (E8M0 exponent 127 = 2^0
// in every byte) is the explicit unit scale and gives the same sums.
constexpr int UNIT_SCALE_ONE = 0;

// SHIFTED: the activation codes are stored 7.5 below an unsigned code u in [0, 15] (all sixteen half-integers -7.5 .. 7.5 are E2M3
// numbers), with a zero point per token; the per-tile scale area then also carries the zero points and the weights' code sums
template <int TM, int TN, int WM, int WN, int STAGES, bool SHIFTED = false>
struct E2m3Cfg {
    static constexpr int NW = WM * WN, THREADS = NW * 64;
    static constexpr int BM = WM * TM * 32, BN = WN * TN * 32, ROWS = BM + BN;
    static constexpr int STAGE_BYTES = ROWS * U_BYTES;
    static constexpr int XT = BM * 3 / 64, NT = ROWS * 3 / 64;      // 1 KiB pieces of a stage: the first XT are token rows
    static constexpr int LPW = (NT + NW - 1) / NW;                  // transfer slots per wave and unit (the last may be empty for some waves)
    static constexpr int LPW_MIN = NT / NW;                         // transfers every wave issues per unit
    static constexpr int NM = TM * TN, NF = TM + TN;
    static constexpr int SC_SYM_BYTES = BM * 4 + BN * 4 + BN * 2;   // per tile: sx f32, sw f32, bias bf16 (as in memory)
    static constexpr int SC_SYM_GROUPS = BM / 64 + BN / 64 + BN / 128;
    static constexpr int SC_BYTES = SC_SYM_BYTES + (SHIFTED ? BM * 4 + BN * 4 : 0);     // then zero points f32, code sums f32
    static constexpr int SC_GROUPS = SC_SYM_GROUPS + (SHIFTED ? BM / 64 + BN / 64 : 0);
    static constexpr int EP_PITCH = 128 + 16;
    static constexpr int EP_BYTES = NW * 32 * EP_PITCH;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES + 2 * SC_BYTES + EP_BYTES;
    static_assert(TN % 2 == 0, "the epilogue handles channel sub-tiles in pairs");
    static_assert(BM % 128 == 0 && BN % 128 == 0, "tiles are whole 128-row blocks of the operand format");
    static_assert(STAGES >= 3, "ring needs one stage being read, one landed, one in flight");
};

// Global memory -> LDS, 16 bytes per lane: lane l reads base + lane_off and writes LDS address lds_base + 16 * l.  M0 carries the
// LDS base; each transfer sets it itself and says so, so nothing depends on what the compiler does with that register elsewhere.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ inline void e_dma16(uint32_t lane_off, const void *base, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(lds_base) : "memory", "m0");
}
// 4 bytes per lane: lane l writes lds_base + 4 * l
__device__ inline void e_dma4(const void *src, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" ::"v"(src), "s"(lds_base) : "memory", "m0");
}
#pragma clang diagnostic pop
template <class F, int... Is>
__device__ inline void e_static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ inline void e_static_for(F &&f)
{
    e_static_for_impl(f, std::make_integer_sequence<int, N>{});
}
template <int N>
__device__ inline void e_wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

}  // namespace

// SHIFTED: sum_j (u_tj - zp_t) qw_oj = sum_j (u_tj - 7.5) qw_oj + (7.5 - zp_t) * wsum_o: the first sum is what the MFMAs give (multiples
// of 0.5 below 2^23: exact), the second term is added in the epilogue (exact as well)
template <int TM, int TN, int WM, int WN, int STAGES, int MINB, bool DEBUG, bool SHIFTED = false>
__global__ __launch_bounds__(WM * WN * 64, MINB) __attribute__((amdgpu_waves_per_eu(WM * WN * MINB / 4, WM * WN * MINB / 4))) void e2m3_gemm_kernel(
    const uint8_t *__restrict__ Xf, const float *__restrict__ sx, const uint8_t *__restrict__ Wf,
    const float *__restrict__ sw, const uint16_t *__restrict__ bias, int M, int N, int K,
    uint16_t *__restrict__ Y, int32_t *__restrict__ acc_debug, int tiles_m, int tiles_n,
    const float *__restrict__ xzero = nullptr, const float *__restrict__ wsum = nullptr)
{
    using C = E2m3Cfg<TM, TN, WM, WN, STAGES, SHIFTED>;
    constexpr int NM = C::NM, NF = C::NF, LPW = C::LPW;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    uint8_t *sc_all = smem + STAGES * C::STAGE_BYTES;           // two buffers of SC_BYTES
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int units = K >> 6;                                   // even: K is a multiple of 128
    const int ntiles = tiles_m * tiles_n;

    // tile assignment: XCD x (blocks are dealt round-robin to the 8 XCDs) owns a contiguous tile range, channel tiles fastest
    const int per_xcd = (ntiles + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
    const int tile_end = min((xcd + 1) * per_xcd, ntiles);
    const int first_tile = xcd * per_xcd + slot;
    if (first_tile >= tile_end) return;
    const int last_tile = tile_end - 1 - ((tile_end - 1 - first_tile) % slots);

    // ---- global -> LDS transfers.  Piece n of a stage (1 KiB: 16-byte chunks 64 n .. 64 n + 63) is moved by wave n % NW in its
    // slot n / NW.  Pieces below XT are token rows, the rest channel rows; six pieces make one 128-row block of the operand format,
    // where the units of a block lie RB_BYTES apart.
    const uint32_t lane_off = (uint32_t)lane * 16;
    const int xblocks = (M + RB - 1) / RB, wblocks = (N + RB - 1) / RB;
    const uint8_t *src[LPW];                                    // wave-uniform: unit 0 of this wave's pieces of the tile under the load cursor
    int ld_tile = first_tile, ld_unit = 0, ld_stage = 0;
    auto set_tile_pointers = [&](int t) {
        const int tm = t / tiles_n, tn = t % tiles_n;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int n = i * C::NW + wave;
            const bool is_x = n < C::XT;
            const int m = is_x ? n : n - C::XT;
            // a block past the operand's end: re-read the last one (results unused)
            const int blk = min((is_x ? tm * (C::BM / RB) : tn * (C::BN / RB)) + m / RB_PIECES, (is_x ? xblocks : wblocks) - 1);
            src[i] = (is_x ? Xf : Wf) + (size_t)blk * units * RB_BYTES + (m % RB_PIECES) * 1024;
        }
    };
    auto issue_transfer = [&](auto i_c) {
        constexpr int i = decltype(i_c)::value;
        const uint32_t dst = lds0 + ld_stage * C::STAGE_BYTES + (i * C::NW + wave) * 1024;
        if constexpr ((i + 1) * C::NW <= C::NT) {
            e_dma16(lane_off, src[i] + (size_t)ld_unit * RB_BYTES, dst);
        } else {
            if (i * C::NW + wave < C::NT) e_dma16(lane_off, src[i] + (size_t)ld_unit * RB_BYTES, dst);     // wave-uniform
        }
    };
    auto advance_cursor = [&]() {
        ld_stage = (ld_stage + 1 == STAGES) ? 0 : ld_stage + 1;
        if (++ld_unit == units) {
            ld_unit = 0;
            ld_tile = min(ld_tile + slots, last_tile);          // past the last tile: re-read it (never used), keeps the stream uniform
            set_tile_pointers(ld_tile);
        }
    };
    auto issue_unit = [&]() {
        e_static_for<LPW>([&](auto i_c) { issue_transfer(i_c); });
        advance_cursor();
    };
    auto issue_scales = [&](int t, int sb) {
        const int tm = t / tiles_n, tn = t % tiles_n;
        const uint32_t dst = lds0 + STAGES * C::STAGE_BYTES + sb * C::SC_BYTES;
#pragma unroll
        for (int g = 0; g < C::SC_GROUPS; ++g) {
            if (g % C::NW != wave) continue;
            if (g < C::BM / 64) {
                e_dma4(sx + min(tm * C::BM + g * 64 + lane, M - 1), dst + g * 256);
            } else if (g < C::BM / 64 + C::BN / 64) {
                const int h = g - C::BM / 64;
                e_dma4(sw + min(tn * C::BN + h * 64 + lane, N - 1), dst + C::BM * 4 + h * 256);
            } else if (g < C::SC_SYM_GROUPS) {
                if (bias != nullptr) {
                    const int h = g - C::BM / 64 - C::BN / 64;      // 64 dwords = 128 bf16 values
                    e_dma4(reinterpret_cast<const uint32_t *>(bias) + min(tn * (C::BN / 2) + h * 64 + lane, N / 2 - 1),
                           dst + C::BM * 4 + C::BN * 4 + h * 256);
                }
            } else if (g < C::SC_SYM_GROUPS + C::BM / 64) {
                const int h = g - C::SC_SYM_GROUPS;
                e_dma4(xzero + min(tm * C::BM + h * 64 + lane, M - 1), dst + C::SC_SYM_BYTES + h * 256);
            } else {
                const int h = g - C::SC_SYM_GROUPS - C::BM / 64;
                e_dma4(wsum + min(tn * C::BN + h * 64 + lane, N - 1), dst + C::SC_SYM_BYTES + C::BM * 4 + h * 256);
            }
        }
    };

    // ---- fragments: [buffer][W sub-tiles, then X sub-tiles]; dwords 0..3 from the 16-byte read, 4..5 from the 8-byte read
    v16f acc[TN][TM];
    v8i F[2][NF];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int f = 0; f < NF; ++f) { F[b][f][6] = 0; F[b][f][7] = 0; }
    const int frow = lane & 31, fhalf = lane >> 5;
    const int w_row = (C::BM + wn * TN * 32 + frow) * U_BYTES, x_row = (wm * TM * 32 + frow) * U_BYTES;
    auto read_lo = [&](auto b_c, int f, int stage) {             // bytes 0..15 of the lane's blob
        constexpr int b = decltype(b_c)::value;
        const uint8_t *p = smem + stage * C::STAGE_BYTES + ((f < TN) ? w_row + f * 32 * U_BYTES : x_row + (f - TN) * 32 * U_BYTES);
        const v4i v = *reinterpret_cast<const v4i *>(p + fhalf * 16);
        F[b][f][0] = v[0]; F[b][f][1] = v[1]; F[b][f][2] = v[2]; F[b][f][3] = v[3];
    };
    auto read_hi = [&](auto b_c, int f, int stage) {             // bytes 16..23
        constexpr int b = decltype(b_c)::value;
        const uint8_t *p = smem + stage * C::STAGE_BYTES + ((f < TN) ? w_row + f * 32 * U_BYTES : x_row + (f - TN) * 32 * U_BYTES);
        const int2 v = *reinterpret_cast<const int2 *>(p + 32 + fhalf * 8);
        F[b][f][4] = v.x; F[b][f][5] = v.y;
    };
    // One unit = one K-step: NM slots of {one MFMA, a share of the side work}: the unit's transfers, and the 2 NF LDS reads
    // of the next unit's fragments (ring stage rd_stage) into the other buffer, in the order the MFMAs will want them.
    auto kstep = [&](auto buf_c, auto fresh_c, int rd_stage) {
        constexpr int BUF = decltype(buf_c)::value;
        constexpr bool FRESH = decltype(fresh_c)::value;
        const v16f zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        e_static_for<NM>([&](auto t_c) {
            constexpr int t = decltype(t_c)::value, j = t / TM, i = t % TM;
            acc[j][i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(F[BUF][j], F[BUF][TN + i], FRESH ? zero : acc[j][i], 2, 2, 0,
                                                                        UNIT_SCALE_ONE, 0, UNIT_SCALE_ONE);
            e_static_for<LPW>([&](auto n_c) {
                constexpr int n = decltype(n_c)::value;
                if constexpr ((2 * n + 1) * NM / (2 * LPW) == t) issue_transfer(n_c);
            });
            e_static_for<2 * NF>([&](auto o_c) {
                constexpr int o = decltype(o_c)::value, fo = o / 2;     // fo-th fragment in order of first use: W0, all X, other W
                constexpr int f = (fo == 0) ? 0 : (fo <= TM ? TN + fo - 1 : fo - TM);
                if constexpr (o * NM / (2 * NF) == t) {
                    if constexpr (o % 2 == 0) read_lo(std::integral_constant<int, BUF ^ 1>{}, f, rd_stage);
                    else read_hi(std::integral_constant<int, BUF ^ 1>{}, f, rd_stage);
                }
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using BT = std::true_type;
    using BF = std::false_type;

    // ---- prologue of the whole stream.  Unit q of the stream lives in ring stage q % STAGES.  Its fragments are read under unit
    // q - 1 (all waves are past them at the barrier that opens unit q), so during unit q that stage is refilled with unit
    // q + STAGES: STAGES - 1 units are in flight or landed ahead of the one being computed.
    if (bias == nullptr) {
        for (int b = 0; b < 2; ++b)
            for (int i = tid; i < C::BN / 2; i += C::THREADS)
                reinterpret_cast<uint32_t *>(sc_all + b * C::SC_BYTES + C::BM * 4 + C::BN * 4)[i] = 0u;
    }
    set_tile_pointers(first_tile);
    issue_scales(first_tile, 0);
#pragma unroll
    for (int s = 0; s < STAGES; ++s) issue_unit();
    e_wait_vmcnt<(STAGES - 1) * C::LPW_MIN>();
    __syncthreads();
#pragma unroll
    for (int f = 0; f < NF; ++f) { read_lo(I0{}, f, 0); read_hi(I0{}, f, 0); }

    const int c = lane & 31, g = lane >> 5;
    int cs = 0, sb = 0;                                   // ring stage of the unit being computed, scale buffer of the current tile
    for (int tile = first_tile; tile < tile_end; tile += slots) {
        // unit q of the stream: once at most STAGES - 2 later units of this wave are outstanding, unit q + 1 has landed for it; after
        // the barrier it has landed for every wave, and every wave has the fragments of unit q in registers: stage cs is refilled
        auto unit = [&](auto buf_c, auto fresh_c) {
            constexpr bool FRESH = decltype(fresh_c)::value;
            e_wait_vmcnt<(STAGES - 2) * C::LPW_MIN>();
            __syncthreads();
            if (FRESH && tile + slots < tile_end) {
                int tnext = tile + slots;
                asm volatile("" : "+s"(tnext));
                issue_scales(tnext, sb ^ 1);
            }
            const int ns = (cs + 1 == STAGES) ? 0 : cs + 1;
            kstep(buf_c, fresh_c, ns);
            advance_cursor();
            cs = ns;
        };
        unit(I0{}, BT{});
        for (int u = 2; u < units; u += 2) {
            unit(I1{}, BF{});
            unit(I0{}, BF{});
        }
        unit(I1{}, BF{});              // its LDS reads fetch the first fragments of the block's next tile: they live through the epilogue

        // ---- epilogue.  32x32 result layout: lane l holds column (l % 32) = token and rows 8*(r/4) + 4*(l/32) + r%4 = channels
        const int tm = tile / tiles_n, tn = tile % tiles_n;
        const int row0 = tm * C::BM + wm * TM * 32, col0 = tn * C::BN + wn * TN * 32;
        const uint8_t *sc = sc_all + sb * C::SC_BYTES;
        const float *scx = reinterpret_cast<const float *>(sc);
        const float *scw = reinterpret_cast<const float *>(sc + C::BM * 4) + wn * TN * 32 + 4 * g;
        const uint16_t *scb = reinterpret_cast<const uint16_t *>(sc + C::BM * 4 + C::BN * 4) + wn * TN * 32 + 4 * g;
        const int rows_left = M - row0, cols_left = N - col0;
        float sxm[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) sxm[i] = scx[(wm * TM + i) * 32 + c];
        const float *scz = reinterpret_cast<const float *>(sc + C::SC_SYM_BYTES);
        const float *scs = reinterpret_cast<const float *>(sc + C::SC_SYM_BYTES + C::BM * 4) + wn * TN * 32 + 4 * g;
        float rz[SHIFTED ? TM : 1];
        if constexpr (SHIFTED) {
#pragma unroll
            for (int i = 0; i < TM; ++i) rz[i] = 7.5f - scz[(wm * TM + i) * 32 + c];
        }
        {
            uint8_t *ep = smem + STAGES * C::STAGE_BYTES + 2 * C::SC_BYTES + wave * (32 * C::EP_PITCH);
            const int rd_row = lane >> 3, rd_col = lane & 7;
#pragma unroll
            for (int jp = 0; jp < TN / 2; ++jp) {
                float4 swq[2][4], bq[2][4], wsq[SHIFTED ? 2 : 1][SHIFTED ? 4 : 1];
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        swq[jj][q] = *reinterpret_cast<const float4 *>(scw + (2 * jp + jj) * 32 + 8 * q);
                        if constexpr (SHIFTED) wsq[jj][q] = *reinterpret_cast<const float4 *>(scs + (2 * jp + jj) * 32 + 8 * q);
                        const uint2 b = *reinterpret_cast<const uint2 *>(scb + (2 * jp + jj) * 32 + 8 * q);
                        bq[jj][q] = make_float4(__uint_as_float(b.x << 16), __uint_as_float(b.x & 0xFFFF0000u),
                                                __uint_as_float(b.y << 16), __uint_as_float(b.y & 0xFFFF0000u));
                    }
                const bool col_ok = rd_col * 8 < cols_left - jp * 64;
                uint16_t *yp = Y + (size_t)(row0 + rd_row) * N + col0 + jp * 64 + rd_col * 8;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    float4 scl[2][4];
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            scl[jj][q] = make_float4(swq[jj][q].x * sxm[i], swq[jj][q].y * sxm[i], swq[jj][q].z * sxm[i], swq[jj][q].w * sxm[i]);
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            float a0, a1, a2, a3;
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a0) : "a"(acc[2 * jp + jj][i][4 * q]));
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a1) : "a"(acc[2 * jp + jj][i][4 * q + 1]));
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a2) : "a"(acc[2 * jp + jj][i][4 * q + 2]));
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a3) : "a"(acc[2 * jp + jj][i][4 * q + 3]));
                            if constexpr (SHIFTED) {
                                a0 = fmaf(rz[i], wsq[jj][q].x, a0); a1 = fmaf(rz[i], wsq[jj][q].y, a1);
                                a2 = fmaf(rz[i], wsq[jj][q].z, a2); a3 = fmaf(rz[i], wsq[jj][q].w, a3);
                            }
                            const float y0 = fmaf(a0, scl[jj][q].x, bq[jj][q].x), y1 = fmaf(a1, scl[jj][q].y, bq[jj][q].y);
                            const float y2 = fmaf(a2, scl[jj][q].z, bq[jj][q].z), y3 = fmaf(a3, scl[jj][q].w, bq[jj][q].w);
                            *reinterpret_cast<uint2 *>(ep + c * C::EP_PITCH + (jj * 32 + 8 * q + 4 * g) * 2) = make_uint2(pack_bf16x2(y0, y1), pack_bf16x2(y2, y3));
                            if constexpr (DEBUG) {
                                const int m = row0 + i * 32 + c, n = col0 + (2 * jp + jj) * 32 + 8 * q + 4 * g;
                                if (m < M && n < N)
                                    *reinterpret_cast<int4 *>(acc_debug + (size_t)m * N + n) = make_int4((int)a0, (int)a1, (int)a2, (int)a3);
                            }
                        }
                    __builtin_amdgcn_sched_barrier(0);
                    lanes_exchange_fence();
                    v4i rowv[4];
#pragma unroll
                    for (int it = 0; it < 4; ++it) rowv[it] = *reinterpret_cast<const v4i *>(ep + (it * 8 + rd_row) * C::EP_PITCH + rd_col * 16);
                    if (rows_left - i * 32 >= 32 && cols_left - jp * 64 >= 64) {
#pragma unroll
                        for (int it = 0; it < 4; ++it) __builtin_nontemporal_store(rowv[it], reinterpret_cast<v4i *>(yp + (size_t)it * 8 * N));
                    } else {
#pragma unroll
                        for (int it = 0; it < 4; ++it)
                            if (col_ok && rd_row < rows_left - (i * 32 + it * 8)) __builtin_nontemporal_store(rowv[it], reinterpret_cast<v4i *>(yp + (size_t)it * 8 * N));
                    }
                    yp += (size_t)32 * N;
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        sb ^= 1;
    }
    e_wait_vmcnt<0>();      // transfers issued past the last tile must not outlive the block's LDS allocation
}

// ---------------------------------------------------------------------------------------
// packed 4-bit codes (library order, two per byte) -> E2M3 blocks.  One thread per (row, unit, half): 16 bytes in, 24 out.
__global__ __launch_bounds__(256) void codes_to_e2m3_kernel(const uint8_t *__restrict__ packed, size_t rows, int K, uint8_t *__restrict__ out,
                                                             unsigned int *__restrict__ n_unrepresentable)
{
    const size_t blobs_per_row = (size_t)K / 32;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * blobs_per_row) return;
    const size_t row = idx / blobs_per_row;
    const int b = (int)(idx - row * blobs_per_row), s = b >> 1, h = b & 1;
    const uint4 in = *reinterpret_cast<const uint4 *>(packed + row * (size_t)(K / 2) + (size_t)b * 16);
    const uint32_t w[4] = {in.x, in.y, in.z, in.w};
    // |q| -> E2M3 magnitude bits (exponent bias 1): 0, 1, 2, 3 = 2 * 1.5, 4, 5 = 4 * 1.25, 6, 7; five bits each
    constexpr uint64_t MAG = 0x00ull | (0x08ull << 5) | (0x10ull << 10) | (0x14ull << 15) | (0x18ull << 20) | (0x1Aull << 25) |
                             (0x1Cull << 30) | (0x1Eull << 35);
    uint64_t blob[3] = {0, 0, 0};
    int minus_eights = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const int n = (int)(w[i >> 3] >> (4 * (i & 7))) & 15;          // two's complement nibble
        const int neg = n >> 3;
        minus_eights += (n == 8);
        const int mag = min(neg ? 16 - n : n, 7);                      // -8 has no E2M3 value: written as -7 and counted
        const uint64_t pat = ((MAG >> (5 * mag)) & 31) | ((uint64_t)neg << 5);
        const int bit = 6 * i, wd = bit >> 6, sh = bit & 63;
        blob[wd] |= pat << sh;
        if (sh > 58) blob[wd + 1] |= pat >> (64 - sh);
    }
    uint8_t *u = out + ((row / RB) * (size_t)(K / 64) + s) * RB_BYTES + (row % RB) * U_BYTES;
    *reinterpret_cast<uint4 *>(u + h * 16) = make_uint4((uint32_t)blob[0], (uint32_t)(blob[0] >> 32), (uint32_t)blob[1], (uint32_t)(blob[1] >> 32));
    *reinterpret_cast<uint2 *>(u + 32 + h * 8) = make_uint2((uint32_t)blob[2], (uint32_t)(blob[2] >> 32));
    if (minus_eights != 0) atomicAdd(n_unrepresentable, (unsigned int)minus_eights);      // rare: the caller's signal that `out` is not faithful
}

hipError_t run_codes_to_e2m3(const uint8_t *packed, int rows, int K, uint8_t *out, unsigned int *n_unrepresentable, hipStream_t stream)
{
    const size_t n = (size_t)rows * (K / 32);
    if (n == 0) return hipSuccess;
    codes_to_e2m3_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(packed, (size_t)rows, K, out, n_unrepresentable);
    return hipGetLastError();
}

// every instantiation launched below, with the dynamic LDS it needs
#define QVGGT_E2M3_KERNELS(TM, TN, WM, WN, ST, MB)                                                                                  \
    {reinterpret_cast<const void *>(e2m3_gemm_kernel<TM, TN, WM, WN, ST, MB, false, false>), E2m3Cfg<TM, TN, WM, WN, ST, false>::LDS_BYTES}, \
    {reinterpret_cast<const void *>(e2m3_gemm_kernel<TM, TN, WM, WN, ST, MB, true, false>), E2m3Cfg<TM, TN, WM, WN, ST, false>::LDS_BYTES},  \
    {reinterpret_cast<const void *>(e2m3_gemm_kernel<TM, TN, WM, WN, ST, MB, false, true>), E2m3Cfg<TM, TN, WM, WN, ST, true>::LDS_BYTES}
static const LdsKernel e2m3_lds_kernel_list[] = {QVGGT_E2M3_KERNELS(4, 4, 2, 2, 5, 1), QVGGT_E2M3_KERNELS(2, 2, 2, 2, 4, 2)};
#undef QVGGT_E2M3_KERNELS
static const LdsKernels e2m3_lds_kernels(e2m3_lds_kernel_list);

template <int TM, int TN, int WM, int WN, int STAGES, int MINB, bool SHIFTED = false>
static hipError_t launch_e2m3(const uint8_t *Xf, const float *sx, const uint8_t *Wf, const float *sw, const void *bias,
                              int M, int N, int K, void *Y, int32_t *acc_debug, hipStream_t stream,
                              const float *xzero = nullptr, const float *wsum = nullptr)
{
    using C = E2m3Cfg<TM, TN, WM, WN, STAGES, SHIFTED>;
    const bool debug = acc_debug != nullptr;
    auto kern = e2m3_gemm_kernel<TM, TN, WM, WN, STAGES, MINB, false, SHIFTED>;
    if constexpr (!SHIFTED) {
        if (debug) kern = e2m3_gemm_kernel<TM, TN, WM, WN, STAGES, MINB, true, false>;
    } else {
        if (debug) return hipErrorInvalidValue;      // the corrected sum is never an integer register: no dump
    }
    hipError_t e = prepare_device();                 // the kernel's dynamic-LDS limit on this device (see e2m3_lds_kernels above)
    if (e != hipSuccess) return e;
    const int tiles_m = (M + C::BM - 1) / C::BM, tiles_n = (N + C::BN - 1) / C::BN;
    const int ntiles = tiles_m * tiles_n;
    int grid = 256 * MINB;
    if (grid > (ntiles + 7) / 8 * 8) grid = (ntiles + 7) / 8 * 8;
    kern<<<grid, C::THREADS, C::LDS_BYTES, stream>>>(Xf, sx, Wf, sw, reinterpret_cast<const uint16_t *>(bias), M, N, K,
                                                     reinterpret_cast<uint16_t *>(Y), acc_debug, tiles_m, tiles_n, xzero, wsum);
    return hipGetLastError();
}

// Which tile shape runs where.  Both configurations work in rounds (256 big tiles, or 512 small ones: two blocks per compute
// unit), and a last round that is mostly empty costs as much as a full one.  A round of small tiles does half the work of a round
// of big ones and measured 0.50 - 0.54 of its duration at K = 1024 and 0.6 - 0.75 at K = 4096.  Three plans are priced in
// hundredths of a big round: everything big, everything small, or the token rows that fill whole big rounds through the big kernel
// and the rest through the small one in a second launch on the same stream (rows are independent; the two launches write disjoint
// rows of Y, and row offsets that are multiples of 256 are whole 128-row blocks of the operand format).  The split has to win by
// 3 % to be taken.  Measured: 32976 x 4096 -> 1024 (2.02 big rounds) 85.5 -> 78.3 us; at K = 1024 the same token count is left as it
// was (a split that ignored the launch cost made 32976 x 1024 -> 1024 11 % slower), and so is 137400 x 4096 -> 1024 (8.4 rounds).
template <class Big, class Small>
static hipError_t e2m3_by_rounds(int M, int N, int K, Big &&big, Small &&small)
{
    const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
    // the second launch costs about 6 us whatever the shape; a big round takes about 4.7 + 6.7 K / 1024 us (11 us at K = 1024, 31 at 4096)
    const long long small_unit = (K <= 2048 ? 55 : 70), launch_cost = 600000 / (4700 + 6700LL * K / 1024);
    const long long big_tiles = (long long)tiles_m * tiles_n;
    const long long big_cost = (big_tiles + 255) / 256 * 100;
    const long long small_cost = (((long long)((M + 127) / 128) * ((N + 127) / 128) + 511) / 512) * small_unit;
    const long long whole_cost = small_cost < big_cost ? small_cost : big_cost;
    const int main_tile_rows = (int)std::min<long long>(tiles_m, big_tiles / 256 * 256 / tiles_n);
    if (main_tile_rows > 0 && main_tile_rows < tiles_m) {
        const int rows_main = main_tile_rows * 256, rows_rem = M - rows_main;
        const long long main_cost = ((long long)main_tile_rows * tiles_n + 255) / 256 * 100;
        const long long rem_cost = (((long long)((rows_rem + 127) / 128) * ((N + 127) / 128) + 511) / 512) * small_unit;
        if ((main_cost + rem_cost + launch_cost) * 100 < whole_cost * 97) {
            const hipError_t e = big(0, rows_main);
            if (e != hipSuccess) return e;
            return small(rows_main, rows_rem);
        }
    }
    return small_cost < big_cost ? small(0, M) : big(0, M);
}

// E2M3 blocks of both operands -> Y.
hipError_t run_e2m3_gemm(const uint8_t *Xf, const float *sx, const uint8_t *Wf, const float *sw, const void *bias, int M, int N,
                         int K, void *Y, int32_t *acc_debug, hipStream_t stream)
{
    if (M <= 0) return hipSuccess;
    const size_t KB = (size_t)K / 4 * 3;                  // bytes per row: row0 below is a multiple of 256, i.e. whole 128-row blocks
    auto big = [&](int row0, int rows) {
        return launch_e2m3<4, 4, 2, 2, 5, 1>(Xf + (size_t)row0 * KB, sx + row0, Wf, sw, bias, rows, N, K,
                                             static_cast<uint16_t *>(Y) + (size_t)row0 * N,
                                             acc_debug ? acc_debug + (size_t)row0 * N : nullptr, stream);
    };
    auto small = [&](int row0, int rows) {
        return launch_e2m3<2, 2, 2, 2, 4, 2>(Xf + (size_t)row0 * KB, sx + row0, Wf, sw, bias, rows, N, K,
                                             static_cast<uint16_t *>(Y) + (size_t)row0 * N,
                                             acc_debug ? acc_debug + (size_t)row0 * N : nullptr, stream);
    };
    return e2m3_by_rounds(M, N, K, big, small);
}

// Activations as u - 7.5 with a zero point per token (xzero), weights as before, wsum their code sums per channel.
hipError_t run_e2m3_gemm_shifted(const uint8_t *Xf, const float *sx, const float *xzero, const uint8_t *Wf, const float *sw,
                                 const float *wsum, const void *bias, int M, int N, int K, void *Y, hipStream_t stream)
{
    if (M <= 0) return hipSuccess;
    const size_t KB = (size_t)K / 4 * 3;
    auto big = [&](int row0, int rows) {
        return launch_e2m3<4, 4, 2, 2, 5, 1, true>(Xf + (size_t)row0 * KB, sx + row0, Wf, sw, bias, rows, N, K,
                                                   static_cast<uint16_t *>(Y) + (size_t)row0 * N, nullptr, stream, xzero + row0, wsum);
    };
    auto small = [&](int row0, int rows) {
        return launch_e2m3<2, 2, 2, 2, 4, 2, true>(Xf + (size_t)row0 * KB, sx + row0, Wf, sw, bias, rows, N, K,
                                                   static_cast<uint16_t *>(Y) + (size_t)row0 * N, nullptr, stream, xzero + row0, wsum);
    };
    return e2m3_by_rounds(M, N, K, big, small);
}

}  // namespace qvggt
