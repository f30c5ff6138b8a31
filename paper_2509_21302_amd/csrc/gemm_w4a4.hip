// Online kernel 2: int4 x int4 GEMM with int32 accumulation on the int8 matrix cores and a
// fused dequantise + bias epilogue (paper Sec. 3.2, granularity paragraph: the scales are
// constant along the summed dimension, so the sum stays in integers and is rescaled once).
//
//   acc[t, o] = sum_j Xq[t, j] * Wq[o, j]
//   Y[t, o]   = bf16( acc[t, o] * sx[t] * sw[o] + bias[o] )
//
// Data movement.  A block owns a tile of BM tokens x BN channels and walks over many such
// tiles (persistent grid).  The packed codes of both operands travel from global memory
// straight into LDS (global_load_lds_dwordx4: no staging registers, no LDS store
// instructions) in K-tiles of 64 bytes = 128 codes per row, through a ring of STAGES
// buffers; the K-tiles of successive output tiles form one continuous stream, so the first
// K-tiles of the next output tile are in flight while the current one finishes.
//
// LDS layout of a stage: rows of 64 bytes (BM token rows, then BN channel rows); the four
// 16-byte chunks of a row are XOR-swizzled with bits 2..3 of the row index.  The transfer
// writes 1 KiB contiguous per wavefront instruction (16 rows); the swizzle is applied on the
// global side (which chunk a lane fetches).  A fragment read is one ds_read_b128 per lane:
// lane (row = lane % 32, half = lane / 32) takes chunk 2*pair + half of its row, i.e. its 8
// bytes of K-step 2*pair and its 8 bytes of K-step 2*pair + 1.  Any 16 consecutive rows hit the
// 16 distinct 16-byte groups of the 64 LDS banks, so these reads are conflict free.  The order in
// which codes meet inside a K-step is the same for both operands, which is all a dot
// product needs.
//
// Arithmetic.  A wavefront expands packed bytes to int8 in registers right before the MFMA:
// each code is kept in the HIGH nibble of its byte (v & 0xF0F0F0F0 for the odd codes,
// (v << 4) & 0xF0F0F0F0 for the even ones), i.e. as 16 * code with the sign in place, so no
// sign extension is needed.  Both operands are expanded the same way, hence the accumulator
// is exactly 256 * acc (|256 * acc| <= 256 * 64 * 8192 = 2^27) and the factor is removed
// exactly afterwards.  The weights are the MFMA row operand and the activations its column
// operand, so a lane ends up with 4 consecutive output channels of one token.
//
// Epilogue.  Accumulators stay in AGPRs; each 32x64 piece is scaled, rounded to bf16 and turned into rows through a
// small wave-private LDS tile, so that every store instruction writes whole 128-byte lines.  They are streaming
// (non-temporal) stores: Y is not read again here, and kept out of L2 it leaves the weights resident there.
//
// Schedule.  A K-step of a wavefront is TM*TN MFMAs (32x32x32 int8); the LDS reads of the
// next pair of K-steps and the expansion of the next K-step's fragments are dealt out one
// piece per MFMA, fenced so that the compiler keeps the interleave: the vector ALU and LDS
// work runs in the shadow of the matrix pipe.
#include "qvggt_common.h"

#include <algorithm>
#include <cstdlib>
#include <type_traits>
#include <utility>

namespace qvggt {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

namespace {

constexpr int KT_BYTES = 64;       // packed bytes per row per K-tile: 128 codes = 4 MFMA K-steps = 2 pairs

// TM x TN: 32x32 sub-tiles per wave along tokens / channels; WM x WN: waves per block; STAGES: LDS ring depth
// ASYM: the per-tile scale area also carries the tokens' zero points and the channels' weight code sums
template <int TM, int TN, int WM, int WN, int STAGES, bool ASYM = false>
struct StreamCfg {
    static constexpr int NW = WM * WN, THREADS = NW * 64;
    static constexpr int BM = WM * TM * 32, BN = WN * TN * 32, ROWS = BM + BN;
    static constexpr int STAGE_BYTES = ROWS * KT_BYTES;
    static constexpr int GROUPS = ROWS / 16;            // 16-row groups: one wave-wide transfer instruction each
    static constexpr int LPW = GROUPS / NW;             // transfers per wave per K-tile
    static constexpr int NM = TM * TN, NF = TM + TN;
    static constexpr int SC_SYM_BYTES = BM * 4 + BN * 4 + BN * 2;   // per tile: sx f32, sw f32, bias bf16 (as in memory)
    static constexpr int SC_SYM_GROUPS = BM / 64 + BN / 64 + BN / 128;
    static constexpr int SC_BYTES = SC_SYM_BYTES + (ASYM ? BM * 4 + BN * 4 : 0);        // then zero points f32, code sums f32
    static constexpr int SC_GROUPS = SC_SYM_GROUPS + (ASYM ? BM / 64 + BN / 64 : 0);
    static constexpr int EP_PITCH = 128 + 16;           // bytes per token row of a wave's epilogue staging tile (64 channels + pad)
    static constexpr int EP_BYTES = NW * 32 * EP_PITCH;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES + 2 * SC_BYTES + EP_BYTES;
    static_assert(TN % 2 == 0, "the epilogue handles channel sub-tiles in pairs");
    static_assert(GROUPS % NW == 0, "16-row groups do not divide among the waves");
    static_assert(BM % 128 == 0 && BN % 128 == 0, "scale transfers assume multiples of 128");
    static_assert(STAGES >= 3, "ring needs one stage being read, one landed, one in flight");
};

// one packed dword (8 codes) -> two dwords of int8: codes 1,3,5,7 and codes 0,2,4,6, each as 16 * code
#define QVGGT_EXPAND_HALF(p, dst, k)                                   \
    do {                                                               \
        const uint32_t p_ = (uint32_t)(p);                             \
        (dst)[(k)] = (int)(p_ & 0xF0F0F0F0u);                          \
        (dst)[(k) + 1] = (int)((p_ << 4) & 0xF0F0F0F0u);               \
    } while (0)

// M0 carries the LDS base of these transfers.  Every transfer sets it itself and names it as clobbered, so nothing depends on what
// the compiler does with that register between two of them.
// 4 bytes per lane from global memory to LDS: lane l writes lds_base + 4 * l
__device__ inline void dma4(const void *src, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" ::"v"(src), "s"(lds_base) : "memory", "m0");
}
// 16 bytes per lane: lane l writes lds_base + OFF + 16 * l.  The instruction offset of such a transfer moves the LDS address and
// the global address alike: with one LDS base, transfers to different places of a stage differ only in OFF (the lane's global
// offset is pre-compensated by -OFF).  The global address is a wave-uniform 64-bit base (scalar registers) plus a 32-bit offset
// per lane: moving along K only touches the scalar base, no vector ALU work.
template <int OFF>
__device__ inline void dma16(uint32_t lane_off, const void *base, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 offset:%3" ::"v"(lane_off), "s"(base), "s"(lds_base), "n"(OFF) : "memory", "m0");
}
template <class F, int... Is>
__device__ inline void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <int N, class F>
__device__ inline void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}
template <int N>
__device__ inline void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

}  // namespace

// CB: bits a stored code occupies: 4 (two codes per byte, expanded in registers) or 8 (int8 codes, fed to the MFMA as read)
// ASYM: activations carry affine codes u with a zero point per token, stored as u - 8 (Xq) and zp (xzero); the epilogue adds
// (8 - zp[t]) * wsum[o] (wsum[o] = sum_j qw[o, j], exact in fp32) to the accumulator before the scales
// BLK (int8 codes): the operands are "int8 blocks": rows grouped in blocks of 128 with the K-tiles outermost, K-tile kt of row r at
// ((r / 128) * (K / 64) + kt) * 8192 + (r % 128) * 64, its four 16-byte chunks already in the swizzled order of the LDS stage, so
// that what a wave fetches of a K-tile is 8 KiB (4 KiB in the small configuration) contiguous in memory
template <int TM, int TN, int WM, int WN, int STAGES, int MINB, int CB, bool DEBUG, bool ASYM = false, bool BLK = false>
__global__ __launch_bounds__(WM * WN * 64, MINB) __attribute__((amdgpu_waves_per_eu(WM * WN * MINB / 4, WM * WN * MINB / 4))) void w4a4_gemm_kernel(
    const uint8_t *__restrict__ Xq, const float *__restrict__ sx, const uint8_t *__restrict__ Wq,
    const float *__restrict__ sw, const uint16_t *__restrict__ bias, int M, int N, int K,
    uint16_t *__restrict__ Y, int32_t *__restrict__ acc_debug, int tiles_m, int tiles_n,
    const float *__restrict__ xzero = nullptr, const float *__restrict__ wsum = nullptr)
{
    using C = StreamCfg<TM, TN, WM, WN, STAGES, ASYM>;
    constexpr int NM = C::NM, NF = C::NF, LPW = C::LPW;
    constexpr int DMA_SHIFT = (LPW > 4) ? 4096 : 0;             // keeps the transfers' instruction offsets inside [-4096, 4095]
    static_assert(LPW <= 8, "instruction offsets of a wave's transfers must fit 13 signed bits");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    uint8_t *sc_all = smem + STAGES * C::STAGE_BYTES;           // two buffers of SC_BYTES
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;            // LDS byte address of the dynamic segment

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    static_assert(CB == 4 || CB == 8, "codes are stored in 4 or 8 bits");
    static_assert(!BLK || CB == 8, "the blocked operand format holds int8 codes");
    constexpr int KSTEPS = (CB == 4) ? 4 : 2;                   // MFMA K-steps (32 codes each) in a K-tile of 64 bytes per row
    const int KB = (CB == 4) ? (K >> 1) : K;                    // bytes per row of codes
    const int ktiles = KB / KT_BYTES;
    const int ntiles = tiles_m * tiles_n;

    // Tile assignment: workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  XCD x owns the
    // contiguous tile range [x * per_xcd, (x + 1) * per_xcd) (channel tiles fastest), its blocks take them in turn.
    const int per_xcd = (ntiles + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
    const int tile_end = min((xcd + 1) * per_xcd, ntiles);
    const int first_tile = xcd * per_xcd + slot;
    if (first_tile >= tile_end) return;
    const int last_tile = tile_end - 1 - ((tile_end - 1 - first_tile) % slots);   // this block's last tile

    // ---- global -> LDS transfers.  Lane l of a transfer covers row l / 4 of a 16-row group and lands in 16-byte
    // slot l % 4 of that row; it fetches the chunk that the swizzle puts there.
    const int t_row = lane >> 2;
    const int t_chunk = (lane & 3) ^ ((t_row >> 2) & 3);
    // A wave's LPW groups lie in one operand (X rows come first in a stage), so all its transfers share one base.
    static_assert((C::BM / 16) % LPW == 0, "a wave's 16-row groups must not straddle the two operands");
    constexpr uint32_t BASE_SHIFT = 4096;                       // keeps the pre-compensated lane offsets non-negative
    const bool loads_x = wave * LPW * 16 < C::BM;
    uint32_t lane_off[LPW];
    const uint8_t *tile_base;                                   // wave-uniform: row 0 of the operand's tile, minus BASE_SHIFT
    int ld_tile = first_tile, ld_kt = 0, ld_stage = 0;
    static_assert(!BLK || 8192 % (LPW * 1024) == 0, "a wave's transfers of a K-tile must lie inside one 128-row block");
    if constexpr (BLK) {
#pragma unroll
        for (int i = 0; i < LPW; ++i) lane_off[i] = (i * 64 + lane) * 16 + BASE_SHIFT - (i * 1024 - DMA_SHIFT);
    }
    auto set_tile_pointers = [&](int t) {
        const int tm = t / tiles_n, tn = t % tiles_n;
        const int row0 = loads_x ? tm * C::BM : tn * C::BN;     // first row of the tile in its operand
        if constexpr (BLK) {
            const int row = row0 + wave * LPW * 16 - (loads_x ? 0 : C::BM);          // first row of this wave's share
            const int blk = min(row / 128, ((loads_x ? M : N) + 127) / 128 - 1);        // past the end: re-read the last block (unused)
            tile_base = (loads_x ? Xq : Wq) + (size_t)blk * ktiles * 8192 + (row % 128) * KT_BYTES - BASE_SHIFT;
            return;
        }
        const int last = (loads_x ? M : N) - 1 - row0;          // last existing row, relative to row0 (>= 0)
        tile_base = (loads_x ? Xq : Wq) + (size_t)row0 * KB - BASE_SHIFT;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int r = (wave * LPW + i) * 16 + t_row - (loads_x ? 0 : C::BM);   // row inside the operand's tile
            lane_off[i] = (uint32_t)min(r, last) * (uint32_t)KB + t_chunk * 16 + BASE_SHIFT - (i * 1024 - DMA_SHIFT);
        }
    };
    // The K-tile under the load cursor goes to ring stage ld_stage, one transfer instruction at a time (a wave that issues
    // them back to back stalls on each: they are dealt out between MFMAs instead); then the cursor moves on, across
    // output tiles (past this block's last tile it re-reads that tile: never used, keeps the transfers in flight uniform).
    auto issue_transfer = [&](auto i_c) {
        constexpr int i = decltype(i_c)::value;
        const uint8_t *base = tile_base + (BLK ? (size_t)ld_kt * 8192 : (size_t)ld_kt * KT_BYTES);
        // the wave's LPW KiB of a stage are contiguous; the LDS base points DMA_SHIFT into them
        dma16<i * 1024 - DMA_SHIFT>(lane_off[i], base, lds0 + ld_stage * C::STAGE_BYTES + wave * LPW * 1024 + DMA_SHIFT);
    };
    auto advance_cursor = [&]() {
        ld_stage = (ld_stage + 1 == STAGES) ? 0 : ld_stage + 1;
        if (++ld_kt == ktiles) {
            ld_kt = 0;
            ld_tile = min(ld_tile + slots, last_tile);
            set_tile_pointers(ld_tile);
        }
    };
    auto issue_ktile = [&]() {
        static_for<LPW>([&](auto i_c) { issue_transfer(i_c); });
        advance_cursor();
    };
    // per-tile scales to LDS buffer sb, as they are in memory: sx of the tile's tokens, sw and bias of its channels
    auto issue_scales = [&](int t, int sb) {
        const int tm = t / tiles_n, tn = t % tiles_n;
        const uint32_t dst = lds0 + STAGES * C::STAGE_BYTES + sb * C::SC_BYTES;
#pragma unroll
        for (int g = 0; g < C::SC_GROUPS; ++g) {
            if (g % C::NW != wave) continue;
            if (g < C::BM / 64) {
                dma4(sx + min(tm * C::BM + g * 64 + lane, M - 1), dst + g * 256);
            } else if (g < C::BM / 64 + C::BN / 64) {
                const int h = g - C::BM / 64;
                dma4(sw + min(tn * C::BN + h * 64 + lane, N - 1), dst + C::BM * 4 + h * 256);
            } else if (g < C::SC_SYM_GROUPS) {
                if (bias != nullptr) {
                    const int h = g - C::BM / 64 - C::BN / 64;      // 64 dwords = 128 bf16 values
                    dma4(reinterpret_cast<const uint32_t *>(bias) + min(tn * (C::BN / 2) + h * 64 + lane, N / 2 - 1),
                         dst + C::BM * 4 + C::BN * 4 + h * 256);
                }
            } else if (g < C::SC_SYM_GROUPS + C::BM / 64) {
                const int h = g - C::SC_SYM_GROUPS;
                dma4(xzero + min(tm * C::BM + h * 64 + lane, M - 1), dst + C::SC_SYM_BYTES + h * 256);
            } else {
                const int h = g - C::SC_SYM_GROUPS - C::BM / 64;
                dma4(wsum + min(tn * C::BN + h * 64 + lane, N - 1), dst + C::SC_SYM_BYTES + C::BM * 4 + h * 256);
            }
        }
    };

    // ---- fragments
    v16i acc[TN][TM];   // [channel sub-tile j][token sub-tile i]
    v4i raw[NF];        // packed fragments of a pair of K-steps: W sub-tiles, then X sub-tiles
    v4i F[2][NF];       // expanded fragments of one K-step: [K-step parity][W sub-tiles, then X sub-tiles]
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fsw = (frow >> 2) & 3;
    // byte offsets inside a stage of this lane's chunk of pair 0; pair 1 is the same with chunk bit 1 (byte bit 5) flipped
    const int w_off = (C::BM + wn * TN * 32 + frow) * KT_BYTES + ((fhalf ^ fsw) << 4);
    const int x_off = (wm * TM * 32 + frow) * KT_BYTES + ((fhalf ^ fsw) << 4);
    auto read_frag = [&](int f, int stage, int pair) {
        const int off = ((f < TN) ? w_off : x_off) ^ (pair << 5);
        raw[f] = *reinterpret_cast<const v4i *>(smem + stage * C::STAGE_BYTES + off + ((f < TN) ? f : f - TN) * 32 * KT_BYTES);
    };
    // One K-step: NM slots of {one MFMA, a share of the side work}.  The side work is the expansion of the NEXT K-step's
    // fragments, a dword (3 ALU ops) at a time, evenly over the slots:
    //   PAR == 0 (first K-step of a pair):  raw[f].zw -> F[1][f].  Once both dwords of raw[f] are used it is dead, and the
    //             read of the next pair's fragment f (ring stage rd_stage, pair rd_pair) is issued into it in the next slot;
    //   PAR == 1 (second K-step of a pair): raw[f].xy -> F[0][f]; slot 0 issues the reads that did not fit into the step before.
    // So a fragment's LDS read is issued most of a K-step before its first use, and reads are spread over the K-step.
    auto kstep = [&](auto step_c, auto fresh_c, int rd_stage, int rd_pair) {
        constexpr int STEP = decltype(step_c)::value, PAR = STEP & 1;   // STEP: K-step inside the K-tile
        constexpr bool FRESH = decltype(fresh_c)::value;
        const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        static_for<NM>([&](auto t_c) {
            constexpr int t = decltype(t_c)::value, j = t / TM, i = t % TM;
            acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(F[PAR][j], F[PAR][TN + i], FRESH ? zero : acc[j][i], 0, 0, 0);
            // this K-tile's share of the global -> LDS transfers: transfer n goes out in slot (2n + 1) * KSTEPS * NM / (2 * LPW) of the K-tile
            static_for<LPW>([&](auto n_c) {
                constexpr int n = decltype(n_c)::value;
                if constexpr ((2 * n + 1) * KSTEPS * NM / (2 * LPW) == STEP * NM + t) issue_transfer(n_c);
            });
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                const int done = ((2 * f + 2) * NM + 2 * NF - 1) / (2 * NF) - 1;   // slot of the PAR == 0 step that uses raw[f] last
                if (PAR == 0 ? (done + 1 == t) : (t == 0 && done + 1 >= NM)) read_frag(f, rd_stage, rd_pair);
            }
#pragma unroll
            for (int h = t * 2 * NF / NM; h < (t + 1) * 2 * NF / NM; ++h) {
                if (PAR == 0) QVGGT_EXPAND_HALF(raw[h >> 1][2 + (h & 1)], F[1][h >> 1], 2 * (h & 1));
                else QVGGT_EXPAND_HALF(raw[h >> 1][h & 1], F[0][h >> 1], 2 * (h & 1));
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // One K-step on int8 codes: a lane's 16 bytes of a fragment are the MFMA operand as they are, so F[STEP] is filled
    // straight from LDS.  While K-step STEP runs on F[STEP], the fragments of the next K-step (ring stage rd_stage, K-step
    // rd_step of that K-tile) are read into F[STEP ^ 1], one every NM / NF slots, in the order the MFMAs will want them.
    auto kstep8 = [&](auto step_c, auto fresh_c, int rd_stage, int rd_step) {
        constexpr int STEP = decltype(step_c)::value;
        constexpr bool FRESH = decltype(fresh_c)::value;
        const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        static_for<NM>([&](auto t_c) {
            constexpr int t = decltype(t_c)::value, j = t / TM, i = t % TM;
            acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(F[STEP][j], F[STEP][TN + i], FRESH ? zero : acc[j][i], 0, 0, 0);
            static_for<LPW>([&](auto n_c) {
                constexpr int n = decltype(n_c)::value;
                if constexpr ((2 * n + 1) * KSTEPS * NM / (2 * LPW) == STEP * NM + t) issue_transfer(n_c);
            });
            static_for<NF>([&](auto o_c) {
                constexpr int o = decltype(o_c)::value;                  // o-th read: W0, all X, then the other W
                constexpr int f = (o == 0) ? 0 : (o <= TM ? TN + o - 1 : o - TM);
                if constexpr (o * NM / NF == t) {
                    const int off = ((f < TN) ? w_off : x_off) ^ (rd_step << 5);
                    F[STEP ^ 1][f] = *reinterpret_cast<const v4i *>(smem + rd_stage * C::STAGE_BYTES + off + ((f < TN) ? f : f - TN) * 32 * KT_BYTES);
                }
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
    using BT = std::true_type;
    using BF = std::false_type;

    // ---- prologue of the whole stream
    if (bias == nullptr) {      // no bias: both bias areas stay zero for the whole kernel
        for (int b = 0; b < 2; ++b)
            for (int i = tid; i < C::BN / 2; i += C::THREADS)
                reinterpret_cast<uint32_t *>(sc_all + b * C::SC_BYTES + C::BM * 4 + C::BN * 4)[i] = 0u;
    }
    set_tile_pointers(first_tile);
    issue_scales(first_tile, 0);
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue_ktile();
    wait_vmcnt<(STAGES - 2) * LPW>();
    __syncthreads();
#pragma unroll
    for (int f = 0; f < NF; ++f) read_frag(f, 0, 0);
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        if constexpr (CB == 4) {
            QVGGT_EXPAND_HALF(raw[f][0], F[0][f], 0);
            QVGGT_EXPAND_HALF(raw[f][1], F[0][f], 2);
        } else {
            F[0][f] = raw[f];
        }
    }

    const int c = lane & 31, g = lane >> 5;

    int cs = 0, sb = 0;                                   // ring stage being computed on, scale buffer of the current tile
    for (int tile = first_tile; tile < tile_end; tile += slots) {
        // one K-tile of the stream: four K-steps on ring stage cs.  The first K-tile of an output tile starts the
        // accumulators from zero (FRESH) and sends for the scales of the block's next output tile.
        auto ktile = [&](auto fresh_c) {
            constexpr bool FRESH = decltype(fresh_c)::value;
            // K-tile q+1 of the stream has landed for this wave once at most (STAGES-3) later K-tiles are outstanding; after
            // the barrier it has landed for every wave, and every wave is done reading K-tile q-1, whose stage is reused.
            wait_vmcnt<(STAGES - 3) * LPW>();
            __syncthreads();
            if (FRESH && tile + slots < tile_end) {
                int tnext = tile + slots;
                asm volatile("" : "+s"(tnext));             // keeps the address arithmetic of the scale transfers inside this branch
                issue_scales(tnext, sb ^ 1);
            }
            const int ns = (cs + 1 == STAGES) ? 0 : cs + 1;
            if constexpr (CB == 4) {
                kstep(I0{}, fresh_c, cs, 1);
                kstep(I1{}, BF{}, cs, 1);
                kstep(I2{}, BF{}, ns, 0);
                kstep(I3{}, BF{}, ns, 0);
            } else {
                kstep8(I0{}, fresh_c, cs, 1);
                kstep8(I1{}, BF{}, ns, 0);
            }
            advance_cursor();
            cs = ns;
        };
        ktile(BT{});
        for (int kt = 1; kt < ktiles; ++kt) ktile(BF{});

        // ---- epilogue.  32x32 result layout: lane l holds column (l % 32) = token and rows 8*(r/4) + 4*(l/32) + r%4 = channels,
        // i.e. per register quad q four consecutive channels 8q + 4*(l/32) + 0..3.  Scale + bias + bf16 in registers.
        const int tm = tile / tiles_n, tn = tile % tiles_n;
        const int row0 = tm * C::BM + wm * TM * 32, col0 = tn * C::BN + wn * TN * 32;   // first token / channel of this wave
        const uint8_t *sc = sc_all + sb * C::SC_BYTES;
        const float *scx = reinterpret_cast<const float *>(sc);
        const float *scw = reinterpret_cast<const float *>(sc + C::BM * 4) + wn * TN * 32 + 4 * g;
        const uint16_t *scb = reinterpret_cast<const uint16_t *>(sc + C::BM * 4 + C::BN * 4) + wn * TN * 32 + 4 * g;
        const int rows_left = M - row0;                      // tokens of this wave's rows that exist
        const int cols_left = N - col0;                      // channels of this wave's columns that exist (a multiple of 16)
        float sxm[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) sxm[i] = scx[(wm * TM + i) * 32 + c] * (CB == 4 ? 1.0f / 256.0f : 1.0f);
        // affine activation codes: (8 - zp) of this lane's tokens, in the accumulator's units (256 per unit for packed codes)
        const float *scz = reinterpret_cast<const float *>(sc + C::SC_SYM_BYTES);
        const float *scs = reinterpret_cast<const float *>(sc + C::SC_SYM_BYTES + C::BM * 4) + wn * TN * 32 + 4 * g;
        float rz[ASYM ? TM : 1];
        if constexpr (ASYM) {
#pragma unroll
            for (int i = 0; i < TM; ++i) rz[i] = (8.0f - scz[(wm * TM + i) * 32 + c]) * (CB == 4 ? 256.0f : 1.0f);
        }
        {
            // A wave-private LDS tile [32 tokens][64 channels] turns the lane-per-token layout into rows, so
            // that a store instruction writes whole 128-byte lines (8 lanes x 16 bytes per token).  Whole lines can be
            // streamed past L2 (non-temporal) without write amplification, which leaves the weights resident there.
            uint8_t *ep = smem + STAGES * C::STAGE_BYTES + 2 * C::SC_BYTES + wave * (32 * C::EP_PITCH);
            const int rd_row = lane >> 3, rd_col = lane & 7;
#pragma unroll
            for (int jp = 0; jp < TN / 2; ++jp) {
                float4 swq[2][4], bq[2][4], wsq[ASYM ? 2 : 1][ASYM ? 4 : 1];
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        swq[jj][q] = *reinterpret_cast<const float4 *>(scw + (2 * jp + jj) * 32 + 8 * q);
                        if constexpr (ASYM) wsq[jj][q] = *reinterpret_cast<const float4 *>(scs + (2 * jp + jj) * 32 + 8 * q);
                        const uint2 b = *reinterpret_cast<const uint2 *>(scb + (2 * jp + jj) * 32 + 8 * q);
                        bq[jj][q] = make_float4(__uint_as_float(b.x << 16), __uint_as_float(b.x & 0xFFFF0000u),
                                                __uint_as_float(b.y << 16), __uint_as_float(b.y & 0xFFFF0000u));
                    }
                const bool col_ok = rd_col * 8 < cols_left - jp * 64;
                uint16_t *yp = Y + (size_t)(row0 + rd_row) * N + col0 + jp * 64 + rd_col * 8;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    // the token's scale folded into the channel scales once per piece: one multiply per channel instead of one per value
                    float4 sc[2][4];
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            sc[jj][q] = make_float4(swq[jj][q].x * sxm[i], swq[jj][q].y * sxm[i], swq[jj][q].z * sxm[i], swq[jj][q].w * sxm[i]);
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            int a0, a1, a2, a3;
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a0) : "a"(acc[2 * jp + jj][i][4 * q]));
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a1) : "a"(acc[2 * jp + jj][i][4 * q + 1]));
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a2) : "a"(acc[2 * jp + jj][i][4 * q + 2]));
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a3) : "a"(acc[2 * jp + jj][i][4 * q + 3]));
                            float f0 = (float)a0, f1 = (float)a1, f2 = (float)a2, f3 = (float)a3;
                            if constexpr (ASYM) {      // integers below 2^27 that are multiples of 256 (packed codes), or below 2^24: exact
                                f0 = fmaf(rz[i], wsq[jj][q].x, f0); f1 = fmaf(rz[i], wsq[jj][q].y, f1);
                                f2 = fmaf(rz[i], wsq[jj][q].z, f2); f3 = fmaf(rz[i], wsq[jj][q].w, f3);
                            }
                            const float y0 = fmaf(f0, sc[jj][q].x, bq[jj][q].x), y1 = fmaf(f1, sc[jj][q].y, bq[jj][q].y);
                            const float y2 = fmaf(f2, sc[jj][q].z, bq[jj][q].z), y3 = fmaf(f3, sc[jj][q].w, bq[jj][q].w);
                            *reinterpret_cast<uint2 *>(ep + c * C::EP_PITCH + (jj * 32 + 8 * q + 4 * g) * 2) = make_uint2(pack_bf16x2(y0, y1), pack_bf16x2(y2, y3));
                            if constexpr (DEBUG) {
                                const int m = row0 + i * 32 + c, n = col0 + (2 * jp + jj) * 32 + 8 * q + 4 * g;
                                if (m < M && n < N)
                                    *reinterpret_cast<int4 *>(acc_debug + (size_t)m * N + n) = make_int4(a0 >> (16 - 2 * CB), a1 >> (16 - 2 * CB), a2 >> (16 - 2 * CB), a3 >> (16 - 2 * CB));
                            }
                        }
                    __builtin_amdgcn_sched_barrier(0);
                    // the staging tile is private to the wave and LDS operations of a wave execute in order: no barrier instruction is
                    // needed, only the compiler has to be told that other lanes' writes are read next
                    lanes_exchange_fence();
                    // all four row groups are read before the first store: one LDS round trip per piece instead of four.  A piece
                    // that lies fully inside Y (the usual case, a wave-uniform test) stores without per-lane predicates.
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
    wait_vmcnt<0>();        // transfers issued past the last tile must not outlive the block's LDS allocation
}

// every instantiation launched below, with the dynamic LDS it needs: packed codes (plain, accumulator dump, affine), int8 codes
// row-major and in blocks (plain, accumulator dump)
#define QVGGT_GEMM_KERNELS(TM, TN, WM, WN, ST, MB)                                                                                        \
    {reinterpret_cast<const void *>(w4a4_gemm_kernel<TM, TN, WM, WN, ST, MB, 4, false, false, false>), StreamCfg<TM, TN, WM, WN, ST, false>::LDS_BYTES}, \
    {reinterpret_cast<const void *>(w4a4_gemm_kernel<TM, TN, WM, WN, ST, MB, 4, true, false, false>), StreamCfg<TM, TN, WM, WN, ST, false>::LDS_BYTES},  \
    {reinterpret_cast<const void *>(w4a4_gemm_kernel<TM, TN, WM, WN, ST, MB, 4, false, true, false>), StreamCfg<TM, TN, WM, WN, ST, true>::LDS_BYTES},   \
    {reinterpret_cast<const void *>(w4a4_gemm_kernel<TM, TN, WM, WN, ST, MB, 8, false, false, false>), StreamCfg<TM, TN, WM, WN, ST, false>::LDS_BYTES}, \
    {reinterpret_cast<const void *>(w4a4_gemm_kernel<TM, TN, WM, WN, ST, MB, 8, true, false, false>), StreamCfg<TM, TN, WM, WN, ST, false>::LDS_BYTES},  \
    {reinterpret_cast<const void *>(w4a4_gemm_kernel<TM, TN, WM, WN, ST, MB, 8, false, false, true>), StreamCfg<TM, TN, WM, WN, ST, false>::LDS_BYTES},  \
    {reinterpret_cast<const void *>(w4a4_gemm_kernel<TM, TN, WM, WN, ST, MB, 8, true, false, true>), StreamCfg<TM, TN, WM, WN, ST, false>::LDS_BYTES}
static const LdsKernel gemm_lds_kernel_list[] = {QVGGT_GEMM_KERNELS(4, 4, 2, 2, 4, 1), QVGGT_GEMM_KERNELS(2, 2, 2, 2, 3, 2)};
#undef QVGGT_GEMM_KERNELS
static const LdsKernels gemm_lds_kernels(gemm_lds_kernel_list);

template <int TM, int TN, int WM, int WN, int STAGES, int MINB, int CB, bool ASYM = false, bool BLK = false>
static hipError_t launch_gemm(const uint8_t *Xq, const float *sx, const uint8_t *Wq, const float *sw, const void *bias,
                              int M, int N, int K, void *Y, int32_t *acc_debug, hipStream_t stream,
                              const float *xzero = nullptr, const float *wsum = nullptr)
{
    using C = StreamCfg<TM, TN, WM, WN, STAGES, ASYM>;
    // the variant that also writes the raw accumulators is a separate instantiation: the production kernel carries none of it
    const bool debug = acc_debug != nullptr;
    auto kern = w4a4_gemm_kernel<TM, TN, WM, WN, STAGES, MINB, CB, false, ASYM, BLK>;
    if constexpr (!ASYM) {
        if (debug) kern = w4a4_gemm_kernel<TM, TN, WM, WN, STAGES, MINB, CB, true, false, BLK>;
    } else {
        if (debug) return hipErrorInvalidValue;      // no accumulator dump with affine codes: the corrected sum is never an integer register
    }
    hipError_t e = prepare_device();                 // the kernel's dynamic-LDS limit on this device (see gemm_lds_kernels above)
    if (e != hipSuccess) return e;
    const int tiles_m = (M + C::BM - 1) / C::BM, tiles_n = (N + C::BN - 1) / C::BN;
    const int ntiles = tiles_m * tiles_n;
    int grid = 256 * MINB;                                // MINB resident blocks on each of the 256 compute units
    if (grid > (ntiles + 7) / 8 * 8) grid = (ntiles + 7) / 8 * 8;
    kern<<<grid, C::THREADS, C::LDS_BYTES, stream>>>(Xq, sx, Wq, sw, reinterpret_cast<const uint16_t *>(bias), M, N, K,
                                                     reinterpret_cast<uint16_t *>(Y), acc_debug, tiles_m, tiles_n, xzero, wsum);
    return hipGetLastError();
}

// Which tile shape runs where.  The big configuration (256 x 256 per block, four waves of 128 x 128, one per SIMD) works in
// rounds of 256 tiles, one per compute unit; a last round that is mostly empty costs as much as a full one.  So the token rows
// that fill whole rounds go to the big kernel and the remaining rows, when they fit better there, to the small configuration
// (128 x 128 per block, two blocks per compute unit) in a second launch on the same stream.  Rows are independent, the two
// launches write disjoint rows of Y.
template <int CB, bool ASYM = false, bool BLK = false>
static hipError_t gemm_by_rounds(const uint8_t *Xq, const float *sx, const uint8_t *Wq, const float *sw, const void *bias,
                                 int M, int N, int K, void *Y, int32_t *acc_debug, hipStream_t stream,
                                 const float *xzero = nullptr, const float *wsum = nullptr)
{
    auto big = [&](int row0, int rows) {
        return launch_gemm<4, 4, 2, 2, 4, 1, CB, ASYM, BLK>(Xq + (size_t)row0 * (CB == 4 ? K / 2 : K), sx + row0, Wq, sw, bias, rows, N, K,
                                                       static_cast<uint16_t *>(Y) + (size_t)row0 * N,
                                                       acc_debug ? acc_debug + (size_t)row0 * N : nullptr, stream,
                                                       ASYM ? xzero + row0 : nullptr, wsum);
    };
    auto small = [&](int row0, int rows) {
        return launch_gemm<2, 2, 2, 2, 3, 2, CB, ASYM, BLK>(Xq + (size_t)row0 * (CB == 4 ? K / 2 : K), sx + row0, Wq, sw, bias, rows, N, K,
                                                       static_cast<uint16_t *>(Y) + (size_t)row0 * N,
                                                       acc_debug ? acc_debug + (size_t)row0 * N : nullptr, stream,
                                                       ASYM ? xzero + row0 : nullptr, wsum);
    };
    const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
    const long long big_tiles = (long long)tiles_m * tiles_n;
    // a round of small tiles takes about 0.5 - 0.7 of a round of big ones (measured at K = 1024 and 4096): 13 / 20 below
    if (big_tiles < 256) {
        // less than one round of big tiles: small tiles unless they need a second round of their own
        const long long small_rounds = ((long long)((M + 127) / 128) * ((N + 127) / 128) + 511) / 512;
        return small_rounds * 13 < 20 ? small(0, M) : big(0, M);
    }
    // whole tile rows that fit into the full rounds
    const int main_tile_rows = (int)std::min<long long>(tiles_m, big_tiles / 256 * 256 / tiles_n);
    const int rem_tile_rows = tiles_m - main_tile_rows;
    if (rem_tile_rows == 0) return big(0, M);
    const int rows_main = main_tile_rows * 256, rows_rem = M - rows_main;
    const long long rem_big_rounds = ((long long)rem_tile_rows * tiles_n + 255) / 256;
    const long long rem_small_rounds = ((long long)((rows_rem + 127) / 128) * ((N + 127) / 128) + 511) / 512;
    if (rem_small_rounds * 13 >= rem_big_rounds * 20) return big(0, M);
    hipError_t e = big(0, rows_main);
    if (e != hipSuccess) return e;
    return small(rows_main, rows_rem);
}

hipError_t run_w4a4_gemm(const uint8_t *Xq, const float *sx, const uint8_t *Wq, const float *sw,
                         const void *bias, int M, int N, int K, void *Y, int32_t *acc_debug, hipStream_t stream)
{
    if (M <= 0) return hipSuccess;
    return gemm_by_rounds<4>(Xq, sx, Wq, sw, bias, M, N, K, Y, acc_debug, stream);
}

// Packed 4-bit codes with affine activations: Xq holds u - 8, xzero the zero points, wsum the weights' code sums per channel.
hipError_t run_w4a4_gemm_asym(const uint8_t *Xq, const float *sx, const float *xzero, const uint8_t *Wq, const float *sw,
                              const float *wsum, const void *bias, int M, int N, int K, void *Y, hipStream_t stream)
{
    if (M <= 0) return hipSuccess;
    return gemm_by_rounds<4, true>(Xq, sx, Wq, sw, bias, M, N, K, Y, nullptr, stream, xzero, wsum);
}

// The same kernel on int8 codes (8- and 6-bit settings): rows of K bytes, no expansion, two K-steps per K-tile.
hipError_t run_i8_gemm(const int8_t *Xq, const float *sx, const int8_t *Wq, const float *sw, const void *bias, int M, int N,
                       int K, void *Y, int32_t *acc_debug, hipStream_t stream)
{
    if (M <= 0) return hipSuccess;
    const uint8_t *xq = reinterpret_cast<const uint8_t *>(Xq), *wq = reinterpret_cast<const uint8_t *>(Wq);
    return gemm_by_rounds<8>(xq, sx, wq, sw, bias, M, N, K, Y, acc_debug, stream);
}

// int8 codes in 128-row blocks (see the kernel): whole tile rows go to either launch, so row offsets stay whole blocks
hipError_t run_i8b_gemm(const int8_t *Xb, const float *sx, const int8_t *Wb, const float *sw, const void *bias, int M, int N,
                        int K, void *Y, int32_t *acc_debug, hipStream_t stream)
{
    if (M <= 0) return hipSuccess;
    return gemm_by_rounds<8, false, true>(reinterpret_cast<const uint8_t *>(Xb), sx, reinterpret_cast<const uint8_t *>(Wb), sw, bias,
                                          M, N, K, Y, acc_debug, stream);
}

}  // namespace qvggt
