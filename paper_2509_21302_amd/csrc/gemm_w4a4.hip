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
//
// LDS tiles are [rows][BKB bytes] with the 8-byte chunks of a row XOR-swizzled by the row
// index, which makes both the 8-byte fragment reads (16 consecutive rows, same chunk) and the
// staging writes bank-conflict free without padding.
#include "qvggt_common.h"
#include <cstdlib>

namespace qvggt {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__device__ inline v4i expand_codes(uint2 p)
{
    v4i r;
    r[0] = (int)(p.x & 0xF0F0F0F0u);
    r[1] = (int)((p.x << 4) & 0xF0F0F0F0u);
    r[2] = (int)(p.y & 0xF0F0F0F0u);
    r[3] = (int)((p.y << 4) & 0xF0F0F0F0u);
    return r;
}

// TM x TN: 32x32 sub-tiles per wave along tokens / channels; WM x WN: waves per block; BKB: packed bytes per row per K-tile
template <int TM, int TN, int WM, int WN, int BKB, int OCC>
struct GemmCfg {
    static constexpr int BM = WM * TM * 32, BN = WN * TN * 32, THREADS = WM * WN * 64;
    static constexpr int CH = BKB / 8;                 // 8-byte chunks per row
    static constexpr int RP = (BKB >= 128) ? 1 : 128 / BKB;   // rows per 128 bytes of LDS
    static constexpr int KSTEPS = BKB / 16;            // MFMA K-steps (32 codes) per K-tile
    static constexpr int TPR = BKB / 16;               // staging threads per row (16 bytes each)
    static constexpr int X_LOADS = BM * TPR / THREADS, W_LOADS = BN * TPR / THREADS;
    static constexpr int LDS_BYTES = 2 * (BM + BN) * BKB;
    static_assert(BM * TPR % THREADS == 0 && BN * TPR % THREADS == 0, "tile does not divide among the threads");
};

template <class C>
__device__ inline int swz(int row) { return (row / C::RP) % C::CH; }

// A block walks over many output tiles and treats the K-tiles of all of
// them as one stream through the LDS double buffer, so the first K-tiles of the next output
// tile are already in flight while the current tile's epilogue runs.  Two such blocks share a
// compute unit; one block's epilogue overlaps the other's MFMA loop.
// SCHED picks the instruction-interleaving hint given to the compiler for a K-step
// (2: its small-GEMM MFMA/LDS interleave, 3: one MFMA then its share of the expansion ALU ops).
template <int TM, int TN, int WM, int WN, int BKB, int OCC, int SCHED>
__global__ __launch_bounds__(WM * WN * 64, OCC) void w4a4_gemm_persistent_kernel(
    const uint8_t *__restrict__ Xq, const float *__restrict__ sx, const uint8_t *__restrict__ Wq,
    const float *__restrict__ sw, const uint16_t *__restrict__ bias, int M, int N, int K,
    uint16_t *__restrict__ Y, int32_t *__restrict__ acc_debug, int tiles_m, int tiles_n)
{
    using C = GemmCfg<TM, TN, WM, WN, BKB, OCC>;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int STAGE = (C::BM + C::BN) * BKB;       // one pipeline stage: X tile then W tile
    constexpr int KS = C::KSTEPS;
    constexpr int EP_PITCH = TN * 64 + 16;             // bytes per token row of a wave's epilogue staging tile
    constexpr int EP_BYTES = (WM * WN) * 32 * EP_PITCH;
    constexpr int SC_FLOATS = C::BM + 2 * C::BN;       // per tile: sx of its tokens, sw and bias of its channels
    uint8_t *ep_all = smem + 2 * STAGE;
    float *sc_all = reinterpret_cast<float *>(smem + 2 * STAGE + EP_BYTES);   // two buffers of SC_FLOATS

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int KB = K >> 1;             // packed bytes per row
    const int ktiles = KB / BKB;
    const int ntiles = tiles_m * tiles_n;

    // Tile assignment: workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  XCD x owns the
    // contiguous tile range [x * per_xcd, (x + 1) * per_xcd) (channel tiles fastest), its blocks take them in turn.
    const int per_xcd = (ntiles + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
    const int tile_end = min((xcd + 1) * per_xcd, ntiles);
    const int first_tile = xcd * per_xcd + slot;
    if (first_tile >= tile_end) return;

    // ---- global -> LDS staging
    const int ld_row = tid / C::TPR, ld_seg = tid % C::TPR;
    constexpr int ROWS_PER_PASS = C::THREADS / C::TPR;
    const uint8_t *gX[C::X_LOADS], *gW[C::W_LOADS];
    int oX[C::X_LOADS][2], oW[C::W_LOADS][2];          // LDS byte offsets of the two 8-byte halves
#pragma unroll
    for (int p = 0; p < C::X_LOADS; ++p) {
        const int r = ld_row + ROWS_PER_PASS * p;
        oX[p][0] = r * BKB + ((2 * ld_seg) ^ swz<C>(r)) * 8;
        oX[p][1] = r * BKB + ((2 * ld_seg + 1) ^ swz<C>(r)) * 8;
    }
#pragma unroll
    for (int p = 0; p < C::W_LOADS; ++p) {
        const int r = ld_row + ROWS_PER_PASS * p;
        oW[p][0] = C::BM * BKB + r * BKB + ((2 * ld_seg) ^ swz<C>(r)) * 8;
        oW[p][1] = C::BM * BKB + r * BKB + ((2 * ld_seg + 1) ^ swz<C>(r)) * 8;
    }
    // load cursor: runs two K-tiles ahead of the compute cursor, across output tiles
    int ld_tile = first_tile, ld_kt = 0;
    auto set_tile_pointers = [&](int t) {
        t = min(t, ntiles - 1);                         // past the end: harmless re-reads, never used
        const int tm = t / tiles_n, tn = t % tiles_n;
#pragma unroll
        for (int p = 0; p < C::X_LOADS; ++p)
            gX[p] = Xq + (size_t)min(tm * C::BM + ld_row + ROWS_PER_PASS * p, M - 1) * KB + ld_seg * 16;
#pragma unroll
        for (int p = 0; p < C::W_LOADS; ++p)
            gW[p] = Wq + (size_t)min(tn * C::BN + ld_row + ROWS_PER_PASS * p, N - 1) * KB + ld_seg * 16;
    };
    uint4 rX[C::X_LOADS], rW[C::W_LOADS];
    auto load_next = [&]() {
        const size_t off = (size_t)ld_kt * BKB;
#pragma unroll
        for (int p = 0; p < C::X_LOADS; ++p) rX[p] = *reinterpret_cast<const uint4 *>(gX[p] + off);
#pragma unroll
        for (int p = 0; p < C::W_LOADS; ++p) rW[p] = *reinterpret_cast<const uint4 *>(gW[p] + off);
        if (++ld_kt == ktiles) { ld_kt = 0; ld_tile += slots; set_tile_pointers(ld_tile < tile_end ? ld_tile : ntiles - 1); }
    };
    auto store_tile = [&](int buf) {
        uint8_t *base = smem + buf * STAGE;
#pragma unroll
        for (int p = 0; p < C::X_LOADS; ++p) {
            *reinterpret_cast<uint2 *>(base + oX[p][0]) = make_uint2(rX[p].x, rX[p].y);
            *reinterpret_cast<uint2 *>(base + oX[p][1]) = make_uint2(rX[p].z, rX[p].w);
        }
#pragma unroll
        for (int p = 0; p < C::W_LOADS; ++p) {
            *reinterpret_cast<uint2 *>(base + oW[p][0]) = make_uint2(rW[p].x, rW[p].y);
            *reinterpret_cast<uint2 *>(base + oW[p][1]) = make_uint2(rW[p].z, rW[p].w);
        }
    };
    // per-tile scales into LDS (buffer `sb`): sx of the tile's tokens, sw and bias of its channels
    auto stage_scales = [&](int t, int sb) {
        const int tm = t / tiles_n, tn = t % tiles_n;
        float *sc = sc_all + sb * SC_FLOATS;
        for (int i = tid; i < C::BM; i += C::THREADS) sc[i] = sx[min(tm * C::BM + i, M - 1)] * (1.0f / 256.0f);
        for (int i = tid; i < C::BN; i += C::THREADS) {
            const int n = min(tn * C::BN + i, N - 1);
            sc[C::BM + i] = sw[n];
            sc[C::BM + C::BN + i] = (bias != nullptr) ? __uint_as_float((uint32_t)bias[n] << 16) : 0.0f;
        }
    };

    v16i acc[TN][TM];   // [channel sub-tile j][token sub-tile i]
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fswz = swz<C>(frow);
    const int xrow_off = (wm * TM * 32 + frow) * BKB, wrow_off = C::BM * BKB + (wn * TN * 32 + frow) * BKB;
    uint2 raw_w[TN], raw_x[TM];
    v4i fw[TN], fx[TM];
    auto read_frags = [&](int buf, int ks) {
        const uint8_t *base = smem + buf * STAGE + ((2 * ks + fhalf) ^ fswz) * 8;
#pragma unroll
        for (int j = 0; j < TN; ++j) raw_w[j] = *reinterpret_cast<const uint2 *>(base + wrow_off + j * 32 * BKB);
#pragma unroll
        for (int i = 0; i < TM; ++i) raw_x[i] = *reinterpret_cast<const uint2 *>(base + xrow_off + i * 32 * BKB);
    };
    auto expand_frags = [&]() {
#pragma unroll
        for (int j = 0; j < TN; ++j) fw[j] = expand_codes(raw_w[j]);
#pragma unroll
        for (int i = 0; i < TM; ++i) fx[i] = expand_codes(raw_x[i]);
    };
    auto mfma_step = [&]() {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int i = 0; i < TM; ++i)
                acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[j], fx[i], acc[j][i], 0, 0, 0);
    };
    auto schedule_step = [&]() {
        constexpr int NM = TM * TN, NV = 6 * (TM + TN);
        if constexpr (SCHED == 2) { __builtin_amdgcn_iglp_opt(0); }
        if constexpr (SCHED == 3) {
#pragma unroll
            for (int t = 0; t < NM; ++t) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, (NV + NM - 1) / NM, 0);
            }
        }
    };

    // prologue of the whole stream
    set_tile_pointers(first_tile);
    load_next();
    stage_scales(first_tile, 0);
    store_tile(0);
    __syncthreads();
    load_next();
    read_frags(0, 0);
    expand_frags();

    const int c = lane & 31, g = lane >> 5;
    uint8_t *ep = ep_all + wave * (32 * EP_PITCH);
    constexpr int LPR = TN * 4;                           // lanes per token row when reading 16 bytes each
    constexpr int RPI = 64 / LPR;                         // token rows per read instruction
    const int rd_row = lane / LPR, rd_col = lane % LPR;

    int buf = 0, sb = 0;
    for (int tile = first_tile; tile < tile_end; tile += slots) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[j][i][r] = 0;
        for (int kt = 0; kt < ktiles; ++kt) {
#pragma unroll
            for (int ks = 0; ks < KS - 1; ++ks) {
                read_frags(buf, ks + 1);
                mfma_step();
                expand_frags();
                schedule_step();
            }
            // the K-tile held in registers goes to the other LDS buffer; after the barrier it is visible to all waves
            // and the buffer it replaces is no longer read by anyone (its last reads were issued before the previous barrier)
            store_tile(buf ^ 1);
            __syncthreads();
            load_next();
            // scales of the next output tile go to the other scale buffer: every wave has left the previous epilogue
            // (which read that buffer) once it is past the barrier above, and later barriers publish the new values
            if (kt == 0 && tile + slots < tile_end) stage_scales(tile + slots, sb ^ 1);
            // last step of this K-tile: its LDS reads already belong to the next K-tile (possibly of the next output tile)
            read_frags(buf ^ 1, 0);
            mfma_step();
            expand_frags();
            schedule_step();
            buf ^= 1;
        }

        // ---- epilogue.  32x32 result layout: lane l holds column (l % 32) = token and rows 8*(r/4) + 4*(l/32) + r%4 = channels.
        // Scale + bias + bf16 in registers, then a wave-private LDS tile [32 tokens][TN*32 channels] turns the
        // lane-per-token layout into full rows: 16-byte global stores, contiguous per token.
        const int tm = tile / tiles_n, tn = tile % tiles_n;
        const int m0 = tm * C::BM, n0 = tn * C::BN;
        const float *sc = sc_all + sb * SC_FLOATS;
        const int n_out = n0 + wn * TN * 32 + rd_col * 8;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mt = m0 + (wm * TM + i) * 32;       // first token of this sub-tile
            const float sxm = sc[(wm * TM + i) * 32 + c];
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int nl = (wn * TN + j) * 32 + 8 * q + 4 * g;     // channel inside the block tile
                    const float4 swq = *reinterpret_cast<const float4 *>(sc + C::BM + nl);
                    const float4 bq = *reinterpret_cast<const float4 *>(sc + C::BM + C::BN + nl);
                    const int a0 = acc[j][i][4 * q], a1 = acc[j][i][4 * q + 1], a2 = acc[j][i][4 * q + 2], a3 = acc[j][i][4 * q + 3];
                    const float y0 = fmaf((float)a0 * sxm, swq.x, bq.x), y1 = fmaf((float)a1 * sxm, swq.y, bq.y);
                    const float y2 = fmaf((float)a2 * sxm, swq.z, bq.z), y3 = fmaf((float)a3 * sxm, swq.w, bq.w);
                    *reinterpret_cast<uint2 *>(ep + c * EP_PITCH + (j * 32 + 8 * q + 4 * g) * 2) = make_uint2(pack_bf16x2(y0, y1), pack_bf16x2(y2, y3));
                    if (acc_debug != nullptr) {
                        const int m = mt + c, n = n0 + nl;
                        if (m < M && n < N)
                            *reinterpret_cast<int4 *>(acc_debug + (size_t)m * N + n) = make_int4(a0 >> 8, a1 >> 8, a2 >> 8, a3 >> 8);
                    }
                }
            // the staging tile is private to the wave and LDS operations of a wave execute in order: no barrier needed
#pragma unroll
            for (int it = 0; it < 32 / RPI; ++it) {
                const int tr = it * RPI + rd_row;
                const uint4 v = *reinterpret_cast<const uint4 *>(ep + tr * EP_PITCH + rd_col * 16);
                const int m = mt + tr;
                if (m < M && n_out < N) *reinterpret_cast<uint4 *>(Y + (size_t)m * N + n_out) = v;
            }
        }
        sb ^= 1;
    }
}

template <int TM, int TN, int WM, int WN, int BKB, int OCC, int SCHED>
static hipError_t launch_gemm_persistent(const uint8_t *Xq, const float *sx, const uint8_t *Wq, const float *sw, const void *bias,
                                         int M, int N, int K, void *Y, int32_t *acc_debug, hipStream_t stream)
{
    using C = GemmCfg<TM, TN, WM, WN, BKB, OCC>;
    auto kern = w4a4_gemm_persistent_kernel<TM, TN, WM, WN, BKB, OCC, SCHED>;
    constexpr int LDS = 2 * (C::BM + C::BN) * BKB + (WM * WN) * 32 * (TN * 64 + 16) + 2 * (C::BM + 2 * C::BN) * 4;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (M + C::BM - 1) / C::BM, tiles_n = (N + C::BN - 1) / C::BN;
    const int ntiles = tiles_m * tiles_n;
    int grid = 256 * OCC;                                 // OCC resident blocks on each of the 256 compute units
    if (grid > (ntiles + 7) / 8 * 8) grid = (ntiles + 7) / 8 * 8;
    kern<<<grid, C::THREADS, LDS, stream>>>(Xq, sx, Wq, sw, reinterpret_cast<const uint16_t *>(bias), M, N, K,
                                            reinterpret_cast<uint16_t *>(Y), acc_debug, tiles_m, tiles_n);
    return hipGetLastError();
}

hipError_t run_w4a4_gemm(const uint8_t *Xq, const float *sx, const uint8_t *Wq, const float *sw,
                         const void *bias, int M, int N, int K, void *Y, int32_t *acc_debug, hipStream_t stream)
{
    if (M <= 0) return hipSuccess;
#define GOP(...) return launch_gemm_persistent<__VA_ARGS__>(Xq, sx, Wq, sw, bias, M, N, K, Y, acc_debug, stream)
#ifdef QVGGT_DEV
    // development builds only (python -m paper_2509_21302_amd.build --dev): pick a tile configuration at run time
    const char *ev = getenv("QVGGT_GEMM_VARIANT");
    switch (ev ? atoi(ev) : 0) {
        case 51: GOP(4, 2, 2, 2, 64, 2, 3);
        case 52: GOP(4, 2, 2, 2, 64, 2, 0);
        case 53: GOP(2, 4, 2, 2, 64, 2, 2);
        case 55: GOP(2, 2, 2, 2, 64, 3, 2);
        case 56: GOP(4, 2, 2, 4, 64, 1, 2);
        default: break;
    }
#endif
    // 256 tokens x 128 channels per block, four waves of 128 x 64, two blocks per compute unit
    GOP(4, 2, 2, 2, 64, 2, 2);
#undef GOP
}

}  // namespace qvggt
