// The statically batched expert GEMM kernel (gfx950 / CDNA4, wave64, MFMA).
//
// One launch covers every expert (Alg. 3/4): a workgroup turns its block index
// into (expert, m-tile, n-tile) with the wavefront vote of Alg. 2, gathers the
// tile's token rows through the expert's token index array (Sec. 4.3), and runs
// an LDS pipeline feeding MFMA (the CDNA4 counterpart of the pipeline of
// Sec. 4.4): a global->LDS DMA ring (no register staging), hand-placed MFMA /
// LDS-read / DMA interleave, per-wavefront skipping of all-padding row blocks in
// an expert's last m-tile.  moe_gemm_pipe_kernel runs one tiling strategy,
// moe_gemm_pipe2_kernel two (Alg. 3 with two task types).  The contraction is computed transposed: the weight
// tile is the MFMA "A" operand (accumulator rows = output columns n) and the
// token tile the "B" operand (accumulator columns = token rows m), so that each
// lane ends up with runs of 4 consecutive n for one token row.
//
// Weights are [K][N] with N contiguous, while MFMA wants K-runs per lane: the
// weight tile is kept in LDS as loaded and read with the transposing LDS reads
// (ds_read_b64_tr_b16 / ds_read_b64_tr_b8).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "task_map.hpp"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;
typedef __attribute__((ext_vector_type(2))) int i32x2_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;

#define MOE_LDS(T) __attribute__((address_space(3))) T

struct GemmArgs {
    const void* X;
    const void* W;
    const int32_t* map;
    void* Y;
    const float* x_scale;
    const float* w_scale;
    int T, k, E, K, N;
    int tile_m_small, small_max_rows;  // second tiling strategy of the map (0, 0 = none)
    int tile_m_slack;                  // slack rows of the map's last m-tiles
    int swiglu;                        // 1: W = [gate | up] halves of N, Y[r, i] = silu(gate_i) * up_i, Y is [R, N/2]
    float* partial;                    // split-k launches: fp32 partial sums [gridDim.y][R (sorted row position)][N]
    // split-k task functions: which part of K this workgroup runs, and where its partial sums go (set per workgroup
    // by the kernel, not by the host): partial_tile != nullptr: row m of the tile at partial_tile + m * BN (a
    // compact per-tile block); else row position p, column n at partial + (k_part * R + p) * N + n
    int k_part, k_parts;
    float* partial_tile;
    // tail-split launches (cus_per_xcd > 0): the tiles of an XCD's last, partly filled round are left to the
    // workgroups of the tail launch whenever those can split them (see tail_parts)
    int cus_per_xcd;
    // heterogeneous launches: a reduction task batched with the GEMM tasks (Alg. 3 with two task types), else red_tiles = 0
    const void* red_Y;                 // [red_T][red_k][red_N] bf16, finished products of an earlier launch
    const float* red_w;                // [red_T][red_k] or nullptr
    void* red_out;                     // [red_T][red_N] bf16
    int red_T, red_k, red_N, red_tiles;
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    bf16x2_t p = {(__bf16)a, (__bf16)b};  // hardware round-to-nearest-even
    return __builtin_bit_cast(uint32_t, p);
}

// ---------------------------------------------------------------------------
// The tile function (all tile shapes, bf16 and fp8)
// ---------------------------------------------------------------------------

// The compiler may not move anything across this point.
#define MOE_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// Global -> LDS copy of 64 lanes x 16 bytes without passing through VGPRs: lane L's 16 bytes land at
// lds_addr + 16*L (lds_addr is wavefront-uniform and goes through M0).  The instruction counts in
// vmcnt like any load; the compiler does not see it, so every wait on it below is explicit.
__device__ __forceinline__ void dma16(uint32_t voff, const void* sbase, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_addr)
                 : "memory", "m0");
}
// Same, marked non-temporal: for weight rows that no other workgroup will ask for (the panel of an expert with a
// single m-tile), so that streaming them does not displace the lines other workgroups share through L2.
__device__ __forceinline__ void dma16_nt(uint32_t voff, const void* sbase, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(voff), "s"(sbase), "s"(lds_addr)
                 : "memory", "m0");
}
// f(integral_constant<int, LO>), ..., f(integral_constant<int, HI>)
template <int LO, int HI, class F>
__device__ __forceinline__ void for_each_int(F& f) {
    if constexpr (LO <= HI) {
        f(std::integral_constant<int, LO>{});
        for_each_int<LO + 1, HI>(f);
    }
}
// s_waitcnt vmcnt(N) only (expcnt / lgkmcnt fields left at "no wait").
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

// NS_ ring stages of token tiles, NSW_ ring stages of weight tiles (each k-tile deep).  SLACK_: rows a tile may
// hold beyond BM_ (the map's tile_m), for maps built with tile_m_slack.  WKC_: the weights are stored [E][N][K]
// (K contiguous, a pre-packed layout) instead of [E][K][N]: the weight tile then has the token tile's geometry
// and needs no transposing LDS reads.
template <int BM_, int BN_, int BK_, int WM_, int WN_, int NS_, bool FP8_ = false, int NSW_ = NS_, int SLACK_ = 0,
          bool WKC_ = false, int MFO_ = 0, int NSWH_ = 0>
struct PipeCfg {
    static constexpr bool SPLITK = false;
    static constexpr bool WKC = WKC_;
    // NSWH_ > 0: the weight ring is NSWH_ stages of HALF a k-tile (when whole stages do not divide the LDS left
    // beside the token ring): k-tile kt lives in half-stages (2 kt) % NSWH_ and (2 kt + 1) % NSWH_, and the loop's
    // reach ahead is that of ceil(NSWH_ / 2) whole stages.
    static constexpr bool WHALF = NSWH_ > 0;
    static constexpr int NSWH = NSWH_;
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, NS = NS_, SLACK = SLACK_;
    static constexpr int NSW = WHALF ? (NSWH_ + 1) / 2 : NSW_;
    static constexpr int BMC = BM + SLACK;                     // row capacity of the tile in LDS and registers
    static constexpr bool FP8 = FP8_;
    static constexpr int ES = FP8 ? 1 : 2;
    static constexpr int NT = 64 * WM * WN;
    static constexpr int WTM = BMC / WM, WTN = BN / WN;
    static constexpr int MF = MFO_ ? MFO_ : ((!FP8 && WTM >= 32) ? 32 : 16);   // MFMA block edge
    static constexpr int KS = MF == 32 ? 16 : 32;              // k elements per MFMA
    static constexpr int KSTEPS = BK / KS;
    static constexpr int NBW = WTN / MF, MBW = WTM / MF;
    static constexpr int MBW_BODY = BM / WM / MF;              // row blocks per wavefront without the slack rows
    static constexpr int ACC = MF == 32 ? 16 : 4;              // accumulator registers per block
    // Large tiles on 16-row MFMA blocks hold twice as many fragments per k-step: the token fragments are then
    // single-buffered, each reloaded for the next k-step as soon as the MFMAs of its row block are issued (XROLL).
    // Tiles of several 16-row blocks per wavefront: every wavefront runs the loop copy compiled for its own
    // number of live blocks (a run-time test around every MFMA defeats the software pipelining there).
    static constexpr bool PERWAVE = MF == 16 && MBW_BODY >= 4;
    // ... and with at least four weight blocks per wavefront the fragments are reloaded in place (see reads_after)
    static constexpr bool XROLL = PERWAVE && WTN / MF >= 4;
    // ... and the bf16 [K][N] ones run their k loop in two alternating roles (see run_pp in pipe_tile)
    static constexpr bool PP = XROLL && !WKC_ && !FP8_ && NS_ == 2 && BK_ / KS == 2;
    static constexpr int XROW = BK * ES, CPR = XROW / 16;
    static constexpr int WROW = BN * ES, CPRW = WROW / 16;
    // the token tile in LDS is rounded up so that every wavefront issues the same number of DMA instructions
    static constexpr int XS_BYTES = (BMC * XROW + 16 * NT - 1) / (16 * NT) * (16 * NT);
    static constexpr int WS_BYTES = BK * WROW;                 // (BN rows of XROW bytes when WKC: same size)
    static constexpr int W_RING = NS * XS_BYTES;               // byte offset of the weight ring
    static constexpr int WH_BYTES = WS_BYTES / 2;
    static constexpr int LDS_BYTES = NS * XS_BYTES + (WHALF ? NSWH * WH_BYTES : NSW * WS_BYTES);
    static_assert(!WHALF || (NS_ == 2 && !FP8_ && !WKC_ && BK_ / (MFO_ == 16 ? 32 : 16) == 2 && NSWH_ % 2 == 1),
                  "half-stage weight ring: two k-steps per k-tile, two token stages, an odd number of half-stages");
    // weight-fragment LDS reads per k-step (two 4-k halves for bf16, one 8-k piece for fp8)
    static constexpr int WREADS = NBW * ((FP8 || WKC) ? 1 : 2);
    // memory-bound tiles start the weight stream before the token rows are known
    static constexpr bool EARLY_W = MF == 16;
    static_assert(XROW == 64 || XROW == 128, "token tile rows are 64 or 128 bytes");
    static_assert(WTM % MF == 0 && WTN % MF == 0 && KSTEPS >= 2 && BK % KS == 0, "wave tile");
    static_assert(BM % (WM * MF) == 0 && SLACK % (WM * MF) == 0, "body and slack rows split evenly over the wavefront rows");
    static_assert(WROW <= 1024, "weight tile row");
    static_assert(XS_BYTES % 1024 == 0 && WS_BYTES % 1024 == 0, "DMA granularity");
    static_assert(NSW >= NS && NS >= 2, "the weight ring is at least as deep as the token ring");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

// The same tile function as one of gridDim.y workgroups that share a tile: workgroup y runs the y-th part of the
// k loop and leaves its fp32 sums in the workspace (row = position in sorted_rows, so no scatter here); a reduction
// kernel adds the parts, rounds once and scatters.  For launches too short to give every CU a tile.
template <class C>
struct SplitK : C {
    static constexpr bool SPLITK = true;
};

template <class C>
__device__ __forceinline__ int pswz_x(int row) {
    return C::CPR == 8 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}
template <class C>
__device__ __forceinline__ int pswz_w(int krow) {
    int s;
    if constexpr (C::FP8) s = C::CPRW >= 16 ? (krow & 15) : ((krow >> 1) & 7);
    else if constexpr (C::MF == 32) s = (krow & 3) << 2;
    else s = ((krow & 3) | ((krow >> 1) & 4)) << 1;
    return s & (C::CPRW - 1);
}

// A workgroup's run of consecutive tiles for the streaming kernel: the task records stay in registers, so the
// tile after the current one is known without touching memory and its loads can be issued while the current
// tile still multiplies.
struct TileStream {
    static constexpr int MAX_GROUPS = 4;  // E <= 256
    int4 rec[MAX_GROUPS];                 // lane-held task records, group by group
    int next_B, end_B;                    // tiles still to run: [next_B, end_B)
    moe_tiling tiling;
    const float* xs_lds;                  // LDS copies of x_scale[T] and w_scale[E] (fp8)
    const float* ws_lds;
};

// Alg. 2 + 4 on registers (see decode_block): B must be below the total tile count.
__device__ __forceinline__ TileCoord decode_from_registers(const TileStream& ts, int B) {
    int h = 0;
#pragma unroll
    for (int gi = 0; gi < TileStream::MAX_GROUPS; ++gi) h += __popcll(__ballot(B >= ts.rec[gi].x));  // pads never vote
    int4 rec = make_int4(0, 0, 0, 0);
    int kprev = 0;
#pragma unroll
    for (int gi = 0; gi < TileStream::MAX_GROUPS; ++gi) {
        if ((h >> 6) == gi) {
            rec.x = __builtin_amdgcn_readlane(ts.rec[gi].x, h & 63);
            rec.y = __builtin_amdgcn_readlane(ts.rec[gi].y, h & 63);
            rec.z = __builtin_amdgcn_readlane(ts.rec[gi].z, h & 63);
            rec.w = __builtin_amdgcn_readlane(ts.rec[gi].w, h & 63);
        }
        if (h > 0 && ((h - 1) >> 6) == gi) kprev = __builtin_amdgcn_readlane(ts.rec[gi].x, (h - 1) & 63);
    }
    const int l = B - kprev;
    TileCoord c;
    c.e = rec.y;
    const int cnt = rec.z;
    c.small = 0;
    const int mt = expert_m_tiles(cnt, ts.tiling);
    c.m_tiles = mt;
    c.n_tile = l / mt;
    c.m_tile = l - c.n_tile * mt;
    const int left = cnt - c.m_tile * ts.tiling.tile_m;
    c.rows = c.m_tile + 1 < mt ? ts.tiling.tile_m : left;
    c.row_base = rec.w + c.m_tile * ts.tiling.tile_m;
    return c;
}

typedef __attribute__((ext_vector_type(8))) int i32x8_t;
// Sixteen consecutive words through the scalar data path (read only): these loads count in lgkmcnt, so they do
// not disturb the vmcnt bookkeeping of the DMA ring.  p must be wavefront-uniform and 4-byte aligned.
// The loads and their wait are ONE statement: the compiler takes an asm's results as available when the
// statement ends, so a load left in flight across statements can have its destination registers spilled (and
// reused) before the data arrives.
__device__ __forceinline__ void scalar_load16(const int32_t* p, i32x8_t& lo, i32x8_t& hi) {
    asm volatile("s_load_dwordx8 %0, %2, 0x0\n\ts_load_dwordx8 %1, %2, 0x20\n\ts_waitcnt lgkmcnt(0)"
                 : "=&s"(lo), "=&s"(hi)
                 : "s"(p)
                 : "memory");
}

// One tile of the batch (STREAM = false), or a run of tiles taken from `ts` (STREAM = true; 16-row tiles only):
// everything after the task-map decode.  A task function in the sense of Alg. 3.
//
// LDS holds two rings: NS stages of token tiles and NSW >= NS stages of weight tiles.
// Main loop, per k-tile kt (token stage kt % NS, weight stage kt % NSW):
//   k-steps 0 .. KSTEPS-2 : MFMA of the step, interleaved with the LDS reads of the next step
//   wait for tile kt+1's DMA, workgroup barrier  (every wavefront has now read all of tile kt)
//   last k-step           : its MFMAs, interleaved with the first LDS reads of tile kt+1 and with the DMA
//                           instructions that refill the two stages with token tile kt+NS and weight tile kt+NSW
// so neither the barrier nor the DMA issue leaves the MFMA pipe without queued work, and NSW-1 tiles of
// weights per workgroup are in flight from HBM at any time.
//
// Rows: MF-row block b of the tile belongs to wavefront row b % WM (its block b / WM), so a partly filled tile
// spreads its live blocks evenly over the wavefront rows.  The loop exists in copies for a compile-time number of
// blocks per wavefront and in one copy that tests each block at run time; tiles of many 16-row blocks (PERWAVE)
// have a copy for every live-block count and each wavefront runs its own.
template <class C, bool STREAM = false>
__device__ __forceinline__ void pipe_tile(const GemmArgs& a, const int32_t* __restrict__ map, const MapLayout& L,
                                          TileCoord tc, char* smem, TileStream* ts = nullptr) {
    constexpr int BN = C::BN, BK = C::BK, ES = C::ES, NT = C::NT, NW = NT / 64, NS = C::NS, NSW = C::NSW, MF = C::MF;
    constexpr int KSTEPS = C::KSTEPS, WREADS = C::WREADS, NBW = C::NBW, MBW = C::MBW;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int g = lane >> 4, li = lane & 15;
    const int lrow = MF == 32 ? (lane & 31) : li;  // row of this lane inside an MF-row block

    // ---- DMA geometry: one wave instruction moves 64 x 16 B = 1 KiB, linear in LDS
    constexpr int XI_TOT = C::XS_BYTES / 1024, WI_TOT = C::WS_BYTES / 1024;
    static_assert(XI_TOT % NW == 0 && WI_TOT % NW == 0, "every wave issues the same number of DMA instructions");
    constexpr int XI = XI_TOT / NW, WI = WI_TOT / NW;
    constexpr int XI_BODY = C::SLACK == 0 ? XI : C::BM * C::XROW / 1024 / NW;   // instructions that cover rows < BM
    static_assert(C::SLACK == 0 || (C::BM * C::XROW) % (1024 * NW) == 0, "slack rows start at a DMA instruction boundary");
    constexpr int XROWS_PER_INST = 1024 / C::XROW, WROWS_PER_INST = 1024 / C::WROW;
    static_assert((NS - 1) * XI + (NSW - 1) * WI < 64, "vmcnt range");
    static_assert(!STREAM || (C::BM == 16 && MF == 16 && MBW == 1 && XI == 1 && NS == NSW && C::SLACK == 0 && KSTEPS % 2 == 0),
                  "the streaming loop is written for 16-row tiles");
    // per-lane source offsets inside a tile; everything that depends on the tile (expert, n-tile) is in the base pointer
    // When a wavefront's weight instructions lie a multiple of 16 k-rows apart they share swizzle and lane
    // pattern: one offset register serves them all and the distance goes into the scalar base.
    constexpr bool W_FOLD = !C::WKC && (NW * WROWS_PER_INST) % 16 == 0;
    constexpr int WI_OFF = W_FOLD ? 1 : WI;
    uint32_t dx_off[XI], dx_next = 0, dw_off[WI_OFF];
    const uint32_t w_row_bytes = (uint32_t)a.N * ES;
#pragma unroll
    for (int j = 0; j < WI_OFF; ++j) {
        const int inst = j * NW + wave;
        if constexpr (C::WKC) {
            // tile row = weight column; a lane's 16 bytes are 8 (16) consecutive k of that column
            const int row = inst * XROWS_PER_INST + lane / C::CPR, pos = lane % C::CPR;
            int src = row;
            if (a.swiglu) src = (row >> 5) * 16 + (row & 15) + ((row >> 4) & 1) * (a.N >> 1);
            dw_off[j] = (uint32_t)src * (uint32_t)(a.K * ES) + ((pos ^ pswz_x<C>(row)) << 4);
            continue;
        }
        const int krow = inst * WROWS_PER_INST + lane / C::CPRW, pos = lane % C::CPRW;
        // 16-byte chunk of the tile's k-row this lane fetches (the swizzle is applied on the source side)
        const int chunk = pos ^ pswz_w<C>(krow);
        uint32_t col_bytes = chunk << 4;
        if (a.swiglu) {
            // Tile columns come in units of 16: even units are gate columns, odd units the up columns of the same
            // 16 outputs, so that a lane ends up with a gate value and its up value in its own accumulators.
            const int c0 = chunk * (16 / ES);                  // first tile column of the chunk
            const int unit = c0 >> 4, src = (unit >> 1) * 16 + (c0 & 15) + (unit & 1) * (a.N >> 1);
            col_bytes = (uint32_t)src * ES;
        }
        dw_off[j] = (uint32_t)krow * w_row_bytes + col_bytes;
    }
    // split-k: this workgroup's part of K (the row pitch of X and the k stride of W are those of the whole K)
    const int k_parts = C::SPLITK ? a.k_parts : 1;
    const int KT = a.K / BK / k_parts;
    const int k_first = C::SPLITK ? a.k_part * KT * BK : 0;
    const char* Xb = static_cast<const char*>(a.X) + (size_t)k_first * ES;
    // weight base of a tile: expert, and the first column the tile reads (half as far with the fused activation)
    auto w_base = [&](const TileCoord& t) {
        const size_t col = (size_t)(a.swiglu ? (t.n_tile * BN) >> 1 : t.n_tile * BN);
        return static_cast<const char*>(a.W) + ((size_t)t.e * a.K * a.N + (C::WKC ? col * a.K + k_first : col + (size_t)k_first * a.N)) * ES;
    };
    const char* Wt = w_base(tc);
    const char* Wt_next = Wt;
    const size_t w_kt_stride = C::WKC ? (size_t)BK * ES : (size_t)BK * w_row_bytes;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(MOE_LDS(char)*)smem;

    // Weight panels that only this tile reads are fetched non-temporally -- when the grid is large enough to
    // stream from all CUs (measured: +10 % HBM throughput on the weight-streaming points, -9 % on a 132-tile grid).
    const bool nt_ok = map[MOE_HDR_TOTAL_TILES] >= 256;
    bool w_once = nt_ok && tc.m_tiles == 1, w_once_next = false;
    // j-th token-row / weight-row DMA instruction of this wave for k-tile kt, into ring stage `stage`
    auto dma_x = [&](int j, int kt, int stage, bool next) __attribute__((always_inline)) {
        dma16(next ? dx_next : dx_off[j], Xb + (size_t)kt * (BK * ES), lds0 + stage * C::XS_BYTES + (j * NW + wave) * 1024);
    };
    // ntm: 0 plain, 1 non-temporal, 2 decided at run time.  The 256-row loops are MFMA-bound and always plain:
    // a branch at each of their DMA instructions measured 2-5 % slower, and a second copy of the loops for the
    // hinted form made the register allocator spill.
    auto dma_w = [&](int j, int kt, int stage, bool next, int ntm) __attribute__((always_inline)) {
        const char* src = (next ? Wt_next : Wt) + (size_t)kt * w_kt_stride +
                          (W_FOLD ? (size_t)(j * NW * WROWS_PER_INST) * w_row_bytes : (size_t)0);
        const uint32_t dst = lds0 + C::W_RING + stage * C::WS_BYTES + (j * NW + wave) * 1024;
        const uint32_t voff = dw_off[W_FOLD ? 0 : j];
        if (ntm == 2 ? (next ? w_once_next : w_once) : ntm == 1) dma16_nt(voff, src, dst);
        else dma16(voff, src, dst);
    };

    // half-stage weight ring: jj-th instruction of this wave for half-k-tile q (k rows [q BK/2, (q+1) BK/2)) into
    // half-stage hs
    static_assert(!C::WHALF || (W_FOLD && C::EARLY_W && WI % 2 == 0 && !STREAM), "half-stage weight ring");
    auto dma_wh = [&](int jj, int q, int hs) __attribute__((always_inline)) {
        const char* src = Wt + (size_t)q * (w_kt_stride / 2) + (size_t)(jj * NW * WROWS_PER_INST) * w_row_bytes;
        dma16(dw_off[0], src, lds0 + C::W_RING + hs * C::WH_BYTES + (jj * NW + wave) * 1024);
    };

    if (C::EARLY_W) {
        if constexpr (C::WHALF) {
            // (alternating roles: the loop's first iteration fetches the ring's last stage like every other one)
#pragma unroll
            for (int q = 0; q < (C::PP ? 4 : C::NSWH); ++q)
                if (q < 2 * KT) {
#pragma unroll
                    for (int jj = 0; jj < WI / 2; ++jj) dma_wh(jj, q, q);
                }
        } else {
#pragma unroll
            for (int s = 0; s < (C::PP ? NS : NSW); ++s)
                if (s < KT) {
#pragma unroll
                    for (int j = 0; j < WI; ++j) dma_w(j, s, s, false, 2);
                }
        }
    }

    // ---- per-tile row information
    const int32_t* rows_of_tile = map + L.off_rows + tc.row_base;
    // streaming: lane j < 16 holds the flat row id of tile row j (row 0's for j past the tile's rows) and the
    // token's scale; fetched through the scalar path and LDS so that no vector-memory wait is ever generated
    int rows_v = 0, rows_v_next = 0;
    auto stream_rows = [&](const TileCoord& t, int& rv, uint32_t& dxo) {
        i32x8_t lo, hi;
        scalar_load16(map + L.off_rows + t.row_base, lo, hi);
        int v = lo[0];
#pragma unroll
        for (int j = 1; j < 16; ++j) v = (lane == j && j < t.rows) ? (j < 8 ? lo[j] : hi[j - 8]) : v;
        rv = v;
        const int tok = v / a.k;                                       // lanes 0..15
        const int row = wave * XROWS_PER_INST + lane / C::CPR, pos = lane % C::CPR;
        const int tok_of_row = __shfl(tok, row);
        dxo = (uint32_t)tok_of_row * (uint32_t)(a.K * ES) + ((pos ^ pswz_x<C>(row)) << 4);
    };
    if constexpr (STREAM) {
        stream_rows(tc, rows_v, dx_off[0]);
    } else {
#pragma unroll
        for (int j = 0; j < XI; ++j) {
            const int inst = j * NW + wave;
            const int row = inst * XROWS_PER_INST + lane / C::CPR, pos = lane % C::CPR;
            // rows past the tile's count: fetch a valid row, never store it
            const int r = rows_of_tile[row < tc.rows ? row : 0];
            dx_off[j] = (uint32_t)(r / a.k) * (uint32_t)(a.K * ES) + ((pos ^ pswz_x<C>(row)) << 4);
        }
    }

    using acc_t = typename std::conditional<MF == 32, f32x16_t, f32x4_t>::type;
    acc_t acc[NBW][MBW];

    // blocks of this wavefront that hold at least one real row: blocks wm, wm + WM, ... below ceil(rows / MF)
    const int live_blocks = (tc.rows + MF - 1) / MF;
    int mb_live = (live_blocks - wm + C::WM - 1) / C::WM;
    mb_live = mb_live < 0 ? 0 : (mb_live > MBW ? MBW : mb_live);

    // ---- fragment registers, double-buffered across k-steps; per-lane LDS offsets of k-step 0
    u32x2_t wq[2][NBW][2];       // (XROLL: [1][nb < NBW / 2] is never used)
    u32x4_t xq[C::XROLL ? 1 : 2][MBW];
    int w_rd[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        int kr0, ncol, c, within;
        if constexpr (C::FP8) {
            kr0 = 8 * g + (li >> 1);
            ncol = wn * C::WTN + nb * 16 + 8 * (li & 1);
            c = ncol >> 4; within = ncol & 15;
        } else if constexpr (MF == 32) {
            kr0 = 8 * (g >> 1) + (li >> 2);
            ncol = wn * C::WTN + nb * 32 + 16 * (g & 1) + 4 * (li & 3);
            c = ncol >> 3; within = (ncol & 7) * 2;
        } else {
            kr0 = 8 * g + (li >> 2);
            ncol = wn * C::WTN + nb * 16 + 4 * (li & 3);
            c = ncol >> 3; within = (ncol & 7) * 2;
        }
        // the swizzle of row kr0 also holds for kr0 + 4 and kr0 + KS*kk (see pswz_w), so later k-steps add a constant
        // The ring's offset is part of the register (and hidden from constant folding), so that what a read adds
        // to it -- k-step, half -- stays within the 16-bit offset field of the LDS instruction.
        w_rd[nb] = C::W_RING + kr0 * C::WROW + ((c ^ pswz_w<C>(kr0)) << 4) + within;
        asm volatile("" : "+v"(w_rd[nb]));
    }
    // tile row of this lane in its block mb; the swizzle only looks at row bits below MF, so it is the same for every block
    const int row0 = wm * MF + lrow;
    const int x_rd = row0 * C::XROW;
    constexpr int X_BLOCK_STRIDE = C::WM * MF * C::XROW;
    static_assert(MF % 16 == 0, "pswz_x must not depend on the block");
    const int xswz = pswz_x<C>(row0);

    // weight fragments are double-buffered across k-steps, except (XROLL) the first half of the blocks
    auto wbuf = [](int buf, int nb) __attribute__((always_inline)) { return (C::XROLL && nb < NBW / 2) ? 0 : buf; };
    // r-th LDS read of k-step kk, ordered by first use in the MFMA sequence (token block 0, weights, token blocks 1..)
    auto read_one = [&](int r, int sx, int sw, int kk, int buf, bool tail) __attribute__((always_inline)) {
        const char* xs = smem + sx * C::XS_BYTES;
        // w_rd holds the ring's offset; with half-stages sw is the tile's first half-stage and k-step kk lives in the
        // kk-th one after it, starting at its row 0
        int hs = sw + kk;
        if (hs >= C::NSWH) hs -= C::NSWH;
        const char* ws = C::WHALF ? smem + hs * C::WH_BYTES - (kk * C::KS) * C::WROW : smem + sw * C::WS_BYTES;
        if (r >= 1 && r <= WREADS) {
            if constexpr (C::WKC) {
                const int nb = r - 1;
                const int row = wn * C::WTN + nb * MF + lrow;
                const char* wrow = ws + C::W_RING + row * C::XROW;
                if constexpr (C::FP8) {
                    const int c = kk * 2 + (g >> 1);
                    wq[wbuf(buf, nb)][nb][0] = *reinterpret_cast<const u32x2_t*>(wrow + ((c ^ pswz_x<C>(row)) << 4) + (g & 1) * 8);
                } else {
                    const int c = MF == 32 ? kk * 2 + (lane >> 5) : kk * 4 + g;
                    const u32x4_t v = *reinterpret_cast<const u32x4_t*>(wrow + ((c ^ pswz_x<C>(row)) << 4));
                    const int wb = wbuf(buf, nb);
                    wq[wb][nb][0].x = v.x; wq[wb][nb][0].y = v.y; wq[wb][nb][1].x = v.z; wq[wb][nb][1].y = v.w;
                }
            } else if constexpr (C::FP8) {
                const int nb = r - 1;
                const char* p = ws + w_rd[nb] + (kk * 32) * C::WROW;
                wq[wbuf(buf, nb)][nb][0] = __builtin_bit_cast(u32x2_t, __builtin_amdgcn_ds_read_tr8_b64_v2i32((MOE_LDS(i32x2_t)*)(p)));
            } else {
                const int nb = (r - 1) >> 1, half = (r - 1) & 1;
                const char* p = ws + w_rd[nb] + (kk * C::KS + half * 4) * C::WROW;
                wq[wbuf(buf, nb)][nb][half] = __builtin_bit_cast(u32x2_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16((MOE_LDS(s16x4_t)*)(p)));
            }
        } else {
            const int mb = r == 0 ? 0 : r - WREADS;
            if (tail && mb >= mb_live) return;
            const char* xrow = xs + x_rd + mb * X_BLOCK_STRIDE;
            if constexpr (C::FP8) {
                const int c = kk * 2 + (g >> 1);
                const u32x2_t v = *reinterpret_cast<const u32x2_t*>(xrow + ((c ^ xswz) << 4) + (g & 1) * 8);
                xq[C::XROLL ? 0 : buf][mb].x = v.x; xq[C::XROLL ? 0 : buf][mb].y = v.y;
            } else {
                const int c = MF == 32 ? kk * 2 + (lane >> 5) : kk * 4 + g;
                xq[C::XROLL ? 0 : buf][mb] = *reinterpret_cast<const u32x4_t*>(xrow + ((c ^ xswz) << 4));
            }
        }
    };
    // i-th MFMA of a k-step over nmb row blocks: row-block-major, or (XROLL) the first half of the weight blocks
    // for every row block and then the second half, which lets the first half's fragments be reloaded in place
    auto mfma_at = [&](int mb, int nb, int buf, bool tail) __attribute__((always_inline)) {
        if (tail && mb >= mb_live) return;
        if constexpr (C::FP8) {
            const u32x2_t xv = {xq[C::XROLL ? 0 : buf][mb].x, xq[C::XROLL ? 0 : buf][mb].y};
            acc[nb][mb] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(__builtin_bit_cast(long, wq[wbuf(buf, nb)][nb][0]),
                                                                     __builtin_bit_cast(long, xv), acc[nb][mb], 0, 0, 0);
        } else {
            const int wb = wbuf(buf, nb);
            const u32x4_t wv = {wq[wb][nb][0].x, wq[wb][nb][0].y, wq[wb][nb][1].x, wq[wb][nb][1].y};
            const bf16x8_t wf = __builtin_bit_cast(bf16x8_t, wv), xf = __builtin_bit_cast(bf16x8_t, xq[C::XROLL ? 0 : buf][mb]);
            if constexpr (C::PP) {
                // Written out so that the sum stays in its registers: left to itself the register allocator moves
                // accumulators into fragment registers that have just become free and copies them back at the end
                // of the loop (tens of moves per k-tile, and spills among the MFMAs).  The accumulator is only ever
                // written by this instruction with the same destination, which may follow itself back to back; its
                // first use outside the loop comes after a barrier and a wait.
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[nb][mb]) : "v"(wf), "v"(xf));
            } else if constexpr (MF == 32) acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[nb][mb], 0, 0, 0);
            else acc[nb][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xf, acc[nb][mb], 0, 0, 0);
        }
    };
    auto mfma_one = [&](int i, int nmb, int buf, bool tail) __attribute__((always_inline)) {
        const int mb = C::XROLL ? (i % (NBW / 2 * nmb)) / (NBW / 2) : i / NBW;
        const int nb = C::XROLL ? i / (NBW / 2 * nmb) * (NBW / 2) + i % (NBW / 2) : i % NBW;
        mfma_at(mb, nb, buf, tail);
    };

    TileCoord tc_next = tc;       // streaming: the tile after the current one
    int cur = 0, curw = 0;        // ring positions; they run on from tile to tile when streaming
    bool first = true;            // the rings are empty: fill them before the loop
    bool has_next = false;        // streaming: another tile follows, its first k-tiles are fetched by this tile's last iterations

    // The tile's whole k loop for NMB row blocks per wavefront and XIL token-row DMA instructions per stage.
    auto run = [&](auto nmb_tag, auto xil_tag, auto tail_tag, auto nt_tag) __attribute__((always_inline)) {
        constexpr int NMB = decltype(nmb_tag)::value, XIL = decltype(xil_tag)::value, NTM = decltype(nt_tag)::value;
        constexpr bool TAIL = decltype(tail_tag)::value;
        constexpr int NM = NBW * NMB, NREADS = WREADS + NMB, ND = XIL + WI;
        // d-th DMA instruction of a stage (token rows first) for k-tile kt of this tile, or, past its end, of the next
        auto dma_one = [&](int d, int ktx, int ktw, int sx, int sw, bool all_in_range) __attribute__((always_inline)) {
            if (d < XIL) {
                if (all_in_range || ktx < KT) dma_x(d, ktx, sx, false);
                else if (STREAM && has_next) dma_x(d, ktx - KT, sx, true);
            } else if constexpr (C::WHALF) {
                // the two half-stages of the k-tile just read take half-k-tiles 2 kt + NSWH and 2 kt + NSWH + 1
                const int h = (d - XIL) / (WI / 2), jj = (d - XIL) % (WI / 2);
                const int q = 2 * (ktx - NS) + C::NSWH + h;
                int hs = sw + h;
                if (hs >= C::NSWH) hs -= C::NSWH;
                if (all_in_range || q < 2 * KT) dma_wh(jj, q, hs);
            } else {
                if (all_in_range || ktw < KT) dma_w(d - XIL, ktw, sw, false, NTM);
                else if (STREAM && has_next) dma_w(d - XIL, ktw - KT, sw, true, NTM);
            }
        };
        if (first) {
            // ---- prologue: fill the rings, first fragments into registers
#pragma unroll
            for (int s = 0; s < NSW; ++s) {
                if (s < KT) {
#pragma unroll
                    for (int d = (s < NS ? 0 : XIL); d < (C::EARLY_W ? XIL : ND); ++d) dma_one(d, s, s, s, s, true);
                }
            }
            // EARLY_W issued weights and token rows in two batches: wait for all of it; else only tile 0 is needed
            if (!C::EARLY_W && NSW <= KT) wait_vmcnt<(NS - 1) * XIL + (NSW - 1) * WI>(); else wait_vmcnt<0>();
            __syncthreads();
#pragma unroll
            for (int r = 0; r < NREADS; ++r) read_one(r, 0, 0, 0, 0, TAIL);
        }

        // LDS reads that follow MFMA i of a k-step, for the step after it.  Evenly spread in order of first use;
        // with single-buffered token fragments a row block's fragment follows the last MFMA that reads it and the
        // weight fragments fill the other slots.
        auto reads_after = [&](int i, int sx, int sw, int kk, int buf) __attribute__((always_inline)) {
            if constexpr (C::XROLL) {
                // first half of the step: the second-half weight blocks for the next step (into the other buffer);
                // second half: the first-half weight blocks (in place, their last use is over) and, behind the
                // last MFMA of each row block, that block's token fragment (in place)
                constexpr int HB = NBW / 2, H = HB * NMB, HR = WREADS / 2;   // HR: weight reads of one half
                static_assert(!C::XROLL || (NBW % 2 == 0 && H >= HR && NMB * (HB - 1) >= HR), "reads fit their slots");
                if (i < H) {
                    if (i < HR) read_one(1 + HR + i, sx, sw, kk, buf, TAIL);
                } else {
                    const int mb = (i - H) / HB, p = (i - H) % HB;
                    if (p == HB - 1) read_one(mb == 0 ? 0 : WREADS + mb, sx, sw, kk, buf, TAIL);
                    else if (mb * (HB - 1) + p < HR) read_one(1 + mb * (HB - 1) + p, sx, sw, kk, buf, TAIL);
                }
            } else {
#pragma unroll
                for (int r = i * NREADS / NM; r < (i + 1) * NREADS / NM; ++r) read_one(r, sx, sw, kk, buf, TAIL);
            }
        };
        auto iteration = [&](int kt, auto steady_tag) __attribute__((always_inline)) {
            constexpr bool STEADY = decltype(steady_tag)::value;  // kt + NSW < KT: every fetch below is in range
            const bool more = STEADY || (STREAM && has_next);     // every fetch below has a target
            const int nxt = cur + 1 == NS ? 0 : cur + 1;
            const int nxtw = C::WHALF ? (curw + 2 >= C::NSWH ? curw + 2 - C::NSWH : curw + 2) : (curw + 1 == NSW ? 0 : curw + 1);
#pragma unroll
            for (int kk = 0; kk < KSTEPS - 1; ++kk) {
#pragma unroll
                for (int i = 0; i < NM; ++i) {
                    mfma_one(i, NMB, kk & 1, TAIL);
                    reads_after(i, cur, curw, kk + 1, (kk + 1) & 1);
                    MOE_SCHED_FENCE();
                }
            }
            // Tile kt+1 must have landed.  Issue order is [X(j+NS) W(j+NSW)] per iteration j, so what may still
            // be in flight is the NS-2 iterations' worth issued after X(kt+1), plus, with a deeper weight ring,
            // the weight rows issued right behind X(kt+1).
            // (Half-stage ring: the iteration before issued X(kt+1), then half-k-tiles 2 kt + 3 and 2 kt + 4; only
            // the last of them is not part of tile kt+1.)
            constexpr int NEWER = C::WHALF ? WI / 2 : (NS - 2) * ND + (NSW > NS ? WI : 0);
            if (more || kt + NSW - 1 < KT) wait_vmcnt<NEWER>(); else wait_vmcnt<0>();
            __syncthreads();
            MOE_SCHED_FENCE();
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                mfma_one(i, NMB, (KSTEPS - 1) & 1, TAIL);
                if (more || kt + 1 < KT) reads_after(i, nxt, nxtw, 0, KSTEPS & 1);
#pragma unroll
                for (int d = i * ND / NM; d < (i + 1) * ND / NM; ++d) dma_one(d, kt + NS, kt + NSW, cur, curw, STEADY);
                MOE_SCHED_FENCE();
            }
            cur = nxt;
            curw = nxtw;
        };
        int kt = 0;
        for (; kt + NSW < KT; ++kt) iteration(kt, std::true_type{});
        if constexpr (STREAM) {
            // the following tile's token-row offsets, just before the iterations that start fetching it; the
            // n-tiles of one (expert, m-tile) follow each other and share their rows
            if (has_next) {
                if (tc_next.row_base == tc.row_base && tc_next.rows == tc.rows) {
                    rows_v_next = rows_v;
                    dx_next = dx_off[0];
                } else {
                    stream_rows(tc_next, rows_v_next, dx_next);
                }
            }
        }
        for (; kt < KT; ++kt) iteration(kt, std::false_type{});
    };

    // The k loop in two alternating roles (PP tiles; two k-steps per k-tile, two token stages).  The hardware places
    // wavefronts w and w + NW/2 of a workgroup on the same SIMD; they take opposite roles.  Time is cut into slots
    // by workgroup barriers, four per k-tile; in every slot one role issues a whole k-step's MFMAs back to back
    // (M), all fragments already in registers, while the other (L) reloads its single-buffered fragments for its
    // next k-step -- so no wavefront ever waits for an LDS read between two MFMAs, and the SIMD's MFMA pipe always
    // has a wavefront that wants it:
    //            slot 1        slot 2        slot 3             slot 4
    //   role 0   M(kt, 0)      L(kt, 1)      M(kt, 1), wait     L(kt+1, 0)
    //   role 1   L(kt, 0)      M(kt, 0)      L(kt, 1), wait     M(kt, 1)
    // After slot 1 nobody reads the weights of k-step 0 of tile kt any more, after slot 3 nothing of tile kt; the
    // wait in slot 3 is for the wavefront's own DMAs of tile kt+1, which the barrier behind it publishes.  Refills,
    // per wavefront in this order: slot 1: first half of the weight instructions that become free with the barrier
    // after slot 3 of tile kt-1; slot 2: the other half (half-stage ring: k-step 0 of tile kt, just read); slot 4:
    // token tile kt+2.  At the wait only the weight instructions of slots 1 and 2 (WI of them) may be in flight.
    // The prologue fills two stages of each ring; the last two iterations of a tile fetch nothing.
    // In an M slot the DMA instructions go between the MFMAs, spread over the slot.
    auto run_pp = [&](auto nmb_tag, auto xil_tag, auto tail_tag, auto role_tag) __attribute__((always_inline)) {
        constexpr int NMB = decltype(nmb_tag)::value, ROLE = decltype(role_tag)::value;
        constexpr bool TAIL = decltype(tail_tag)::value;
        constexpr int NM = NBW * NMB, NREADS = WREADS + NMB, WH = WI / 2;
        // token-row instructions of this role's wavefronts that cover at least one row of the tile (the tile in LDS
        // is rounded up to whole instructions per wavefront; the upper wavefronts' last one may be all padding)
        constexpr int XI_ROLE = (C::BMC + XROWS_PER_INST * NW - 1 - ROLE * (NW / 2) * XROWS_PER_INST) / (XROWS_PER_INST * NW);
        constexpr int XIL = decltype(xil_tag)::value < XI_ROLE ? decltype(xil_tag)::value : XI_ROLE;
        static_assert(KSTEPS == 2 && NS == 2 && NSW == 3 && WI % 2 == 0 && !STREAM && C::EARLY_W && C::XROLL, "alternating roles");
        auto bar = []() __attribute__((always_inline)) {
            MOE_SCHED_FENCE();
            __builtin_amdgcn_s_barrier();
            MOE_SCHED_FENCE();
        };
        auto lgkm0 = []() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0xc07f); };
        auto reads = [&](int sx, int sw, int kk) __attribute__((always_inline)) {
            MOE_SCHED_FENCE();
#pragma unroll
            for (int r = 0; r < NREADS; ++r) read_one(r, sx, sw, kk, 0, TAIL);
        };
        // a k-step's MFMAs, with ND DMA instructions dma(0) .. dma(ND-1) spread between them
        auto mma = [&](auto nd_tag, auto&& dma) __attribute__((always_inline)) {
            constexpr int ND = decltype(nd_tag)::value, SP = ND > 0 ? NM / ND : NM;
            static_assert(ND <= NM, "one DMA instruction per MFMA at most");
            MOE_SCHED_FENCE();
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                // row block by row block, the weight blocks back and forth: every MFMA differs from the one before
                // in one operand only (measured: +1.2 % on the headline against always ascending weight blocks)
                mfma_at(i / NBW, ((i / NBW) & 1) ? NBW - 1 - i % NBW : i % NBW, 0, TAIL);
                if (ND > 0 && i % SP == SP / 2 && i / SP < ND) dma(i / SP);
                MOE_SCHED_FENCE();
            }
        };
        if (first) {
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                if (s < KT) {
#pragma unroll
                    for (int d = 0; d < XIL; ++d) dma_x(d, s, s, false);
                }
            }
            wait_vmcnt<0>();
            __syncthreads();
            if (ROLE == 0) {
                reads(0, 0, 0);
                lgkm0();
            }
        }
        auto iteration = [&](int kt, auto steady_tag) __attribute__((always_inline)) {
            constexpr bool STEADY = decltype(steady_tag)::value;   // kt + 2 < KT: the refills have a target (else there are none)
            const int nxt = cur ^ 1;
            const int nxtw = C::WHALF ? (curw + 2 >= C::NSWH ? curw + 2 - C::NSWH : curw + 2) : (curw + 1 == NSW ? 0 : curw + 1);
            const int prevw = C::WHALF ? (curw == 0 ? C::NSWH - 1 : curw - 1) : (curw == 0 ? NSW - 1 : curw - 1);
            // weight instructions into the stage that the barrier after slot 3 of tile kt-1 freed (whole stages: tile
            // kt+2, first half of its instructions; half-stages: half-k-tile 2 kt + 4), then the second half (half-stages:
            // half-k-tile 2 kt + 5 into the half-stage of k-step 0 of tile kt); the loop's first iteration fills the
            // stage that the prologue left empty
            auto wa = [&](int j) __attribute__((always_inline)) {
                if constexpr (STEADY) {
                    if constexpr (C::WHALF) dma_wh(j, 2 * kt + 4, prevw);
                    else dma_w(j, kt + 2, prevw, false, 0);
                }
            };
            auto wb = [&](int j) __attribute__((always_inline)) {
                if constexpr (STEADY) {
                    if constexpr (C::WHALF) dma_wh(j, 2 * kt + 5, curw);
                    else dma_w(WH + j, kt + 2, prevw, false, 0);
                }
            };
            auto xr = [&](int j) __attribute__((always_inline)) {
                if constexpr (STEADY) dma_x(j, kt + 2, cur, false);
            };
            auto none = [](int) __attribute__((always_inline)) {};
            using std::integral_constant;
            if constexpr (ROLE == 0) {
                mma(integral_constant<int, WH>{}, wa);
                bar();
                reads(cur, curw, 1);
#pragma unroll
                for (int j = 0; j < WH; ++j) wb(j);
                lgkm0();
                bar();
                mma(integral_constant<int, 0>{}, none);
                if (STEADY) wait_vmcnt<WI>(); else wait_vmcnt<0>();
                bar();
                if (STEADY || kt + 1 < KT) reads(nxt, nxtw, 0);
#pragma unroll
                for (int j = 0; j < XIL; ++j) xr(j);
                lgkm0();
                bar();
            } else {
                reads(cur, curw, 0);
#pragma unroll
                for (int j = 0; j < WH; ++j) wa(j);
                lgkm0();
                bar();
                mma(integral_constant<int, WH>{}, wb);
                bar();
                reads(cur, curw, 1);
                lgkm0();
                if (STEADY) wait_vmcnt<WI>(); else wait_vmcnt<0>();
                bar();
                mma(integral_constant<int, XIL>{}, xr);
                bar();
            }
            cur = nxt;
            curw = nxtw;
        };
        int kt = 0;
        for (; kt + 2 < KT; ++kt) iteration(kt, std::true_type{});
        for (; kt < KT; ++kt) iteration(kt, std::false_type{});
        // The MFMAs above are written out (see mfma_at), so the compiler does not know that the accumulators come from
        // the matrix pipe: keep the distance it would otherwise keep between an MFMA and the first ordinary
        // instruction that reads its result.
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7");
    };

    char* Yb = static_cast<char*>(a.Y);
    const size_t y_row_bytes = (size_t)(a.swiglu ? a.N >> 1 : a.N) * 2;
    auto store4 = [](char* p, float v0, float v1, float v2, float v3) {
        u32x2_t v;
        v.x = pack_bf16(v0, v1);
        v.y = pack_bf16(v2, v3);
        *reinterpret_cast<u32x2_t*>(p) = v;
    };
    // (the hardware reciprocal is good to one unit in the last place of an fp32: far inside the bf16 rounding of the result)
    auto silu_mul = [](float gate, float up) { return gate * __builtin_amdgcn_rcpf(1.f + __expf(-gate)) * up; };
    // Tiles of 64 rows and more leave through LDS: a lane's results are runs of 4 columns of one row (8 bytes), so
    // direct stores write every 128-byte line of Y in four pieces from four instructions.  Staged, each wavefront
    // writes its own WTM x WTN corner of the tile into the (now idle) rings and reads it back row-wise, 16 bytes
    // per lane, so that one store instruction covers whole lines (measured on the headline: the stores cost 5.5 %
    // of the kernel, 10 % on the paper's shorter-K shape).  Rows keep a fixed stride of 2*WTN bytes (the fused
    // activation fills half of it); 16-byte chunks are XOR-swizzled with the row.
    constexpr int RBMAX = C::WTN * 2, CPROF = RBMAX / 16;
    // (the 64-row-slack tile is larger than its rings and keeps the direct stores,
    // and so do the K-contiguous layout and fp8, whose large-tile kernels the extra code pushed into register spills)
    constexpr bool STAGED = !STREAM && C::BM >= 64 && NW * C::WTM * RBMAX <= C::LDS_BYTES && !C::WKC && !C::FP8 && !C::SPLITK;
    static_assert(!STAGED || (C::WTM * (CPROF / 2)) % 64 == 0, "staging area");
    char* const stage = smem + wave * (C::WTM * RBMAX);
    // 4 values of tile row block mb (this lane's row in it), tile columns n_out .. n_out + 3 of the OUTPUT row
    auto put4 = [&](char* yrow, int mb, int n_out, float v0, float v1, float v2, float v3) __attribute__((always_inline)) {
        if constexpr (STAGED) {
            const int lr = mb * MF + lrow;
            const int cbyte = (n_out - (a.swiglu ? (wn * C::WTN) >> 1 : wn * C::WTN)) * 2;
            u32x2_t v;
            v.x = pack_bf16(v0, v1);
            v.y = pack_bf16(v2, v3);
            *reinterpret_cast<u32x2_t*>(stage + lr * RBMAX + (((cbyte >> 4) ^ (lr & (CPROF - 1))) << 4) + (cbyte & 15)) = v;
        } else {
            store4(yrow + n_out * 2, v0, v1, v2, v3);
        }
    };

    while (true) {
        const int n0 = tc.n_tile * BN;
        if constexpr (STREAM) {
            has_next = ts->next_B < ts->end_B;
            if (has_next) {
                tc_next = decode_from_registers(*ts, ts->next_B);
                ts->next_B += 1;
                Wt_next = w_base(tc_next);
                w_once_next = nt_ok && tc_next.m_tiles == 1;
            }
        }
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
                for (int j = 0; j < C::ACC; ++j) acc[nb][mb][j] = 0.f;

        using std::integral_constant;
        auto run_nt = [&](auto nmb_tag, auto xil_tag, auto tail_tag) __attribute__((always_inline)) {
            if constexpr (C::PP) {
                if (wave < NW / 2) run_pp(nmb_tag, xil_tag, tail_tag, integral_constant<int, 0>{});
                else run_pp(nmb_tag, xil_tag, tail_tag, integral_constant<int, 1>{});
            } else {
                run(nmb_tag, xil_tag, tail_tag, integral_constant<int, C::BM <= 128 ? 2 : 0>{});
            }
        };
        if constexpr (C::PERWAVE) {
            // 16-row blocks: every wavefront runs the copy of the loop compiled for its own number of live blocks
            // (the copies agree in their barriers and DMA instructions, so wavefronts of one workgroup may differ);
            // fewer than half the body's blocks only happens when the launch has no narrower task function.
            const bool over = C::SLACK > 0 && tc.rows > C::BM;
            bool done = false;
            auto try_nmb = [&](auto nmb_tag) __attribute__((always_inline)) {
                if (!done && mb_live == decltype(nmb_tag)::value) {
                    if (over) { if constexpr (C::SLACK > 0 && decltype(nmb_tag)::value >= C::MBW_BODY) run_nt(nmb_tag, integral_constant<int, XI>{}, std::false_type{}); }
                    else { if constexpr (decltype(nmb_tag)::value <= C::MBW_BODY) run_nt(nmb_tag, integral_constant<int, XI_BODY>{}, std::false_type{}); }
                    done = true;
                }
            };
            for_each_int<C::MBW_BODY / 2, MBW>(try_nmb);
            if (!done) {
                // (alternating roles: the copy for the fewest blocks instead; its surplus blocks multiply rows that
                // are never stored, and every wavefront of the workgroup keeps the same barriers)
                if constexpr (C::PP) run_nt(integral_constant<int, C::MBW_BODY / 2>{}, integral_constant<int, XI_BODY>{}, std::false_type{});
                else run_nt(integral_constant<int, C::MBW_BODY>{}, integral_constant<int, XI_BODY>{}, std::true_type{});
            }
        } else if (C::SLACK > 0 && tc.rows > C::BM) {
            // every wavefront moves its share of the slack rows; only those whose slack block holds a real row compute it
            if (mb_live == MBW) run_nt(integral_constant<int, MBW>{}, integral_constant<int, XI>{}, std::false_type{});
            else run_nt(integral_constant<int, C::MBW_BODY>{}, integral_constant<int, XI>{}, std::false_type{});
        } else if (STREAM || mb_live == C::MBW_BODY) {
            run_nt(integral_constant<int, C::MBW_BODY>{}, integral_constant<int, XI_BODY>{}, std::false_type{});
        } else {
            run_nt(integral_constant<int, C::MBW_BODY>{}, integral_constant<int, XI_BODY>{}, std::true_type{});
        }
        if (!(STREAM && has_next)) wait_vmcnt<0>();  // a following tile's loads stay in flight across the epilogue

        // ---- epilogue: fp32 -> bf16 (RNE), scatter to Y[r, n]; fp8 applies the two scales first
        if constexpr (STAGED) __syncthreads();   // every wavefront has read its last fragments and all DMAs have landed
        // Every row id the epilogue needs is fetched here, in one batch and without branches (rows past the tile's
        // count read row 0's id and are never stored).  Loads and stores share one in-order counter: a load placed
        // between the stores waits for the store before it to be acknowledged, once per row group (measured: 6.5 us
        // of an 18-group epilogue).
        constexpr int PASSES = STAGED ? C::WTM * CPROF / 64 : 1;
        int r_pass[PASSES], r_mb[MBW];
        const int cu_ = a.swiglu ? CPROF / 2 : CPROF;   // 16-byte chunks per staged row; 64 / cu_ rows per instruction
        if constexpr (STAGED) {
#pragma unroll
            for (int pass = 0; pass < PASSES; ++pass) {
                const int lr = pass * (64 / cu_) + lane / cu_;
                const int m_local = ((lr / MF) * C::WM + wm) * MF + (lr % MF);
                const bool live = lr < C::WTM && m_local < tc.rows;
                const int r = rows_of_tile[live ? m_local : 0];
                r_pass[pass] = live ? r : -1;
            }
        } else if constexpr (C::SPLITK) {
            static_assert(!C::SPLITK || (!STREAM && !C::FP8 && !C::WKC), "split-k: bf16, weights as [E][K][N]");
            // fp32 partial sums, 16 bytes (4 columns of one row) per lane and block; no row ids needed
            float* const part = a.partial + (size_t)a.k_part * ((size_t)a.T * a.k) * a.N;
#pragma unroll
            for (int mb = 0; mb < MBW; ++mb) {
                const int m_local = (mb * C::WM + wm) * MF + lrow;
                if (m_local >= tc.rows) continue;
                float* prow = a.partial_tile ? a.partial_tile + (size_t)m_local * BN
                                             : part + (size_t)(tc.row_base + m_local) * a.N + n0;
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) {
#pragma unroll
                    for (int jq = 0; jq < C::ACC / 4; ++jq) {
                        const int n_local = MF == 32 ? wn * C::WTN + nb * 32 + 8 * jq + 4 * (lane >> 5) : wn * C::WTN + nb * 16 + 4 * g;
                        const f32x4_t v = {acc[nb][mb][4 * jq + 0], acc[nb][mb][4 * jq + 1], acc[nb][mb][4 * jq + 2], acc[nb][mb][4 * jq + 3]};
                        *reinterpret_cast<f32x4_t*>(prow + n_local) = v;
                    }
                }
            }
            break;
        } else if constexpr (!STREAM) {
#pragma unroll
            for (int mb = 0; mb < MBW; ++mb) {
                const int m_local = (mb * C::WM + wm) * MF + lrow;
                r_mb[mb] = rows_of_tile[m_local < tc.rows ? m_local : 0];
            }
        }
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb) {
            const int m_local = (mb * C::WM + wm) * MF + lrow;
            int r = 0;
            float xsc = 1.f, wsc = 1.f;
            if constexpr (STREAM) {
                r = __shfl(rows_v, m_local);
                if constexpr (C::FP8) { xsc = ts->xs_lds[r / a.k]; wsc = ts->ws_lds[tc.e]; }
                if (m_local >= tc.rows) continue;
            } else {
                if (m_local >= tc.rows) continue;
                if constexpr (!STAGED) r = r_mb[mb];
                if constexpr (C::FP8) { xsc = a.x_scale[r / a.k]; wsc = a.w_scale[tc.e]; }
            }
            if (!a.swiglu) {
                char* yrow = Yb + (size_t)r * y_row_bytes + (size_t)n0 * 2;
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) {
#pragma unroll
                    for (int jq = 0; jq < C::ACC / 4; ++jq) {
                        const int n_local = MF == 32 ? wn * C::WTN + nb * 32 + 8 * jq + 4 * (lane >> 5) : wn * C::WTN + nb * 16 + 4 * g;
                        float v0 = acc[nb][mb][4 * jq + 0], v1 = acc[nb][mb][4 * jq + 1];
                        float v2 = acc[nb][mb][4 * jq + 2], v3 = acc[nb][mb][4 * jq + 3];
                        if constexpr (C::FP8) {
                            v0 = (v0 * xsc) * wsc; v1 = (v1 * xsc) * wsc; v2 = (v2 * xsc) * wsc; v3 = (v3 * xsc) * wsc;
                        }
                        put4(yrow, mb, n_local, v0, v1, v2, v3);
                    }
                }
            } else {
                // gate and up of one output sit in the same lane: accumulators j and j + 8 of a 32-row block
                // (its rows 0-15 are a gate unit, 16-31 the up unit), or blocks nb and nb + 1 of 16 rows
                char* yrow = Yb + (size_t)r * y_row_bytes + (size_t)(n0 >> 1) * 2;
                if constexpr (MF == 32) {
#pragma unroll
                    for (int nb = 0; nb < NBW; ++nb) {
#pragma unroll
                        for (int jq = 0; jq < 2; ++jq) {
                            const int n_local = ((wn * C::WTN + nb * 32) >> 1) + 8 * jq + 4 * (lane >> 5);
                            float h[4];
#pragma unroll
                            for (int i = 0; i < 4; ++i) h[i] = silu_mul((acc[nb][mb][4 * jq + i] * xsc) * wsc, (acc[nb][mb][8 + 4 * jq + i] * xsc) * wsc);
                            put4(yrow, mb, n_local, h[0], h[1], h[2], h[3]);
                        }
                    }
                } else {
                    static_assert(MF == 32 || NBW % 2 == 0, "gate and up blocks pair up inside a wavefront");
#pragma unroll
                    for (int nb = 0; nb + 1 < NBW; nb += 2) {
                        const int n_local = ((wn * C::WTN + nb * 16) >> 1) + 4 * g;
                        float h[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) h[i] = silu_mul((acc[nb][mb][i] * xsc) * wsc, (acc[nb + 1][mb][i] * xsc) * wsc);
                        put4(yrow, mb, n_local, h[0], h[1], h[2], h[3]);
                    }
                }
            }
        }
        if constexpr (STAGED) {
            // read the corner back row by row: cu 16-byte chunks per row, 64 / cu rows per instruction
            wait_vmcnt<0>();   // the row ids, long since there; told here so that no wait lands between the stores
            const int cu = cu_;
            const int rpi = 64 / cu;
            const int c = lane & (cu - 1), lr0 = lane / cu;
            const size_t col_bytes = (size_t)(a.swiglu ? (n0 + wn * C::WTN) >> 1 : n0 + wn * C::WTN) * 2 + c * 16;
#pragma unroll
            for (int pass = 0; pass < PASSES; ++pass) {
                const int lr = pass * rpi + lr0;
                const int r = r_pass[pass];
                if (r >= 0) {
                    const u32x4_t v = *reinterpret_cast<const u32x4_t*>(stage + lr * RBMAX + ((c ^ (lr & (CPROF - 1))) << 4));
                    *reinterpret_cast<u32x4_t*>(Yb + (size_t)r * y_row_bytes + col_bytes) = v;
                }
            }
        }
        if (!(STREAM && has_next)) break;
        // the following tile becomes the current one; its first k-tiles are already in the rings
        tc = tc_next;
        Wt = Wt_next;
        w_once = w_once_next;
        dx_off[0] = dx_next;
        rows_v = rows_v_next;
        first = false;
    }
}

// Whether the map belongs to this launch (shape, tiling, strategy, slack, status); a launch whose map does not
// match does nothing.
template <int BM_BIG, int BN, int BM_SMALL, int SLACK>
__device__ __forceinline__ bool map_matches(const GemmArgs& a, const int32_t* __restrict__ map) {
    return map[MOE_HDR_MAGIC] == MOE_MAP_MAGIC && map[MOE_HDR_T] == a.T && map[MOE_HDR_K_TOP] == a.k &&
           map[MOE_HDR_E] == a.E && map[MOE_HDR_N] == a.N && map[MOE_HDR_TILE_M] == BM_BIG &&
           map[MOE_HDR_TILE_N] == BN && map[MOE_HDR_STATUS] == 0 &&
           map[MOE_HDR_TILE_M_SMALL] == BM_SMALL && map[MOE_HDR_SMALL_MAX_ROWS] == a.small_max_rows &&
           a.tile_m_small == BM_SMALL && map[MOE_HDR_TILE_M_SLACK] == SLACK && a.tile_m_slack == SLACK;
}

// Which block index slot `slot` of XCD `xcd` runs (the XCD-aware remap in front of Alg. 2 / 4: a bijection between
// a launch's slots and the map's blocks, not part of the map).  Workgroup ids are dealt round-robin to the 8 XCDs;
// every XCD gets one contiguous run of block indices so that neighbours in the map share an L2.  Returns false
// for slots beyond the XCD's share (and then for every larger slot as well).
__device__ __forceinline__ bool slot_to_block(const int32_t* __restrict__ map, int total, int xcd, int slot, int& B) {
    if (map[MOE_HDR_SIGMA_ORDER] == MOE_ORDER_INTERLEAVE) {
        // Sec. 4.2: blocks [0, heavy) are compute-bound, [heavy, total) only stream weights.  Every XCD gets a
        // contiguous share of each part and walks the two shares interleaved in proportion (slot s takes the
        // next light block whenever floor((s+1) * nl / n) exceeds floor(s * nl / n)), so that the light tiles'
        // HBM traffic is spread over the whole run of the heavy ones.
        const int heavy = map[MOE_HDR_HEAVY_TILES], light = total - heavy;
        const int h0 = (int)((long long)heavy * xcd >> 3), h1 = (int)((long long)heavy * (xcd + 1) >> 3);
        const int l0 = (int)((long long)light * xcd >> 3), l1 = (int)((long long)light * (xcd + 1) >> 3);
        const int nh = h1 - h0, nl = l1 - l0, n = nh + nl;
        if (slot >= n) return false;
        const int before = (int)((long long)slot * nl / n), upto = (int)((long long)(slot + 1) * nl / n);
        B = upto > before ? heavy + l0 + before : h0 + slot - before;
        return true;
    }
    const int per_xcd = (total + 7) >> 3;
    if (slot >= per_xcd) return false;
    B = xcd * per_xcd + slot;
    return B < total;
}
// Slots of XCD `xcd` for which slot_to_block returns true.
__device__ __forceinline__ int slots_of_xcd(const int32_t* __restrict__ map, int total, int xcd) {
    if (map[MOE_HDR_SIGMA_ORDER] == MOE_ORDER_INTERLEAVE) {
        const int heavy = map[MOE_HDR_HEAVY_TILES], light = total - heavy;
        return (int)(((long long)heavy * (xcd + 1) >> 3) - ((long long)heavy * xcd >> 3)) +
               (int)(((long long)light * (xcd + 1) >> 3) - ((long long)light * xcd >> 3));
    }
    const int per_xcd = (total + 7) >> 3;
    const int left = total - xcd * per_xcd;
    return left < 0 ? 0 : (left < per_xcd ? left : per_xcd);
}

// Tail split.  With one workgroup per tile an XCD's tiles run in rounds of `cus` (its CUs); when the last round is
// only partly filled, the other CUs idle for a whole tile's duration.  The t tiles of that round can instead be run
// by P = 2 or 4 workgroups each, every one over a part of K (fp32 partial sums, added afterwards): the t * P parts
// then take ceil(t * P / cus) sub-rounds of 1 / P of a tile's duration.  P is the smallest of 1, 2, 4 that makes
// this shortest (parts keep at least 8 k-tiles).  The map is untouched: this is a property of the launch.
__host__ __device__ inline int tail_parts(int t, int cus, int k_tiles) {
    if (t <= 0) return 1;
    int best = 1, best_len = 4;                       // duration of the last round in quarters of a tile
    for (int P = 2; P <= 4; P *= 2) {
        if (k_tiles % P != 0 || k_tiles / P < 8) break;
        const int len = (t * P + cus - 1) / cus * (4 / P);
        if (len < best_len) { best = P; best_len = len; }
    }
    return best;
}
constexpr int kTailBlocksPerXcd = 128;   // upper bound on t * P (t < cus <= 32, P <= 4): blocks of the tail workspace per XCD
struct TailSplit { int full, tail, parts; };   // slots [0, full) run whole tiles, slots [full, full + tail) are split
__device__ __forceinline__ TailSplit tail_split(const int32_t* __restrict__ map, int total, int xcd, int cus, int k_tiles) {
    const int n_x = slots_of_xcd(map, total, xcd);
    TailSplit ts;
    ts.full = n_x / cus * cus;
    ts.tail = n_x - ts.full;
    ts.parts = tail_parts(ts.tail, cus, k_tiles);
    return ts;
}

// Block index -> tile (Alg. 2 + 4), shared by the kernels below.  Returns false for surplus workgroups and for
// a map that does not belong to this launch (wrong shape, tiling or status): those do nothing.
template <int BM_BIG, int BN, int BM_SMALL, int SLACK>
__device__ __forceinline__ bool locate_tile(const GemmArgs& a, const int32_t* __restrict__ map, MapLayout& L, TileCoord& tc) {
    // the first 64 task records travel together with the header: one memory round trip before the tile is known
    L = map_layout(a.E);
    const int4 first_record = reinterpret_cast<const int4*>(map + L.off_records)[__lane_id()];
    const int total = map[MOE_HDR_TOTAL_TILES];
    if (!map_matches<BM_BIG, BN, BM_SMALL, SLACK>(a, map)) return false;
    int B;
    if (!slot_to_block(map, total, blockIdx.x & 7, blockIdx.x >> 3, B)) return false;
    if (a.cus_per_xcd > 0) {
        const TailSplit ts = tail_split(map, total, blockIdx.x & 7, a.cus_per_xcd, a.K / 64);
        if (ts.parts > 1 && (int)(blockIdx.x >> 3) >= ts.full) return false;   // the tail launch runs this tile
    }
    const moe_tiling g = {BM_BIG, BN, 0, BM_SMALL, a.small_max_rows, SLACK};
    tc = decode_block(map, L, g, B, first_record);
    return true;
}

// Run one tile with the narrowest task function that holds its rows.  An expert's last m-tile is often almost
// empty (c_e just above a multiple of tile_m); a narrower function of the same launch shape moves fewer token
// rows and issues no MFMA for the padding.  The map is unchanged: the choice only depends on the tile's row count.
template <class C>
__device__ __forceinline__ void run_tile(const GemmArgs& a, const int32_t* __restrict__ map, const MapLayout& L,
                                         const TileCoord& tc, char* smem) {
    pipe_tile<C>(a, map, L, tc, smem);
}
template <class C, class T0, class... Ts>
__device__ __forceinline__ void run_tile(const GemmArgs& a, const int32_t* __restrict__ map, const MapLayout& L,
                                         const TileCoord& tc, char* smem) {
    static_assert(T0::BM < C::BM && T0::NT == C::NT && T0::BN == C::BN && T0::FP8 == C::FP8 && T0::LDS_BYTES <= C::LDS_BYTES,
                  "a tail function shares the launch shape of the full one");
    if (tc.rows <= T0::BM) pipe_tile<T0>(a, map, L, tc, smem);
    else run_tile<C, Ts...>(a, map, L, tc, smem);
}

// One tiling strategy for every expert.  Tails: narrower task functions for partly filled tiles, narrowest first.
template <class C, class... Tails>
__global__ __launch_bounds__(C::NT) void moe_gemm_pipe_kernel(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    MapLayout L;
    TileCoord tc;
    if (!locate_tile<C::BM, C::BN, 0, C::SLACK>(a, a.map, L, tc)) return;
    if constexpr (C::SPLITK) {
        // one of gridDim.y workgroups that share the tile
        GemmArgs b = a;
        b.k_part = (int)blockIdx.y;
        b.k_parts = (int)gridDim.y;
        run_tile<C, Tails...>(b, a.map, L, tc, smem);
    } else {
        run_tile<C, Tails...>(a, a.map, L, tc, smem);
    }
}

// The tail launch of a tail-split product: workgroup i of XCD x runs part i % P of the x-th XCD's tail tile i / P
// (P = that XCD's number of parts) and leaves its fp32 sums in its own compact block of the workspace,
// [x][i][BM + SLACK][BN].  C and Tails are split-k task functions.
template <class C, class... Tails>
__global__ __launch_bounds__(C::NT) void moe_gemm_tail_kernel(GemmArgs a) {
    static_assert(C::SPLITK, "split-k task functions");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int32_t* __restrict__ map = a.map;
    const MapLayout L = map_layout(a.E);
    const int4 first_record = reinterpret_cast<const int4*>(map + L.off_records)[__lane_id()];
    const int total = map[MOE_HDR_TOTAL_TILES];
    if (!map_matches<C::BM, C::BN, 0, C::SLACK>(a, map)) return;
    const int xcd = blockIdx.x & 7, i = blockIdx.x >> 3;
    const TailSplit ts = tail_split(map, total, xcd, a.cus_per_xcd, a.K / 64);
    if (ts.parts == 1 || i >= ts.tail * ts.parts) return;
    int B;
    if (!slot_to_block(map, total, xcd, ts.full + i / ts.parts, B)) return;
    const moe_tiling g = {C::BM, C::BN, 0, 0, 0, C::SLACK};
    const TileCoord tc = decode_block(map, L, g, B, first_record);
    GemmArgs b = a;
    b.k_part = i % ts.parts;
    b.k_parts = ts.parts;
    b.partial_tile = a.partial + ((size_t)(xcd * kTailBlocksPerXcd + i) * C::BMC) * C::BN;
    run_tile<C, Tails...>(b, map, L, tc, smem);
}

// Two tiling strategies in one launch (Alg. 3 with K = 2 task types): the expert's row count picks the task
// function; both share the thread count, the n-tile width and the LDS allocation.
template <class CBIG, class CSMALL, class... Tails>
__global__ __launch_bounds__(CBIG::NT) void moe_gemm_pipe2_kernel(GemmArgs a) {
    static_assert(CBIG::NT == CSMALL::NT && CBIG::BN == CSMALL::BN && CBIG::FP8 == CSMALL::FP8, "task functions must be launch-compatible");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    MapLayout L;
    TileCoord tc;
    if (!locate_tile<CBIG::BM, CBIG::BN, CSMALL::BM, CBIG::SLACK>(a, a.map, L, tc)) return;
    if (tc.small) pipe_tile<CSMALL>(a, a.map, L, tc, smem);
    else run_tile<CBIG, Tails...>(a, a.map, L, tc, smem);
}

// Streaming launch for 16-row tiles (the weight-streaming regime): a fixed number of resident workgroups, each
// running a contiguous share of its XCD's tiles through pipe_tile<C, true>, so that the weight stream of a
// workgroup does not stop at tile boundaries.  Requires E <= 256, K / BK >= ring depth, one tiling strategy;
// fp8 scales are staged in LDS behind the rings (T + E floats).
template <class C>
__global__ __launch_bounds__(C::NT) void moe_gemm_stream_kernel(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int32_t* __restrict__ map = a.map;
    const MapLayout L = map_layout(a.E);
    const int lane = __lane_id();
    TileStream ts;
    const int4* recs = reinterpret_cast<const int4*>(map + L.off_records);
#pragma unroll
    for (int gi = 0; gi < TileStream::MAX_GROUPS; ++gi)
        ts.rec[gi] = 64 * gi < L.E64 ? recs[64 * gi + lane] : make_int4(0x7fffffff, -1, 0, 0);
    const int total = map[MOE_HDR_TOTAL_TILES];
    const bool hdr_ok = map[MOE_HDR_MAGIC] == MOE_MAP_MAGIC && map[MOE_HDR_T] == a.T && map[MOE_HDR_K_TOP] == a.k &&
                        map[MOE_HDR_E] == a.E && map[MOE_HDR_N] == a.N && map[MOE_HDR_TILE_M] == C::BM &&
                        map[MOE_HDR_TILE_N] == C::BN && map[MOE_HDR_STATUS] == 0 && map[MOE_HDR_TILE_M_SMALL] == 0 &&
                        map[MOE_HDR_SMALL_MAX_ROWS] == 0 && a.tile_m_small == 0 && a.small_max_rows == 0 &&
                        map[MOE_HDR_TILE_M_SLACK] == 0 && a.tile_m_slack == 0;
    if (!hdr_ok) return;
    // each XCD owns one contiguous run of block indices (see locate_tile); its resident workgroups split it evenly
    const int per_xcd = (total + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
    const int x0 = xcd * per_xcd;
    const int n_x = total - x0 < per_xcd ? total - x0 : per_xcd;
    if (n_x <= 0) return;
    const int per_wg = (n_x + slots - 1) / slots;
    const int t0 = x0 + slot * per_wg;
    int t1 = t0 + per_wg;
    if (t1 > x0 + n_x) t1 = x0 + n_x;
    if (t0 >= t1) return;
    float* xs_lds = reinterpret_cast<float*>(smem + C::LDS_BYTES);
    float* ws_lds = xs_lds + a.T;
    if constexpr (C::FP8) {
        for (int i = threadIdx.x; i < a.T; i += C::NT) xs_lds[i] = a.x_scale[i];
        for (int i = threadIdx.x; i < a.E; i += C::NT) ws_lds[i] = a.w_scale[i];
        __syncthreads();
    }
    ts.xs_lds = xs_lds;
    ts.ws_lds = ws_lds;
    ts.tiling = moe_tiling{C::BM, C::BN, 0, 0, 0, 0};
    ts.next_B = t0 + 1;
    ts.end_B = t1;
    const TileCoord tc = decode_from_registers(ts, t0);
    pipe_tile<C, true>(a, map, L, tc, smem, &ts);
}

}  // namespace moe
