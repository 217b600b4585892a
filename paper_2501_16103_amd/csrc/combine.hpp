// Sum over a token's selected experts (Sec. 2.2: the last step of the MoE layer), optionally weighted
// by the router: out[t, n] = bf16( sum_j w[t, j] * Y[t, j, n] ), j ascending, fp32.
// Pure streaming: each lane owns 8 consecutive n of one token (16-byte loads and stores).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_kernel.hpp"

namespace moe {

__device__ __forceinline__ float bf16_lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }

// Chunks (8 columns) [c_begin, c_end) of all tokens, walked by `nthreads` threads of which this is number `tid`:
// chunk index c -> token c / (N/8), column 8 * (c % (N/8)).
// KU > 0: k is the compile-time KU and all k loads of a chunk are issued before the first is used.
template <int KU>
__device__ __forceinline__ void combine_range(const u32x4_t* __restrict__ Y, const float* __restrict__ w, u32x4_t* __restrict__ out,
                                              int k_rt, int N, long long c_begin, long long c_end, long long tid, long long nthreads) {
    const int k = KU > 0 ? KU : k_rt;
    const int cpr = N >> 3;  // chunks per row
    for (long long c = c_begin + tid; c < c_end; c += nthreads) {
        const int t = (int)(c / cpr), col = (int)(c - (long long)t * cpr);
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const u32x4_t* src = Y + ((size_t)t * k) * cpr + col;
        auto add = [&](const u32x4_t v, float wj) {
            acc[0] += wj * bf16_lo(v.x); acc[1] += wj * bf16_hi(v.x);
            acc[2] += wj * bf16_lo(v.y); acc[3] += wj * bf16_hi(v.y);
            acc[4] += wj * bf16_lo(v.z); acc[5] += wj * bf16_hi(v.z);
            acc[6] += wj * bf16_lo(v.w); acc[7] += wj * bf16_hi(v.w);
        };
        if constexpr (KU > 0) {
            u32x4_t v[KU];
            float wj[KU];
#pragma unroll
            for (int j = 0; j < KU; ++j) {
                v[j] = __builtin_nontemporal_load(src + (size_t)j * cpr);
                wj[j] = w ? w[(size_t)t * KU + j] : 1.f;
            }
#pragma unroll
            for (int j = 0; j < KU; ++j) add(v[j], wj[j]);
        } else {
            for (int j = 0; j < k; ++j) add(src[(size_t)j * cpr], w ? w[(size_t)t * k + j] : 1.f);
        }
        u32x4_t o;
        o.x = pack_bf16(acc[0], acc[1]); o.y = pack_bf16(acc[2], acc[3]);
        o.z = pack_bf16(acc[4], acc[5]); o.w = pack_bf16(acc[6], acc[7]);
        out[(size_t)t * cpr + col] = o;
    }
}

template <int KU>
__global__ __launch_bounds__(256) void moe_combine_kernel(const u32x4_t* __restrict__ Y, const float* __restrict__ w,
                                                          u32x4_t* __restrict__ out, int T, int k_rt, int N) {
    combine_range<KU>(Y, w, out, k_rt, N, 0, (long long)T * (N >> 3), (long long)blockIdx.x * 256 + threadIdx.x,
                      (long long)gridDim.x * 256);
}

// Last step of a tail-split product: blocks (x, j, 0 .. kTailReduceSlices-1) add the parts of the x-th XCD's tail tile j
// (compact blocks [x][j * P + p][BM + SLACK][BN] of the workspace, kTailBlocksPerXcd blocks per XCD, p ascending), round
// once to bf16 and scatter the tile's rows to Y; each of the slices takes every kTailReduceSlices-th stretch of 256
// chunks (a tile by one workgroup streamed at a fifth of the rate: 42 us of an 0.8 ms product).
constexpr int kTailReduceSlices = 8;
template <int BM, int BN, int SLACK>
__global__ __launch_bounds__(256) void moe_tail_reduce_kernel(GemmArgs a) {
    constexpr int BMC = BM + SLACK;   // rows of a workspace block
    const int32_t* __restrict__ map = a.map;
    const MapLayout L = map_layout(a.E);
    const int4 first_record = reinterpret_cast<const int4*>(map + L.off_records)[__lane_id()];
    const int total = map[MOE_HDR_TOTAL_TILES];
    if (!map_matches<BM, BN, 0, SLACK>(a, map)) return;
    const int xcd = blockIdx.x & 7, j = (int)(blockIdx.x >> 3) / kTailReduceSlices, slice = (int)(blockIdx.x >> 3) % kTailReduceSlices;
    const TailSplit ts = tail_split(map, total, xcd, a.cus_per_xcd, a.K / 64);
    if (ts.parts == 1 || j >= ts.tail) return;
    int B;
    if (!slot_to_block(map, total, xcd, ts.full + j, B)) return;
    const moe_tiling g = {BM, BN, 0, 0, 0, SLACK};
    const TileCoord tc = decode_block(map, L, g, B, first_record);
    const float* base = a.partial + ((size_t)(xcd * kTailBlocksPerXcd + j * ts.parts) * BMC) * BN;
    const int32_t* rows = map + L.off_rows + tc.row_base;
    u32x4_t* Y = static_cast<u32x4_t*>(a.Y);
    constexpr int CPR = BN / 8;   // 8-column chunks per tile row
    for (int c = slice * 256 + threadIdx.x; c < tc.rows * CPR; c += 256 * kTailReduceSlices) {
        const int m = c / CPR, col = c - m * CPR;
        const float* src = base + (size_t)m * BN + col * 8;
        f32x4_t lo = *reinterpret_cast<const f32x4_t*>(src), hi = *reinterpret_cast<const f32x4_t*>(src + 4);
        for (int p = 1; p < ts.parts; ++p) {
            lo += *reinterpret_cast<const f32x4_t*>(src + (size_t)p * BMC * BN);
            hi += *reinterpret_cast<const f32x4_t*>(src + (size_t)p * BMC * BN + 4);
        }
        u32x4_t o;
        o.x = pack_bf16(lo[0], lo[1]); o.y = pack_bf16(lo[2], lo[3]);
        o.z = pack_bf16(hi[0], hi[1]); o.w = pack_bf16(hi[2], hi[3]);
        Y[((size_t)rows[m] * a.N + (size_t)tc.n_tile * BN) / 8 + col] = o;
    }
}

// ---- heterogeneous batching (Sec. 3.2, Alg. 3): GEMM tasks and one reduction task in the same launch

// 8-column chunks of output per tile of the reduction task: nu(reduction) = ceil(T * N / 8 / kReduceTileChunks).
constexpr int kReduceTileChunks = 4096;

// Tile l of the reduction task: the sum over a token's experts (see combine_range) for chunks
// [l * kReduceTileChunks, (l + 1) * kReduceTileChunks) of [red_T, red_N], run by all threads of the workgroup.
__device__ __forceinline__ void reduce_tile(const GemmArgs& a, int l, int nthreads) {
    const long long total = (long long)a.red_T * (a.red_N >> 3);
    const long long c0 = (long long)l * kReduceTileChunks;
    const long long c1 = c0 + kReduceTileChunks < total ? c0 + kReduceTileChunks : total;
    const u32x4_t* y = static_cast<const u32x4_t*>(a.red_Y);
    u32x4_t* o = static_cast<u32x4_t*>(a.red_out);
    switch (a.red_k) {
        case 2: combine_range<2>(y, a.red_w, o, 2, a.red_N, c0, c1, threadIdx.x, nthreads); break;
        case 6: combine_range<6>(y, a.red_w, o, 6, a.red_N, c0, c1, threadIdx.x, nthreads); break;
        case 8: combine_range<8>(y, a.red_w, o, 8, a.red_N, c0, c1, threadIdx.x, nthreads); break;
        default: combine_range<0>(y, a.red_w, o, a.red_k, a.red_N, c0, c1, threadIdx.x, nthreads); break;
    }
}

// One launch, two task types: the blocks of the GEMM tasks (all experts, as in moe_gemm_pipe_kernel) and the
// a.red_tiles blocks of one reduction task.  In the terms of Sec. 3.1 the batch's TilePrefix is the GEMM map's with
// one more entry, total_tiles + red_tiles, for the reduction task; a block at or beyond total_tiles belongs to it
// (the vote of Alg. 2 on that last entry) and runs the other task function (Alg. 3).  The reduction tiles only move
// memory, so every XCD walks its share of them spread in proportion over its share of the GEMM blocks (the
// placement idea of Sec. 4.2): they stream while the neighbours multiply.
template <class C, class... Tails>
__global__ __launch_bounds__(C::NT) void moe_gemm_batched_kernel(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int32_t* __restrict__ map = a.map;
    MapLayout L = map_layout(a.E);
    const int4 first_record = reinterpret_cast<const int4*>(map + L.off_records)[__lane_id()];
    const int total = map[MOE_HDR_TOTAL_TILES];
    if (!map_matches<C::BM, C::BN, 0, C::SLACK>(a, map)) return;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int ng = slots_of_xcd(map, total, xcd);
    const int r0 = (int)((long long)a.red_tiles * xcd >> 3), r1 = (int)((long long)a.red_tiles * (xcd + 1) >> 3);
    const int nr = r1 - r0, n = ng + nr;
    if (slot >= n) return;
    const int before = (int)((long long)slot * nr / n), upto = (int)((long long)(slot + 1) * nr / n);
    if (upto > before) {
        reduce_tile(a, r0 + before, C::NT);
        return;
    }
    int B;
    if (!slot_to_block(map, total, xcd, slot - before, B)) return;
    const moe_tiling g = {C::BM, C::BN, 0, 0, 0, C::SLACK};
    const TileCoord tc = decode_block(map, L, g, B, first_record);
    run_tile<C, Tails...>(a, map, L, tc, smem);
}

// Second half of a split-k product: Y[r(p), n] = bf16( sum_s partial[s][p][n] ), s ascending, for every position p of
// sorted_rows (r(p) = sorted_rows[p]); each lane owns 8 consecutive n of one position.  A map that is invalid,
// empty, or not the one this product was described with (the same header test as the product's own, locate_tile:
// shape, 256 x 256 tiles, one strategy, no slack, status 0) makes this a no-op, like the product itself: no tile
// ran then, the workspace holds nothing, and the row ids behind the header are not to be trusted.
__global__ __launch_bounds__(256) void moe_splitk_reduce_kernel(const float* __restrict__ partial, const int32_t* __restrict__ map,
                                                                const int32_t* __restrict__ sorted_rows, u32x4_t* __restrict__ Y,
                                                                int T, int k_top, int E, int N, int parts) {
    const bool hdr_ok = map[MOE_HDR_MAGIC] == MOE_MAP_MAGIC && map[MOE_HDR_T] == T && map[MOE_HDR_K_TOP] == k_top &&
                        map[MOE_HDR_E] == E && map[MOE_HDR_N] == N && map[MOE_HDR_TILE_M] == 256 &&
                        map[MOE_HDR_TILE_N] == 256 && map[MOE_HDR_STATUS] == 0 && map[MOE_HDR_TILE_M_SMALL] == 0 &&
                        map[MOE_HDR_SMALL_MAX_ROWS] == 0 && map[MOE_HDR_TILE_M_SLACK] == 0;
    if (!hdr_ok || map[MOE_HDR_TOTAL_TILES] == 0) return;
    const int R = T * k_top;
    const int cpr = N >> 3;
    const long long total = (long long)R * cpr;
    const size_t part_stride = (size_t)R * N;
    for (long long c = (long long)blockIdx.x * 256 + threadIdx.x; c < total; c += (long long)gridDim.x * 256) {
        const int p = (int)(c / cpr), col = (int)(c - (long long)p * cpr);
        const float* src = partial + (size_t)p * N + (size_t)col * 8;
        f32x4_t lo = *reinterpret_cast<const f32x4_t*>(src), hi = *reinterpret_cast<const f32x4_t*>(src + 4);
        for (int sp = 1; sp < parts; ++sp) {
            lo += *reinterpret_cast<const f32x4_t*>(src + sp * part_stride);
            hi += *reinterpret_cast<const f32x4_t*>(src + sp * part_stride + 4);
        }
        u32x4_t o;
        o.x = pack_bf16(lo[0], lo[1]); o.y = pack_bf16(lo[2], lo[3]);
        o.z = pack_bf16(hi[0], hi[1]); o.w = pack_bf16(hi[2], hi[3]);
        Y[(size_t)sorted_rows[p] * cpr + col] = o;
    }
}

}  // namespace moe
