// Task-map construction and decode for the statically batched MoE GEMM (gfx950).
//
// Builds, on the device, what Sec. 4.1 asks for after the token route: the
// per-expert counts, the list sigma of non-empty experts, the inclusive
// TilePrefix over the non-empty experts (Alg. 1), and the per-expert token
// index arrays of Sec. 4.3 (here a stable counting sort of the flat row ids,
// so the result does not depend on atomic ordering).  `mapping()` is Alg. 2
// for a 64-lane wavefront; `decode_block()` adds the sigma stage of Alg. 4.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/moe_sb.h"

namespace moe {

constexpr int kChunkRows = 1024;  // routed rows handled by one scatter workgroup
constexpr int kMapThreads = 1024; // = kChunkRows: one row per thread, 16 wavefronts
constexpr int kMaxE = 1024;
constexpr int kWaves = kMapThreads / 64;

struct MapLayout {
    int E64;
    size_t off_counts, off_offsets, off_sigma, off_prefix, off_records, off_rows;
};

__host__ __device__ inline MapLayout map_layout(int E) {
    MapLayout L;
    L.E64 = (E + 63) / 64 * 64;
    L.off_counts = MOE_MAP_HDR_WORDS;
    L.off_offsets = L.off_counts + L.E64;
    L.off_sigma = L.off_offsets + L.E64 + 64;
    L.off_prefix = L.off_sigma + L.E64;
    L.off_records = L.off_prefix + L.E64;
    L.off_rows = L.off_records + 4 * (size_t)L.E64;
    return L;
}

__host__ __device__ inline size_t round_up64(size_t v) { return (v + 63) / 64 * 64; }
// per-chunk histogram row: E64 expert columns + 64 spare (column E64 counts bad ids)
__host__ __device__ inline int hist_stride(int E64) { return E64 + 64; }

// ---------------------------------------------------------------- decode

// Alg. 2 on one wavefront: lane t tests p = (B >= TilePrefix[t]); the ballot is the
// warp vote, its population count is the task index h.  Pads are INT32_MAX and never vote.
// The prefix comes from the packed task records {TilePrefix, expert, count, row offset}, so the record of
// task h is already in a register of lane h when the vote is over: rec = that record, l = tile index in the task.
// More than 64 tasks (Sec. 3.1, two-level TilePrefix): the last entry of every group of 64 tasks is the
// first level; one vote over it (read in place, up to 64 groups) finds the group, a second vote the task in it.
// `first` is records[lane] (the caller loads it early, next to the header); B must be below the total tile count.
__device__ __forceinline__ void mapping(const int4* __restrict__ records, int E64, int B, int4 first, int& h, int& l, int4& rec) {
    const int lane = __lane_id();
    int4 r = first;
    int base = 0, kprev = 0;
    if (E64 > 64) {
        const int groups = E64 >> 6;  // <= 16 for E <= 1024
        const int top = lane < groups ? records[64 * lane + 63].x : 0x7fffffff;
        const int grp = __popcll(__ballot(B >= top));  // groups that end at or before B
        if (grp > 0) {
            base = grp << 6;
            kprev = __builtin_amdgcn_readlane(top, grp - 1);
            r = records[base + lane];
        }
    }
    const int votes = __popcll(__ballot(B >= r.x));  // < 64: the group's last entry is above B
    h = base + votes;
    rec.x = __builtin_amdgcn_readlane(r.x, votes);
    rec.y = __builtin_amdgcn_readlane(r.y, votes);
    rec.z = __builtin_amdgcn_readlane(r.z, votes);
    rec.w = __builtin_amdgcn_readlane(r.w, votes);
    if (votes > 0) kprev = __builtin_amdgcn_readlane(r.x, votes - 1);
    l = B - kprev;
}

struct TileCoord {
    int e, m_tile, n_tile, rows, row_base;  // row_base: index into sorted_rows of the tile's first row
    int small;                              // task type (Alg. 3): 1 = the expert uses the small tiling strategy
    int m_tiles;                            // m-tiles of the expert: 1 = no other tile reads this tile's weight panel
};

// Tiling strategy of an expert with cnt rows: tile_m_small when cnt <= small_max_rows (0 = one strategy).
__host__ __device__ __forceinline__ int expert_tile_m(int cnt, int tile_m, int tile_m_small, int small_max_rows) {
    return (small_max_rows > 0 && cnt <= small_max_rows) ? tile_m_small : tile_m;
}
// m-tiles of an expert with cnt rows.  With slack > 0 the last tile of a big-strategy expert may hold up to
// tile_m + slack rows, so a remainder of at most `slack` rows does not open a tile of its own.
__host__ __device__ __forceinline__ int expert_m_tiles(int cnt, const moe_tiling& g) {
    if (cnt <= 0) return 0;
    if (g.small_max_rows > 0 && cnt <= g.small_max_rows) return (cnt + g.tile_m_small - 1) / g.tile_m_small;
    const int mt = (cnt - g.tile_m_slack + g.tile_m - 1) / g.tile_m;
    return mt < 1 ? 1 : mt;
}

// Alg. 2 + Alg. 4 for workgroup B, then the tile index split m-fastest (the task function's own convention).
__device__ __forceinline__ TileCoord decode_block(const int32_t* __restrict__ map, const MapLayout& L, const moe_tiling& g, int B,
                                                  int4 first_record) {
    int h, l;
    int4 rec;
    mapping(reinterpret_cast<const int4*>(map + L.off_records), L.E64, B, first_record, h, l, rec);
    TileCoord c;
    c.e = rec.y;
    const int cnt = rec.z;
    c.small = g.small_max_rows > 0 && cnt <= g.small_max_rows;
    const int tile_m = c.small ? g.tile_m_small : g.tile_m;
    const int mt = expert_m_tiles(cnt, g);
    c.m_tiles = mt;
    c.n_tile = l / mt;
    c.m_tile = l - c.n_tile * mt;
    const int left = cnt - c.m_tile * tile_m;
    c.rows = c.m_tile + 1 < mt ? tile_m : left;
    c.row_base = rec.w + c.m_tile * tile_m;
    return c;
}

// ---------------------------------------------------------------- build

// Among the lanes of a wavefront holding the same key: my rank (lanes below me with
// my key) and the group size.  Invalid lanes take no part.
__device__ __forceinline__ void wave_match(int key, bool valid, int nbits, int& rank, int& size) {
    unsigned long long peers = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
        const int bit = (key >> b) & 1;
        const unsigned long long m = __ballot(bit);
        peers &= bit ? m : ~m;
    }
    const unsigned long long below = (1ull << __lane_id()) - 1ull;
    rank = __popcll(peers & below);
    size = __popcll(peers);
}

__device__ __forceinline__ int wave_incl_scan(int v) {
    const int lane = __lane_id();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}

// Inclusive scan across the 1024 threads of the block (s_tmp: >= 16 ints of LDS).
__device__ __forceinline__ int block_incl_scan(int v, int* s_tmp) {
    const int w = threadIdx.x >> 6, lane = __lane_id();
    const int incl = wave_incl_scan(v);
    __syncthreads();
    if (lane == 63) s_tmp[w] = incl;
    __syncthreads();
    int base = 0;
    for (int i = 0; i < w; ++i) base += s_tmp[i];
    return incl + base;
}

__device__ __forceinline__ int bit_reverse(int r, int nbits) { return nbits ? (int)(__brev((unsigned)r) >> (32 - nbits)) : 0; }

// From the per-expert count held by thread e (< E64; 0 beyond E): write counts, offsets,
// sigma, tile_prefix and the header.  Executed by all kMapThreads threads of one block.
// order 0: sigma ascending in expert index.  order 1 (spread, our reading of the interval-halving placement of
// Sec. 4.2): non-empty experts ranked by tile count (largest first, ties by lower index), rank r
// keyed by bitrev(r) over ceil(log2 M) bits, sigma by increasing key.
// s_work: >= 2*E64 ints of LDS.  Returns this thread's exclusive row offset (valid for tid < E).
__device__ __forceinline__ int finish_map(int32_t* __restrict__ map, const MapLayout& L, int cnt, int bad, int T, int k,
                                          int E, int N, const moe_tiling& g, int* s_tmp, int* s_work, bool write = true) {
    const int tid = threadIdx.x;
    const int R = T * k;
    const int nt = (N + g.tile_n - 1) / g.tile_n;
    const int nonempty = cnt > 0;
    const int tiles = expert_m_tiles(cnt, g) * nt;
    const int order = g.order;
    const int off_incl = block_incl_scan(cnt, s_tmp);
    const int ne_incl = block_incl_scan(nonempty, s_tmp);
    __syncthreads();
    if (tid == kMapThreads - 1) s_tmp[16] = ne_incl;
    __syncthreads();
    const int M = s_tmp[16];
    // position of this expert in sigma
    int pos = ne_incl - 1;
    if (order == 1) {
        if (tid < L.E64) s_work[tid] = nonempty ? tiles : -1;
        __syncthreads();
        int rank = 0;
        if (nonempty)
            for (int j = 0; j < L.E64; ++j) {
                const int tj = s_work[j];
                rank += (tj > tiles) || (tj == tiles && j < tid);
            }
        int nbits = 0;
        while ((1 << nbits) < M) ++nbits;
        const int key = bit_reverse(rank, nbits);
        if (tid < L.E64) s_work[L.E64 + tid] = nonempty ? key : 0x7fffffff;
        __syncthreads();
        pos = 0;
        if (nonempty)
            for (int j = 0; j < L.E64; ++j) pos += s_work[L.E64 + j] < key;
        __syncthreads();
    }
    // order 2: heavy experts (more than a quarter of an m-tile) by falling tile count, ties by lower index, then the
    // light ones by rising index; the tiles of the heavy part are summed for the header
    const bool light = 4 * cnt <= g.tile_m;
    if (tid == 0) s_tmp[18] = 0;
    if (order == 2) {
        const int heavy_key = light ? 0 : tiles;   // every heavy expert has at least one tile
        if (tid < L.E64) s_work[tid] = nonempty ? heavy_key : -1;
        __syncthreads();
        pos = 0;
        if (nonempty) {
            for (int j = 0; j < L.E64; ++j) {
                const int tj = s_work[j];
                pos += (tj > heavy_key) || (tj == heavy_key && j < tid);
            }
            if (!light) atomicAdd(&s_tmp[18], tiles);   // integer sum: the order of the adds does not matter
        }
        __syncthreads();
    }
    // `write` is false for the workgroups that only need the returned offsets (every scatter workgroup repeats
    // this function; the first one stores its results)
    if (tid < L.E64) {
        if (write) {
            map[L.off_counts + tid] = cnt;
            map[L.off_sigma + tid] = -1;
            map[L.off_records + 4 * tid + 1] = -1;
            map[L.off_records + 4 * tid + 2] = 0;
            map[L.off_records + 4 * tid + 3] = 0;
        }
        s_work[tid] = 0;
    }
    if (write)
        for (int i = tid; i < L.E64 + 64; i += kMapThreads) map[L.off_offsets + i] = i <= E ? 0 : R;
    __syncthreads();
    if (write && tid < E) map[L.off_offsets + tid] = off_incl - cnt;
    if (write && tid == 0) map[L.off_offsets + E] = R - bad;
    if (nonempty) {
        if (write) {
            map[L.off_sigma + pos] = tid;
            map[L.off_records + 4 * pos + 1] = tid;
            map[L.off_records + 4 * pos + 2] = cnt;
            map[L.off_records + 4 * pos + 3] = off_incl - cnt;
        }
        s_work[pos] = tiles;
    }
    __syncthreads();
    // Alg. 1 over the non-empty experts in sigma order
    const int tile_incl = block_incl_scan(tid < M ? s_work[tid] : 0, s_tmp);
    if (write && tid < L.E64) {
        map[L.off_prefix + tid] = tid < M ? tile_incl : 0x7fffffff;
        map[L.off_records + 4 * tid] = tid < M ? tile_incl : 0x7fffffff;
    }
    __syncthreads();
    if (tid == kMapThreads - 1) s_tmp[17] = tile_incl;
    __syncthreads();
    const int total = s_tmp[17];
    if (tid < MOE_MAP_HDR_WORDS) {
        int v = 0;
        switch (tid) {
            case MOE_HDR_MAGIC: v = MOE_MAP_MAGIC; break;
            case MOE_HDR_T: v = T; break;
            case MOE_HDR_K_TOP: v = k; break;
            case MOE_HDR_E: v = E; break;
            case MOE_HDR_N: v = N; break;
            case MOE_HDR_TILE_M: v = g.tile_m; break;
            case MOE_HDR_TILE_N: v = g.tile_n; break;
            case MOE_HDR_NT: v = nt; break;
            case MOE_HDR_M: v = M; break;
            case MOE_HDR_TOTAL_TILES: v = bad ? 0 : total; break;
            case MOE_HDR_ORDER: v = 0; break;
            case MOE_HDR_STATUS: v = bad; break;
            case MOE_HDR_R: v = R; break;
            case MOE_HDR_E64: v = L.E64; break;
            case MOE_HDR_SIGMA_ORDER: v = order; break;
            case MOE_HDR_TILE_M_SMALL: v = g.tile_m_small; break;
            case MOE_HDR_SMALL_MAX_ROWS: v = g.small_max_rows; break;
            case MOE_HDR_TILE_M_SLACK: v = g.tile_m_slack; break;
            case MOE_HDR_HEAVY_TILES: v = (order == 2 && !bad) ? s_tmp[18] : 0; break;
            default: v = 0;
        }
        if (write) map[tid] = v;
    }
    return off_incl - cnt;
}

__device__ __forceinline__ int key_bits(int E) {
    int nb = 1;
    while ((1 << nb) < E) ++nb;
    return nb;
}

// One-workgroup build for R <= kChunkRows: histogram, scans and stable scatter fused.
// Dynamic LDS: kWaves * E64 ints (per-wavefront counts) + E64 ints (offsets) + 32 + 2 * E64 (ordering).
__global__ __launch_bounds__(kMapThreads) void map_build_small(const int32_t* __restrict__ ids, int32_t* __restrict__ map,
                                                                int T, int k, int E, int N, moe_tiling g) {
    extern __shared__ int s_mem[];
    const MapLayout L = map_layout(E);
    int* s_wave = s_mem;                   // [kWaves][E64]
    int* s_off = s_mem + kWaves * L.E64;   // [E64]
    int* s_tmp = s_off + L.E64;            // [32]
    int* s_work = s_tmp + 32;              // [2*E64]
    const int tid = threadIdx.x, w = tid >> 6;
    const int R = T * k;
    for (int i = tid; i < kWaves * L.E64; i += kMapThreads) s_wave[i] = 0;
    if (tid == 0) s_tmp[31] = 0;
    __syncthreads();
    const bool in_range = tid < R;
    const int e = in_range ? ids[tid] : 0;
    const bool valid = in_range && e >= 0 && e < E;
    int rank, size;
    wave_match(e, valid, key_bits(E), rank, size);
    if (valid && rank == 0) s_wave[w * L.E64 + e] = size;
    const int nbad = __popcll(__ballot(in_range && !valid));
    if (nbad && __lane_id() == 0) atomicAdd(&s_tmp[31], nbad);
    __syncthreads();
    const int bad = s_tmp[31];
    int cnt = 0;
    if (tid < L.E64) {
        for (int i = 0; i < kWaves; ++i) {  // exclusive scan over wavefronts, in row order
            const int c = s_wave[i * L.E64 + tid];
            s_wave[i * L.E64 + tid] = cnt;
            cnt += c;
        }
    }
    const int off = finish_map(map, L, cnt, bad, T, k, E, N, g, s_tmp, s_work);
    if (tid < L.E64) s_off[tid] = off;
    __syncthreads();
    if (valid) map[L.off_rows + s_off[e] + s_wave[w * L.E64 + e] + rank] = tid;
}

// Multi-chunk path, step 1: per-chunk histogram (integer LDS atomics: order-free).
__global__ __launch_bounds__(256) void map_hist(const int32_t* __restrict__ ids, int R, int E, int E64,
                                                 int32_t* __restrict__ chunk_hist) {
    extern __shared__ int s_mem[];
    const int hs = hist_stride(E64);
    for (int i = threadIdx.x; i < hs; i += 256) s_mem[i] = 0;
    __syncthreads();
    const int base = blockIdx.x * kChunkRows;
    for (int i = threadIdx.x; i < kChunkRows; i += 256) {
        const int r = base + i;
        if (r < R) {
            const int e = ids[r];
            atomicAdd(&s_mem[(e >= 0 && e < E) ? e : E64], 1);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < hs; i += 256) chunk_hist[(size_t)blockIdx.x * hs + i] = s_mem[i];
}

// Multi-chunk path, step 2: every workgroup turns the chunk histograms into counts, offsets and its own chunk's
// bases (plain loads, no stores in between, so they pipeline), the first one also writes counts / offsets /
// sigma / TilePrefix / task records / header; then each scatters its chunk of rows, stably, into the token
// index arrays.  Repeating the scans in every workgroup costs less than a third kernel launch.
// Dynamic LDS: kWaves * E64 ints (per-wavefront counts) + E64 ints (this chunk's destination per expert).
__global__ __launch_bounds__(kMapThreads) void map_scan_scatter(const int32_t* __restrict__ ids, int32_t* __restrict__ map,
                                                                const int32_t* __restrict__ chunk_hist, int nchunks,
                                                                int T, int k, int E, int N, moe_tiling g) {
    extern __shared__ int s_mem[];
    __shared__ int s_tmp[32];
    __shared__ int s_work[2 * kMaxE];
    const MapLayout L = map_layout(E);
    const int hs = hist_stride(L.E64);
    int* s_wave = s_mem;                  // [kWaves][E64]
    int* s_off = s_mem + kWaves * L.E64;  // [E64]
    const int tid = threadIdx.x, w = tid >> 6;
    const int R = T * k;
    for (int i = tid; i < kWaves * L.E64; i += kMapThreads) s_wave[i] = 0;
    __syncthreads();
    const int r = blockIdx.x * kChunkRows + tid;
    const bool in_range = r < R;
    const int e = in_range ? ids[r] : 0;
    const bool valid = in_range && e >= 0 && e < E;
    int rank, size;
    wave_match(e, valid, key_bits(E), rank, size);
    if (valid && rank == 0) s_wave[w * L.E64 + e] = size;
    int cnt = 0, base = 0;
    if (tid < L.E64) {
        for (int c = 0; c < nchunks; ++c) {
            const int v = chunk_hist[(size_t)c * hs + tid];
            if (c < (int)blockIdx.x) base += v;
            cnt += v;
        }
    }
    if (tid == kMapThreads - 1) {
        int b = 0;
        for (int c = 0; c < nchunks; ++c) b += chunk_hist[(size_t)c * hs + L.E64];
        s_tmp[31] = b;
    }
    __syncthreads();
    const int bad = s_tmp[31];
    const int off = finish_map(map, L, cnt, bad, T, k, E, N, g, s_tmp, s_work, blockIdx.x == 0);
    if (tid < L.E64) {
        s_off[tid] = off + base;
        int run = 0;
        for (int i = 0; i < kWaves; ++i) {  // exclusive scan over wavefronts, in row order
            const int c = s_wave[i * L.E64 + tid];
            s_wave[i * L.E64 + tid] = run;
            run += c;
        }
    }
    __syncthreads();
    if (valid) map[L.off_rows + s_off[e] + s_wave[w * L.E64 + e] + rank] = r;
}

// Full per-block table from the compressed map, one wavefront per block index.
__global__ __launch_bounds__(256) void map_expand(const int32_t* __restrict__ map, int E, int32_t* __restrict__ table,
                                                   long long grid) {
    const MapLayout L = map_layout(E);
    const int total = map[MOE_HDR_TOTAL_TILES];
    moe_tiling g;
    g.tile_m = map[MOE_HDR_TILE_M]; g.tile_n = map[MOE_HDR_TILE_N]; g.order = map[MOE_HDR_SIGMA_ORDER];
    g.tile_m_small = map[MOE_HDR_TILE_M_SMALL]; g.small_max_rows = map[MOE_HDR_SMALL_MAX_ROWS];
    g.tile_m_slack = map[MOE_HDR_TILE_M_SLACK];
    const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long nwaves = (long long)gridDim.x * 4;
    for (long long B = wave; B < grid; B += nwaves) {
        int4 out = make_int4(-1, -1, -1, -1);
        if (B < total) {
            const TileCoord c = decode_block(map, L, g, (int)B, reinterpret_cast<const int4*>(map + L.off_records)[__lane_id()]);
            out = make_int4(c.e, c.m_tile, c.n_tile, c.rows);
        }
        if (__lane_id() == 0) reinterpret_cast<int4*>(table)[B] = out;
    }
}

}  // namespace moe
