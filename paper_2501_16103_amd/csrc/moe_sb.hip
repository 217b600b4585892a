// C-ABI entry points of libmoe_sb: argument checks, launch geometry, kernel selection.
// Everything that computes lives in task_map.hpp / gemm_kernel.hpp.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <mutex>
#include <type_traits>

#include "../../include/moe_sb.h"
#include "gemm_kernel.hpp"
#include "combine.hpp"
#include "task_map.hpp"

using namespace moe;

// Scratch memory of moe_grouped_gemm_splitk_static, the entry point for callers that cannot allocate: the fp32
// partial sums of a split-k product.  One copy per GPU, held until the process ends; host code reaches it only
// through the pointer hipGetSymbolAddress returns for the current device (static_scratch below).
constexpr size_t kStaticScratchBytes = size_t(32) << 20;
static __device__ __align__(256) float scratch[kStaticScratchBytes / sizeof(float)];

namespace {

bool tile_m_ok(int v) { return v == 16 || v == 32 || v == 64 || v == 128 || v == 256; }
bool tile_n_ok(int v) { return v == 64 || v == 128 || v == 256; }

int check_map_args(int T, int k, int E, int tile_m, int tile_n, int N) {
    if (T < 0 || k < 1 || E < 1 || k > E || N < 1) return MOE_ERR_INVALID_ARG;
    if (E > kMaxE) return MOE_ERR_UNSUPPORTED;
    if ((int64_t)T * k > (1 << 24)) return MOE_ERR_UNSUPPORTED;
    if (!tile_m_ok(tile_m) || !tile_n_ok(tile_n)) return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

// Guards the launch-attribute caches below (set once per kernel and device): calls may come from several host threads.
std::mutex g_attr_lock;

int nchunks_for(int64_t R) { return (int)((R + kChunkRows - 1) / kChunkRows); }

// `mode` is moe_gemm_desc.launch_mode (only the launches that have a resident form look at it)
typedef int (*gemm_launch_fn)(const GemmArgs&, int64_t grid, int mode, hipStream_t);

// The large-LDS attribute of a kernel is set once per device (bit d of *done: device d, d < 64).
inline int ensure_lds_attr(const void* fn, int lds, unsigned long long* done) {
    std::lock_guard<std::mutex> hold(g_attr_lock);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
    const unsigned long long bit = dev >= 0 && dev < 64 ? 1ull << dev : 0;
    if (bit && (*done & bit)) return MOE_OK;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess) return MOE_ERR_HIP;
    *done |= bit;
    return MOE_OK;
}

template <class C, class... Tails>
int launch_pipe(const GemmArgs& a, int64_t grid, int /*mode*/, hipStream_t s) {
    static unsigned long long attr_done = 0;
    if (ensure_lds_attr(reinterpret_cast<const void*>(&moe_gemm_pipe_kernel<C, Tails...>), C::LDS_BYTES, &attr_done) != MOE_OK)
        return MOE_ERR_HIP;
    moe_gemm_pipe_kernel<C, Tails...><<<dim3((unsigned)grid), dim3(C::NT), C::LDS_BYTES, s>>>(a);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// Split-k launch: `parts` workgroups per tile (grid.y), fp32 partial sums into a.partial.
template <class C, class... Tails>
int launch_splitk(const GemmArgs& a, int64_t grid, int parts, hipStream_t s) {
    static unsigned long long attr_done = 0;
    if (ensure_lds_attr(reinterpret_cast<const void*>(&moe_gemm_pipe_kernel<SplitK<C>, SplitK<Tails>...>), C::LDS_BYTES, &attr_done) != MOE_OK)
        return MOE_ERR_HIP;
    moe_gemm_pipe_kernel<SplitK<C>, SplitK<Tails>...><<<dim3((unsigned)grid, (unsigned)parts), dim3(C::NT), C::LDS_BYTES, s>>>(a);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// Heterogeneous launch: the GEMM tasks' blocks plus a.red_tiles blocks of the reduction task.
template <class C, class... Tails>
int launch_batched(const GemmArgs& a, int64_t grid, int /*mode*/, hipStream_t s) {
    static unsigned long long attr_done = 0;
    if (ensure_lds_attr(reinterpret_cast<const void*>(&moe_gemm_batched_kernel<C, Tails...>), C::LDS_BYTES, &attr_done) != MOE_OK)
        return MOE_ERR_HIP;
    moe_gemm_batched_kernel<C, Tails...><<<dim3((unsigned)grid), dim3(C::NT), C::LDS_BYTES, s>>>(a);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// Workgroups of `fn` that stay resident at once on the current device with `lds` bytes of dynamic LDS (also sets
// the kernel's large-LDS attribute); cached per kernel instance in *cache for the last (device, lds) asked for.
struct ResidentCache { int lds = -1, dev = -1, resident = 0; };
inline int resident_workgroups(const void* fn, int threads, int lds, ResidentCache* cache, int* resident) {
    std::lock_guard<std::mutex> hold(g_attr_lock);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
    if (lds != cache->lds || dev != cache->dev) {
        int cus = 0, per_cu = 0;
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, threads, lds) != hipSuccess || per_cu < 1 || cus < 8)
            return MOE_ERR_HIP;
        cache->resident = per_cu * cus / 8 * 8;
        cache->lds = lds;
        cache->dev = dev;
    }
    *resident = cache->resident;
    return MOE_OK;
}

// Streaming launch: as many workgroups as stay resident at once (grid is only an upper bound here).
template <class C>
int launch_stream(const GemmArgs& a, int64_t grid, int mode, hipStream_t s) {
    const int lds = C::LDS_BYTES + (C::FP8 ? 4 * (a.T + a.E) : 0);
    static ResidentCache cache;
    int resident = 0;
    if (resident_workgroups(reinterpret_cast<const void*>(&moe_gemm_stream_kernel<C>), C::NT, lds, &cache, &resident) != MOE_OK)
        return MOE_ERR_HIP;
    // with fewer than two tiles per resident workgroup there is nothing to stream across: one workgroup per tile
    if (mode == MOE_LAUNCH_PER_TILE || (mode == MOE_LAUNCH_AUTO && grid < 2 * (int64_t)resident))
        return launch_pipe<C>(a, grid, mode, s);
    int64_t g = grid < resident ? grid : resident;
    if (mode >= 8 && g > mode) g = mode / 8 * 8;
    moe_gemm_stream_kernel<C><<<dim3((unsigned)g), dim3(C::NT), lds, s>>>(a);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

template <class CBIG, class CSMALL, class... Tails>
int launch_pipe2(const GemmArgs& a, int64_t grid, int /*mode*/, hipStream_t s) {
    constexpr int lds = CBIG::LDS_BYTES > CSMALL::LDS_BYTES ? CBIG::LDS_BYTES : CSMALL::LDS_BYTES;
    static unsigned long long attr_done = 0;
    if (ensure_lds_attr(reinterpret_cast<const void*>(&moe_gemm_pipe2_kernel<CBIG, CSMALL, Tails...>), lds, &attr_done) != MOE_OK)
        return MOE_ERR_HIP;
    moe_gemm_pipe2_kernel<CBIG, CSMALL, Tails...><<<dim3((unsigned)grid), dim3(CBIG::NT), lds, s>>>(a);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

struct GemmVariant {
    int dtype, tile_m, tile_n, bk;
    gemm_launch_fn fn;
    int tile_m_small = 0;  // second tiling strategy handled by the same launch (0 = none)
    int tile_m_slack = 0;  // rows the last m-tile may hold beyond tile_m
    int w_layout = MOE_W_LAYOUT_KN;
    // the same tile as a streaming launch (resident workgroups run several tiles back to back), or nullptr
    gemm_launch_fn fn_stream = nullptr;
    int ring = 0;  // ring depth of the streaming kernel: it needs K / bk >= ring
    // the same GEMM tasks batched with a reduction task in one launch (moe_grouped_gemm_batched), or nullptr
    gemm_launch_fn fn_batched = nullptr;
};

// Pipelined bf16 kernels:  BM   BN   BK  WM WN  ring stages
// The large tiles run on 16x16x32 MFMA blocks: same LDS traffic and accumulator count as 32x32x16, but the chip
// sustains about 13 % more of them on random operands before its power limit lowers the clock.
using Pb_256x256 = PipeCfg<256, 256, 64, 2, 4, 2, false, 3, 0, false, 16>;
// same, for maps whose last m-tiles hold up to 64 slack rows
using Pb_256x256s = PipeCfg<256, 256, 64, 2, 4, 2, false, 2, 64>;
// (token ring 2 x 40 KB; the 80 KB left hold five half-stages of weights: 2.5 k-tiles instead of 2)
using Pb_256x256s32 = PipeCfg<256, 256, 64, 2, 4, 2, false, 2, 32, false, 16, 5>;
// (eight wavefronts of 128 x 32: two per SIMD keep MFMAs and LDS reads of different wavefronts overlapping;
// against four wavefronts of 128 x 64: -1 % on mixtral_up T=256 / 384, -7 % on a 1536-row down projection)
using Pb_128x256 = PipeCfg<128, 256, 64, 1, 8, 3>;
using Pb_128x128 = PipeCfg<128, 128, 64, 2, 4, 4>;   // eight wavefronts of 64 x 32 (-1 ... -7 % against four of 64 x 64)
using Pb_64x256 = PipeCfg<64, 256, 64, 1, 4, 3>;
using Pb_64x128 = PipeCfg<64, 128, 64, 1, 4, 3>;   // 72 KB: two workgroups per CU
using Pb_32x256 = PipeCfg<32, 256, 64, 1, 4, 4>;
using Pb_32x128 = PipeCfg<32, 128, 64, 1, 4, 6>;
// Narrow task functions that share the launch shape (512 threads, 256-wide n-tiles) of Pb_256x256: used for its
// partly filled tiles and as the small-expert strategy of a two-strategy launch
using Ps_64x256 = PipeCfg<64, 256, 64, 1, 8, 3>;
using Ps_128x256 = PipeCfg<128, 256, 64, 1, 8, 2>;
// 16-row tiles (two wavefronts) and fp8: the weight stream starts before the token rows are known
using Pb_16x256 = PipeCfg<16, 256, 64, 1, 2, 2>;
using Pb_16x128 = PipeCfg<16, 128, 64, 1, 2, 4>;
using P8_16x256 = PipeCfg<16, 256, 128, 1, 2, 2, true>;
using P8_16x128 = PipeCfg<16, 128, 128, 1, 2, 4, true>;
using P8_16x64 = PipeCfg<16, 64, 128, 1, 2, 4, true>;
using P8_32x128 = PipeCfg<32, 128, 128, 1, 2, 4, true>;
// fp8 at prefill sizes: the 256 x 256 launch shape with its two narrow task functions, and a 64-row tile
using P8_256x256 = PipeCfg<256, 256, 128, 2, 4, 2, true, 3>;
using P8s_64x256 = PipeCfg<64, 256, 128, 1, 8, 3, true>;
using P8s_128x256 = PipeCfg<128, 256, 128, 1, 8, 2, true>;
using P8_64x256 = PipeCfg<64, 256, 128, 1, 4, 3, true>;

// The pre-packed weight layout [E][N][K] (K contiguous): the shapes the benchmark uses
using Pk_256x256 = PipeCfg<256, 256, 64, 2, 4, 2, false, 3, 0, true, 16>;
using Pk_256x256s = PipeCfg<256, 256, 64, 2, 4, 2, false, 2, 64, true>;
using Pks_64x256 = PipeCfg<64, 256, 64, 1, 8, 3, false, 3, 0, true>;
using Pks_128x256 = PipeCfg<128, 256, 64, 1, 8, 2, false, 2, 0, true>;
using Pk_128x256 = PipeCfg<128, 256, 64, 1, 4, 3, false, 3, 0, true>;
using Pk_16x256 = PipeCfg<16, 256, 64, 1, 2, 2, false, 2, 0, true>;
using P8k_16x256 = PipeCfg<16, 256, 128, 1, 2, 2, true, 2, 0, true>;
using P8k_16x128 = PipeCfg<16, 128, 128, 1, 2, 4, true, 4, 0, true>;

const GemmVariant kVariants[] = {
    {MOE_DTYPE_BF16, 256, 256, 64, &launch_pipe<Pk_256x256, Pks_64x256, Pks_128x256>, 0, 0, MOE_W_LAYOUT_NK},
    {MOE_DTYPE_BF16, 256, 256, 64, &launch_pipe<Pk_256x256s, Pks_64x256, Pks_128x256>, 0, 64, MOE_W_LAYOUT_NK},
    {MOE_DTYPE_BF16, 128, 256, 64, &launch_pipe<Pk_128x256>, 0, 0, MOE_W_LAYOUT_NK},
    {MOE_DTYPE_BF16, 16, 256, 64, &launch_pipe<Pk_16x256>, 0, 0, MOE_W_LAYOUT_NK},
    {MOE_DTYPE_FP8_E4M3, 16, 256, 128, &launch_pipe<P8k_16x256>, 0, 0, MOE_W_LAYOUT_NK},
    {MOE_DTYPE_FP8_E4M3, 16, 128, 128, &launch_pipe<P8k_16x128>, 0, 0, MOE_W_LAYOUT_NK},
    {MOE_DTYPE_BF16, 256, 256, 64, &launch_pipe<Pb_256x256, Ps_64x256, Ps_128x256>, 0, 0, MOE_W_LAYOUT_KN, nullptr, 0,
     &launch_batched<Pb_256x256, Ps_64x256, Ps_128x256>},
    {MOE_DTYPE_BF16, 256, 256, 64, &launch_pipe<Pb_256x256s, Ps_64x256, Ps_128x256>, 0, 64},
    {MOE_DTYPE_BF16, 256, 256, 64, &launch_pipe<Pb_256x256s32, Ps_64x256, Ps_128x256>, 0, 32, MOE_W_LAYOUT_KN, nullptr, 0,
     &launch_batched<Pb_256x256s32, Ps_64x256, Ps_128x256>},
    {MOE_DTYPE_BF16, 128, 256, 64, &launch_pipe<Pb_128x256, Ps_64x256>},
    {MOE_DTYPE_BF16, 128, 128, 64, &launch_pipe<Pb_128x128>},
    {MOE_DTYPE_BF16, 64, 256, 64, &launch_pipe<Pb_64x256>},
    {MOE_DTYPE_BF16, 64, 128, 64, &launch_pipe<Pb_64x128>},
    {MOE_DTYPE_BF16, 32, 256, 64, &launch_pipe<Pb_32x256>},
    {MOE_DTYPE_BF16, 32, 128, 64, &launch_pipe<Pb_32x128>},
    {MOE_DTYPE_BF16, 16, 256, 64, &launch_pipe<Pb_16x256>, 0, 0, MOE_W_LAYOUT_KN, &launch_stream<Pb_16x256>, Pb_16x256::NS},
    {MOE_DTYPE_BF16, 16, 128, 64, &launch_pipe<Pb_16x128>, 0, 0, MOE_W_LAYOUT_KN, &launch_stream<Pb_16x128>, Pb_16x128::NS},
    {MOE_DTYPE_FP8_E4M3, 16, 256, 128, &launch_pipe<P8_16x256>, 0, 0, MOE_W_LAYOUT_KN, &launch_stream<P8_16x256>, P8_16x256::NS},
    {MOE_DTYPE_FP8_E4M3, 16, 128, 128, &launch_pipe<P8_16x128>, 0, 0, MOE_W_LAYOUT_KN, &launch_stream<P8_16x128>, P8_16x128::NS},
    {MOE_DTYPE_FP8_E4M3, 16, 64, 128, &launch_pipe<P8_16x64>, 0, 0, MOE_W_LAYOUT_KN, &launch_stream<P8_16x64>, P8_16x64::NS},
    {MOE_DTYPE_FP8_E4M3, 32, 128, 128, &launch_pipe<P8_32x128>},
    {MOE_DTYPE_FP8_E4M3, 256, 256, 128, &launch_pipe<P8_256x256, P8s_64x256, P8s_128x256>},
    {MOE_DTYPE_FP8_E4M3, 64, 256, 128, &launch_pipe<P8_64x256>},
};

const GemmVariant kPairVariants[] = {
    {MOE_DTYPE_BF16, 256, 256, 64, &launch_pipe2<Pb_256x256, Ps_64x256, Ps_64x256, Ps_128x256>, 64},
    {MOE_DTYPE_BF16, 256, 256, 64, &launch_pipe2<Pb_256x256, Ps_128x256, Ps_64x256, Ps_128x256>, 128},
};

const GemmVariant* find_variant(int dtype, int tile_m, int tile_n, int tile_m_small = 0, int tile_m_slack = 0,
                                int w_layout = MOE_W_LAYOUT_KN) {
    if (tile_m_small == 0) {
        for (const GemmVariant& v : kVariants)
            if (v.dtype == dtype && v.tile_m == tile_m && v.tile_n == tile_n && v.tile_m_slack == tile_m_slack &&
                v.w_layout == w_layout)
                return &v;
    } else {
        for (const GemmVariant& v : kPairVariants)
            if (v.dtype == dtype && v.tile_m == tile_m && v.tile_n == tile_n && v.tile_m_small == tile_m_small &&
                v.tile_m_slack == tile_m_slack && v.w_layout == w_layout)
                return &v;
    }
    return nullptr;
}

int check_small_args(int tile_m, int tile_m_small, int small_max_rows, int tile_m_slack = 0) {
    if (tile_m_slack < 0 || tile_m_slack >= tile_m) return MOE_ERR_INVALID_ARG;
    if (tile_m_small == 0 && small_max_rows == 0) return MOE_OK;
    if (tile_m_small != 16 && tile_m_small != 32 && tile_m_small != 64 && tile_m_small != 128) return MOE_ERR_UNSUPPORTED;
    if (tile_m_small >= tile_m) return MOE_ERR_INVALID_ARG;
    if (small_max_rows < 1 || small_max_rows > 4 * tile_m_small) return MOE_ERR_INVALID_ARG;
    return MOE_OK;
}

// moe_grouped_gemm, optionally with a reduction task batched into the same launch (red != nullptr).
int grouped_gemm_impl(const void* X, const void* W, const void* task_map, void* Y, const moe_gemm_desc* d,
                      const moe_reduce_task* red, void* stream) {
    if (!d || !task_map) return MOE_ERR_INVALID_ARG;
    const int rc = check_map_args(d->T, d->k, d->E, d->tile_m, d->tile_n, d->N);
    if (rc != MOE_OK) return rc;
    if (d->K < 1) return MOE_ERR_INVALID_ARG;
    if (d->dtype != MOE_DTYPE_BF16 && d->dtype != MOE_DTYPE_FP8_E4M3) return MOE_ERR_UNSUPPORTED;
    {
        const int rcs = check_small_args(d->tile_m, d->tile_m_small, d->small_max_rows, d->tile_m_slack);
        if (rcs != MOE_OK) return rcs;
    }
    if (d->w_layout != MOE_W_LAYOUT_KN && d->w_layout != MOE_W_LAYOUT_NK) return MOE_ERR_INVALID_ARG;
    if (d->launch_mode < 0) return MOE_ERR_INVALID_ARG;
    const GemmVariant* v = find_variant(d->dtype, d->tile_m, d->tile_n, d->tile_m_small, d->tile_m_slack, d->w_layout);
    if (!v) return MOE_ERR_UNSUPPORTED;
    if (red && !v->fn_batched) return MOE_ERR_UNSUPPORTED;
    if (d->K % v->bk != 0 || d->N % d->tile_n != 0) return MOE_ERR_UNSUPPORTED;
    if (d->epilogue != MOE_EPILOGUE_NONE && d->epilogue != MOE_EPILOGUE_SWIGLU) return MOE_ERR_INVALID_ARG;
    const int es = d->dtype == MOE_DTYPE_FP8_E4M3 ? 1 : 2;
    if ((int64_t)d->T * d->K * es >= (int64_t)1 << 32) return MOE_ERR_UNSUPPORTED;
    const int64_t red_tiles = red ? moe_reduce_task_tiles(red->T, red->N) : 0;
    if (d->T == 0 && red_tiles == 0) return MOE_OK;
    if (d->T > 0) {
        if (!X || !W || !Y) return MOE_ERR_INVALID_ARG;
        if (((uintptr_t)X & 15) || ((uintptr_t)W & 15) || ((uintptr_t)Y & 15)) return MOE_ERR_INVALID_ARG;
        if (d->dtype == MOE_DTYPE_FP8_E4M3 && (!d->x_scale || !d->w_scale)) return MOE_ERR_INVALID_ARG;
    }
    if ((uintptr_t)task_map & 15) return MOE_ERR_INVALID_ARG;
    GemmArgs a{};
    a.X = X; a.W = W; a.map = static_cast<const int32_t*>(task_map); a.Y = Y;
    a.x_scale = d->x_scale; a.w_scale = d->w_scale;
    a.T = d->T; a.k = d->k; a.E = d->E; a.K = d->K; a.N = d->N;
    a.tile_m_small = d->tile_m_small; a.small_max_rows = d->small_max_rows; a.tile_m_slack = d->tile_m_slack;
    a.swiglu = d->epilogue == MOE_EPILOGUE_SWIGLU;
    a.partial = nullptr;
    if (red_tiles > 0) {
        a.red_Y = red->Y; a.red_w = red->topk_weights; a.red_out = red->out;
        a.red_T = red->T; a.red_k = red->k; a.red_N = red->N; a.red_tiles = (int)red_tiles;
    }
    int64_t grid = moe_grid_upper_bound_tiled(d->T, d->k, d->E, d->tile_m, d->tile_n, d->N, d->tile_m_small,
                                              d->small_max_rows) + red_tiles;
    if (grid == 0) return MOE_OK;
    grid = (grid + 7) / 8 * 8 + 16;  // spare slots per XCD: the interleaved dealings round their shares up
    if (grid > 0x7fffffff) return MOE_ERR_UNSUPPORTED;
    if (red) return v->fn_batched(a, grid, d->launch_mode, static_cast<hipStream_t>(stream));
    // weight-streaming tiles: keep the workgroups resident and stream tile after tile where the shape allows it
    const bool can_stream = v->fn_stream && d->E <= 256 && d->K / v->bk >= v->ring &&
                            (d->dtype != MOE_DTYPE_FP8_E4M3 || d->T + d->E <= 2048) && d->launch_mode != MOE_LAUNCH_PER_TILE;
    return (can_stream ? v->fn_stream : v->fn)(a, grid, d->launch_mode, static_cast<hipStream_t>(stream));
}

// ---- split-k: shared by the entry point that takes a workspace and by the one that allocates nothing

int check_splitk_args(const moe_gemm_desc* d, int k_parts) {
    if (!d) return MOE_ERR_INVALID_ARG;
    if (d->T < 0 || d->k < 1 || d->E < 1 || d->E > kMaxE || d->k > d->E || d->K < 1 || d->N < 1) return MOE_ERR_INVALID_ARG;
    if (d->dtype != MOE_DTYPE_BF16 || d->w_layout != MOE_W_LAYOUT_KN || d->epilogue != MOE_EPILOGUE_NONE ||
        d->tile_m != 256 || d->tile_n != 256 || d->tile_m_small != 0 || d->small_max_rows != 0 || d->tile_m_slack != 0)
        return MOE_ERR_UNSUPPORTED;
    if (k_parts != 2 && k_parts != 4) return MOE_ERR_UNSUPPORTED;
    if (d->K % 64 != 0 || (d->K / 64) % k_parts != 0 || d->K / 64 / k_parts < 8 || d->N % 256 != 0) return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

// The two launches of a split-k product (arguments already checked by check_splitk_args, T > 0): the product with
// k_parts workgroups per tile leaves fp32 partial sums in `ws`, the reduction adds them and scatters.
int run_splitk(const void* X, const void* W, const void* task_map, void* Y, const moe_gemm_desc* d, int k_parts, float* ws,
               hipStream_t s) {
    if (!X || !W || !task_map || !Y || !ws) return MOE_ERR_INVALID_ARG;
    if (((uintptr_t)X & 15) || ((uintptr_t)W & 15) || ((uintptr_t)Y & 15) || ((uintptr_t)task_map & 15)) return MOE_ERR_INVALID_ARG;
    GemmArgs a{};
    a.X = X; a.W = W; a.map = static_cast<const int32_t*>(task_map); a.Y = Y;
    a.T = d->T; a.k = d->k; a.E = d->E; a.K = d->K; a.N = d->N;
    a.tile_m_slack = d->tile_m_slack;
    a.partial = ws;
    int64_t grid = moe_grid_upper_bound_tiled(d->T, d->k, d->E, 256, 256, d->N, 0, 0);
    if (grid == 0) return MOE_OK;
    grid = (grid + 7) / 8 * 8 + 8;
    if (grid > 0x7fffffff) return MOE_ERR_UNSUPPORTED;
    const int rc = launch_splitk<Pb_256x256, Ps_64x256, Ps_128x256>(a, grid, k_parts, s);
    if (rc != MOE_OK) return rc;
    const int64_t R = (int64_t)d->T * d->k;
    const long long chunks = (long long)R * (d->N / 8);
    long long blocks = (chunks + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    const MapLayout L = map_layout(d->E);
    moe_splitk_reduce_kernel<<<(unsigned)blocks, 256, 0, s>>>(a.partial, a.map, a.map + L.off_rows, static_cast<u32x4_t*>(Y), d->T,
                                                             d->k, d->E, d->N, k_parts);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// ---- tail split (see tail_parts in gemm_kernel.hpp); MI355X: 8 XCDs of 32 CUs
constexpr int kCusPerXcd = 32;
static_assert(kTailBlocksPerXcd >= 4 * (kCusPerXcd - 1), "workspace blocks per XCD");

size_t tail_workspace_bytes(int tile_m, int tile_n) {   // (256-row blocks with room for 32 slack rows)
    return size_t(8) * kTailBlocksPerXcd * (tile_m == 256 ? 288 : tile_m) * tile_n * sizeof(float);
}

// The three launches of a tail-split product: whole tiles, the parts of the tail tiles, their sums.
template <class C, class... Tails>
int launch_tail_split(const GemmArgs& a, int64_t grid, hipStream_t s) {
    const int r1 = launch_pipe<C, Tails...>(a, grid, 0, s);
    if (r1 != MOE_OK) return r1;
    using TailC = SplitK<C>;
    static unsigned long long attr_done = 0;
    const void* fn = reinterpret_cast<const void*>(&moe_gemm_tail_kernel<TailC, SplitK<Tails>...>);
    if (ensure_lds_attr(fn, TailC::LDS_BYTES, &attr_done) != MOE_OK) return MOE_ERR_HIP;
    moe_gemm_tail_kernel<TailC, SplitK<Tails>...><<<dim3(8 * kTailBlocksPerXcd), dim3(TailC::NT), TailC::LDS_BYTES, s>>>(a);
    if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
    moe_tail_reduce_kernel<C::BM, C::BN, C::SLACK><<<dim3(8 * kCusPerXcd * kTailReduceSlices), dim3(256), 0, s>>>(a);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// This device's address of the static scratch array, looked up once per device (with that device current) and
// kept: every GPU the library runs on holds its own copy of the array at its own address.  In host code the
// array's name is only a handle for this lookup, never a device address.
int static_scratch(float** out) {
    static float* ptr_of_device[64] = {};
    std::lock_guard<std::mutex> hold(g_attr_lock);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
    if (dev < 0 || dev >= 64) return MOE_ERR_UNSUPPORTED;
    if (!ptr_of_device[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MOE_ERR_HIP;
        ptr_of_device[dev] = static_cast<float*>(p);
    }
    *out = ptr_of_device[dev];
    return MOE_OK;
}

}  // namespace

extern "C" {

size_t moe_map_off_counts(int E) { return map_layout(E).off_counts; }
size_t moe_map_off_offsets(int E) { return map_layout(E).off_offsets; }
size_t moe_map_off_sigma(int E) { return map_layout(E).off_sigma; }
size_t moe_map_off_tile_prefix(int E) { return map_layout(E).off_prefix; }
size_t moe_map_off_task_records(int E) { return map_layout(E).off_records; }
size_t moe_map_off_sorted_rows(int E) { return map_layout(E).off_rows; }

size_t moe_task_map_bytes(int T_max, int k, int E, int tile_m, int tile_n, int N) {
    if (check_map_args(T_max, k, E, tile_m, tile_n, N) != MOE_OK) return 0;
    const MapLayout L = map_layout(E);
    const int64_t R = (int64_t)T_max * k;
    const size_t words = L.off_rows + round_up64((size_t)R) + (size_t)nchunks_for(R) * hist_stride(L.E64) + 64;
    return words * sizeof(int32_t);
}

int64_t moe_grid_upper_bound(int T, int k, int E, int tile_m, int tile_n, int N) {
    if (check_map_args(T, k, E, tile_m, tile_n, N) != MOE_OK) return 0;
    const int64_t R = (int64_t)T * k;
    const int64_t nt = (N + tile_n - 1) / tile_n;
    return (R / tile_m + (E < R ? E : R)) * nt;
}

int moe_build_task_map(const int32_t* topk_ids, int T, int k, int E, int tile_m, int tile_n, int N, void* task_map,
                       void* stream) {
    return moe_build_task_map_ordered(topk_ids, T, k, E, tile_m, tile_n, N, MOE_ORDER_ASCENDING, task_map, stream);
}

int moe_build_task_map_ordered(const int32_t* topk_ids, int T, int k, int E, int tile_m, int tile_n, int N, int order,
                               void* task_map, void* stream) {
    return moe_build_task_map_tiled(topk_ids, T, k, E, tile_m, tile_n, N, order, 0, 0, task_map, stream);
}

int64_t moe_grid_upper_bound_tiled(int T, int k, int E, int tile_m, int tile_n, int N, int tile_m_small,
                                   int small_max_rows) {
    if (check_map_args(T, k, E, tile_m, tile_n, N) != MOE_OK) return 0;
    if (check_small_args(tile_m, tile_m_small, small_max_rows) != MOE_OK) return 0;
    const int64_t R = (int64_t)T * k;
    const int64_t nt = (N + tile_n - 1) / tile_n;
    const int64_t per_expert = tile_m_small ? (small_max_rows + tile_m_small - 1) / tile_m_small : 1;
    return (R / tile_m + (E < R ? E : R) * (per_expert > 1 ? per_expert : 1)) * nt;
}

int moe_tile_pair_supported(int dtype, int tile_m, int tile_n, int tile_m_small) {
    return tile_m_small > 0 && find_variant(dtype, tile_m, tile_n, tile_m_small) != nullptr;
}

int moe_build_task_map_tiled(const int32_t* topk_ids, int T, int k, int E, int tile_m, int tile_n, int N, int order,
                             int tile_m_small, int small_max_rows, void* task_map, void* stream) {
    const moe_tiling g = {tile_m, tile_n, order, tile_m_small, small_max_rows, 0};
    return moe_build_task_map_ex(topk_ids, T, k, E, N, &g, task_map, stream);
}

int moe_default_tiling(int dtype, int T, int k, int E, int K, int N, moe_tiling* out) {
    if (!out || T < 0 || k < 1 || E < 1 || k > E || K < 1 || N < 1) return MOE_ERR_INVALID_ARG;
    if (dtype != MOE_DTYPE_BF16 && dtype != MOE_DTYPE_FP8_E4M3) return MOE_ERR_INVALID_ARG;
    const int64_t R = (int64_t)T * k;
    const double mean_rows = (double)R / E;
    const int64_t active = R < E ? R : E;   // experts that can have rows at all
    const int cus = 256;
    moe_tiling g = {16, 128, MOE_ORDER_ASCENDING, 0, 0, 0};
    if (dtype == MOE_DTYPE_FP8_E4M3 && mean_rows > 24) {
        // prefill sizes
        g.tile_m = mean_rows > 96 ? 256 : 64; g.tile_n = 256;
    } else if (dtype == MOE_DTYPE_FP8_E4M3) {
        // expected tiles under a uniform routing: E * (1 - (1 - 1/E)^R) experts are hit, plus full extra m-tiles
        const double hit = E * (1.0 - pow(1.0 - 1.0 / E, (double)R));
        const double t256 = (hit + (double)(R / 16)) * ((N + 255) / 256);
        g.tile_m = 16;
        g.tile_n = (N % 256 == 0 && t256 >= cus && t256 <= 2 * cus) ? 256 : 128;
    } else if (mean_rows <= 48 && active * ((N + 255) / 256) < cus && N % 128 == 0) {
        // too few 256-wide tiles to give every CU one: halve the tile width; 128 rows also hold a skewed
        // routing's busiest expert in one tile
        g.tile_m = 128; g.tile_n = 128;
    } else if (mean_rows <= 8) {
        // nearly every expert's rows fit one 16-row tile (count ~ mean +- 3 sqrt(mean))
        g.tile_m = 16; g.tile_n = 256;
    } else {
        // expected tiles of a tiling under a balanced routing: counts spread around the mean, so an expert takes
        // mean / tile_m + 1/2 m-tiles on average, and at least one
        auto tiles = [&](int tm, int tn) {
            const double mt = mean_rows / tm + 0.5;
            return (double)active * (mt < 1.0 ? 1.0 : mt) * ((N + tn - 1) / tn);
        };
        bool short_grid;
        if (mean_rows > 48 && mean_rows <= 96) {
            // counts straddle 64: the four-wave 64- and 128-row functions of the 128-row launch
            g.tile_m = active * ((N + 255) / 256) >= 3 * cus ? 128 : 64;
            g.tile_n = 256;
            short_grid = active * ((N + 255) / 256) < cus;
        } else {
            // 256-row tiles; their launch runs tiles of at most 64 / 128 rows with narrower task functions, which
            // covers the small counts too.  Slack rows pay once experts hold several tiles.
            g.tile_m = 256; g.tile_n = 256; g.tile_m_slack = mean_rows > 192 ? 32 : 0;
            short_grid = tiles(256, 256) < 0.75 * cus;
        }
        if (short_grid) {
            // few experts and a narrow N (a down projection at a few hundred tokens): the launch would leave CUs
            // idle through a long k loop.  Take the largest tile that still gives three quarters of the CUs one.
            const int cand[3][2] = {{128, 256}, {128, 128}, {64, 128}};
            for (int c = 0; c < 3; ++c) {
                if (N % cand[c][1] != 0) continue;
                g.tile_m = cand[c][0]; g.tile_n = cand[c][1]; g.tile_m_slack = 0;
                if (tiles(cand[c][0], cand[c][1]) >= 0.75 * cus) break;
            }
        }
    }
    // the n-tile must divide N; narrower tiles keep the same row tiling where a kernel exists
    for (int tn = g.tile_n; tn >= 64; tn >>= 1) {
        if (N % tn != 0) continue;
        moe_tiling c = g;
        c.tile_n = tn;
        if (find_variant(dtype, c.tile_m, c.tile_n, 0, c.tile_m_slack)) { *out = c; return MOE_OK; }
        c.tile_m_slack = 0;
        if (find_variant(dtype, c.tile_m, c.tile_n, 0, 0)) { *out = c; return MOE_OK; }
        for (int tm : {128, 64, 32, 16}) {
            c.tile_m = tm;
            if (tm <= g.tile_m && find_variant(dtype, tm, tn, 0, 0)) { *out = c; return MOE_OK; }
        }
    }
    return MOE_ERR_UNSUPPORTED;
}

int moe_tiling_supported(int dtype, const moe_tiling* g) {
    if (!g || check_small_args(g->tile_m, g->tile_m_small, g->small_max_rows, g->tile_m_slack) != MOE_OK) return 0;
    return find_variant(dtype, g->tile_m, g->tile_n, g->tile_m_small, g->tile_m_slack) != nullptr;
}

int moe_build_task_map_ex(const int32_t* topk_ids, int T, int k, int E, int N, const moe_tiling* tiling,
                          void* task_map, void* stream) {
    if (!tiling) return MOE_ERR_INVALID_ARG;
    const moe_tiling g = *tiling;
    const int tile_m = g.tile_m, tile_n = g.tile_n, order = g.order;
    if (!task_map || (T > 0 && !topk_ids)) return MOE_ERR_INVALID_ARG;
    if (tile_m < 1) return MOE_ERR_UNSUPPORTED;
    {
        const int rcs = check_small_args(tile_m, g.tile_m_small, g.small_max_rows, g.tile_m_slack);
        if (rcs != MOE_OK) return rcs;
    }
    if (order != MOE_ORDER_ASCENDING && order != MOE_ORDER_SPREAD && order != MOE_ORDER_INTERLEAVE) return MOE_ERR_INVALID_ARG;
    if (((uintptr_t)task_map & 15) || ((uintptr_t)topk_ids & 3)) return MOE_ERR_INVALID_ARG;
    const int rc = check_map_args(T, k, E, tile_m, tile_n, N);
    if (rc != MOE_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t* map = static_cast<int32_t*>(task_map);
    const MapLayout L = map_layout(E);
    const int64_t R = (int64_t)T * k;
    if (R <= kChunkRows) {
        const size_t lds = ((size_t)kWaves * L.E64 + L.E64 + 32 + 2 * (size_t)L.E64) * sizeof(int);
        static unsigned long long attr_done = 0;
        if (ensure_lds_attr(reinterpret_cast<const void*>(&map_build_small),
                            (int)(((size_t)kWaves * kMaxE + 3 * (size_t)kMaxE + 32) * sizeof(int)), &attr_done) != MOE_OK)
            return MOE_ERR_HIP;
        map_build_small<<<1, kMapThreads, lds, s>>>(topk_ids, map, T, k, E, N, g);
    } else {
        const int nchunks = nchunks_for(R);
        int32_t* chunk_hist = map + L.off_rows + round_up64((size_t)R);
        const int hs = hist_stride(L.E64);
        map_hist<<<nchunks, 256, hs * sizeof(int), s>>>(topk_ids, (int)R, E, L.E64, chunk_hist);
        static unsigned long long attr_done2 = 0;
        if (ensure_lds_attr(reinterpret_cast<const void*>(&map_scan_scatter),
                            (int)(((size_t)kWaves * kMaxE + kMaxE) * sizeof(int)), &attr_done2) != MOE_OK)
            return MOE_ERR_HIP;
        map_scan_scatter<<<nchunks, kMapThreads, ((size_t)kWaves * L.E64 + L.E64) * sizeof(int), s>>>(
            topk_ids, map, chunk_hist, nchunks, T, k, E, N, g);
    }
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int moe_task_map_status(const void* task_map, void* stream) {
    if (!task_map) return MOE_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t hdr[MOE_MAP_HDR_WORDS];
    if (hipMemcpyAsync(hdr, task_map, sizeof(hdr), hipMemcpyDeviceToHost, s) != hipSuccess) return MOE_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return MOE_ERR_HIP;
    if (hdr[MOE_HDR_MAGIC] != MOE_MAP_MAGIC) return MOE_ERR_INVALID_ARG;
    return hdr[MOE_HDR_STATUS] ? MOE_ERR_ROUTING : MOE_OK;
}

int moe_task_map_expand(const void* task_map, int E, int32_t* table, int64_t grid, void* stream) {
    if (!task_map || grid < 0 || (grid > 0 && !table) || E < 1 || E > kMaxE) return MOE_ERR_INVALID_ARG;
    if ((uintptr_t)table & 15) return MOE_ERR_INVALID_ARG;
    if (grid == 0) return MOE_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int64_t blocks = (grid + 3) / 4;
    if (blocks > 4096) blocks = 4096;
    map_expand<<<(unsigned)blocks, 256, 0, s>>>(static_cast<const int32_t*>(task_map), E, table, (long long)grid);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int moe_tile_supported(int dtype, int tile_m, int tile_n) { return find_variant(dtype, tile_m, tile_n) != nullptr; }

int moe_w_layout_supported(int dtype, const moe_tiling* g, int w_layout) {
    if (!g || check_small_args(g->tile_m, g->tile_m_small, g->small_max_rows, g->tile_m_slack) != MOE_OK) return 0;
    return find_variant(dtype, g->tile_m, g->tile_n, g->tile_m_small, g->tile_m_slack, w_layout) != nullptr;
}

int moe_grouped_gemm(const void* X, const void* W, const int32_t* topk_ids, const void* task_map, void* Y,
                     const moe_gemm_desc* d, void* stream) {
    (void)topk_ids;
    return grouped_gemm_impl(X, W, task_map, Y, d, nullptr, stream);
}

int64_t moe_reduce_task_tiles(int T, int N) {
    if (T < 0 || N < 8 || N % 8 != 0) return 0;
    const long long chunks = (long long)T * (N / 8);
    return (chunks + kReduceTileChunks - 1) / kReduceTileChunks;
}

int moe_grouped_gemm_batched(const void* X, const void* W, const void* task_map, void* Y, const moe_gemm_desc* d,
                             const moe_reduce_task* red, void* stream) {
    if (!red) return MOE_ERR_INVALID_ARG;
    if (red->T < 0 || red->k < 1 || red->N < 1) return MOE_ERR_INVALID_ARG;
    if (red->N % 8 != 0) return MOE_ERR_UNSUPPORTED;
    if (red->T > 0 && (!red->Y || !red->out || ((uintptr_t)red->Y & 15) || ((uintptr_t)red->out & 15) ||
                       ((uintptr_t)red->topk_weights & 3)))
        return MOE_ERR_INVALID_ARG;
    if (moe_reduce_task_tiles(red->T, red->N) > (1 << 24)) return MOE_ERR_UNSUPPORTED;
    return grouped_gemm_impl(X, W, task_map, Y, d, red, stream);
}

size_t moe_splitk_workspace_bytes(int T, int k, int N, int k_parts) {
    if (T < 0 || k < 1 || N < 1 || k_parts < 2) return 0;
    return (size_t)k_parts * (size_t)T * k * N * sizeof(float);
}

int moe_default_k_parts(int T, int k, int E, int K, int N) {
    if (T < 0 || k < 1 || E < 1 || k > E || K < 1 || N < 1) return MOE_ERR_INVALID_ARG;
    if (K % 64 != 0 || N % 256 != 0) return 1;
    const int64_t R = (int64_t)T * k;
    const double mean_rows = (double)R / E;
    const int64_t active = R < E ? R : E;
    const double mt = mean_rows / 256 + 0.5;
    const double tiles = (double)active * (mt < 1.0 ? 1.0 : mt) * (N / 256);
    const int cus = 256, kt = K / 64;
    // worth it where 256 x 256 tiles would leave CUs idle through a long k loop and the experts are not tiny
    // (measured on 8 experts, N = 4096, K = 14336, us with map build and reduction: 1024 rows 255 -> 198, 1536 rows
    // 294 -> 224; at 768 rows the 128 x 128 tiles of moe_default_tiling are faster, 171 against 190)
    if (mean_rows < 120 || tiles >= 0.75 * cus) return 1;
    // the fewest parts that cover three quarters of the CUs, else the most that keep 16 k-tiles each
    int best = 1;
    for (int parts = 2; parts <= 4; parts *= 2) {
        if (kt % parts != 0 || kt / parts < 16) break;
        best = parts;
        if (tiles * parts >= 0.75 * cus) break;
    }
    return best;
}

int moe_grouped_gemm_splitk(const void* X, const void* W, const void* task_map, void* Y, const moe_gemm_desc* d,
                            int k_parts, void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_splitk_args(d, k_parts);
    if (rc != MOE_OK) return rc;
    if (d->T == 0) return MOE_OK;
    if (!workspace || ((uintptr_t)workspace & 15)) return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < moe_splitk_workspace_bytes(d->T, d->k, d->N, k_parts)) return MOE_ERR_INVALID_ARG;
    return run_splitk(X, W, task_map, Y, d, k_parts, static_cast<float*>(workspace), static_cast<hipStream_t>(stream));
}

size_t moe_splitk_static_scratch_bytes(void) { return kStaticScratchBytes; }

size_t moe_tail_split_workspace_bytes(int tile_m, int tile_n) {
    if ((tile_m != 64 && tile_m != 128 && tile_m != 256) || tile_n != 256) return 0;
    return tail_workspace_bytes(tile_m, tile_n);
}

int moe_grouped_gemm_tail_split(const void* X, const void* W, const void* task_map, void* Y, const moe_gemm_desc* d,
                                void* workspace, size_t workspace_bytes, void* stream) {
    if (!d) return MOE_ERR_INVALID_ARG;
    if (d->T < 0 || d->k < 1 || d->E < 1 || d->E > kMaxE || d->k > d->E || d->K < 1 || d->N < 1) return MOE_ERR_INVALID_ARG;
    // the shapes the split-k task functions cover (how many parts, if any, is decided per XCD on the device)
    if (d->dtype != MOE_DTYPE_BF16 || d->w_layout != MOE_W_LAYOUT_KN || d->epilogue != MOE_EPILOGUE_NONE ||
        (d->tile_m != 64 && d->tile_m != 128 && d->tile_m != 256) || d->tile_n != 256 || d->tile_m_small != 0 ||
        d->small_max_rows != 0 || (d->tile_m_slack != 0 && !(d->tile_m == 256 && d->tile_m_slack == 32)))
        return MOE_ERR_UNSUPPORTED;
    if (d->K % 64 != 0 || d->N % 256 != 0) return MOE_ERR_UNSUPPORTED;
    if (d->T == 0) return MOE_OK;
    if (!X || !W || !task_map || !Y || !workspace) return MOE_ERR_INVALID_ARG;
    if (((uintptr_t)X & 15) || ((uintptr_t)W & 15) || ((uintptr_t)Y & 15) || ((uintptr_t)task_map & 15) || ((uintptr_t)workspace & 15))
        return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < tail_workspace_bytes(d->tile_m, d->tile_n)) return MOE_ERR_INVALID_ARG;
    if ((int64_t)d->T * d->K * 2 >= (int64_t)1 << 32) return MOE_ERR_UNSUPPORTED;
    GemmArgs a{};
    a.X = X; a.W = W; a.map = static_cast<const int32_t*>(task_map); a.Y = Y;
    a.T = d->T; a.k = d->k; a.E = d->E; a.K = d->K; a.N = d->N;
    a.tile_m_slack = d->tile_m_slack;
    a.partial = static_cast<float*>(workspace);
    a.cus_per_xcd = kCusPerXcd;
    int64_t grid = moe_grid_upper_bound_tiled(d->T, d->k, d->E, d->tile_m, d->tile_n, d->N, 0, 0);
    if (grid == 0) return MOE_OK;
    grid = (grid + 7) / 8 * 8 + 16;
    if (grid > 0x7fffffff) return MOE_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (d->tile_m) {
        case 256: return d->tile_m_slack == 32 ? launch_tail_split<Pb_256x256s32, Ps_64x256, Ps_128x256>(a, grid, s)
                                               : launch_tail_split<Pb_256x256, Ps_64x256, Ps_128x256>(a, grid, s);
        case 128: return launch_tail_split<Pb_128x256, Ps_64x256>(a, grid, s);
        default: return launch_tail_split<Pb_64x256>(a, grid, s);
    }
}

int moe_grouped_gemm_splitk_static(const void* X, const void* W, const void* task_map, void* Y, const moe_gemm_desc* d,
                                   int k_parts, void* stream) {
    const int rc = check_splitk_args(d, k_parts);
    if (rc != MOE_OK) return rc;
    if (moe_splitk_workspace_bytes(d->T, d->k, d->N, k_parts) > kStaticScratchBytes) return MOE_ERR_TOO_LARGE;
    if (d->T == 0) return MOE_OK;
    float* ws = nullptr;
    const int rs = static_scratch(&ws);
    if (rs != MOE_OK) return rs;
    return run_splitk(X, W, task_map, Y, d, k_parts, ws, static_cast<hipStream_t>(stream));
}

int moe_combine(const void* Y, const float* topk_weights, int T, int k, int N, void* out, void* stream) {
    if (T < 0 || k < 1 || N < 1) return MOE_ERR_INVALID_ARG;
    if (N % 8 != 0) return MOE_ERR_UNSUPPORTED;
    if (T == 0) return MOE_OK;
    if (!Y || !out || ((uintptr_t)Y & 15) || ((uintptr_t)out & 15) || ((uintptr_t)topk_weights & 3)) return MOE_ERR_INVALID_ARG;
    const long long chunks = (long long)T * (N / 8);
    long long blocks = (chunks + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;  // grid-stride beyond 64 workgroups per CU
    hipStream_t s = static_cast<hipStream_t>(stream);
    const u32x4_t* y = static_cast<const u32x4_t*>(Y);
    u32x4_t* o = static_cast<u32x4_t*>(out);
    switch (k) {  // the usual top-k values get their loads unrolled
        case 1: moe_combine_kernel<1><<<(unsigned)blocks, 256, 0, s>>>(y, topk_weights, o, T, k, N); break;
        case 2: moe_combine_kernel<2><<<(unsigned)blocks, 256, 0, s>>>(y, topk_weights, o, T, k, N); break;
        case 4: moe_combine_kernel<4><<<(unsigned)blocks, 256, 0, s>>>(y, topk_weights, o, T, k, N); break;
        case 6: moe_combine_kernel<6><<<(unsigned)blocks, 256, 0, s>>>(y, topk_weights, o, T, k, N); break;
        case 8: moe_combine_kernel<8><<<(unsigned)blocks, 256, 0, s>>>(y, topk_weights, o, T, k, N); break;
        default: moe_combine_kernel<0><<<(unsigned)blocks, 256, 0, s>>>(y, topk_weights, o, T, k, N); break;
    }
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

const char* moe_strerror(int code) {
    switch (code) {
        case MOE_OK: return "ok";
        case MOE_ERR_INVALID_ARG: return "invalid argument";
        case MOE_ERR_UNSUPPORTED: return "unsupported size, tile shape or dtype";
        case MOE_ERR_ROUTING: return "routing id outside [0, E)";
        case MOE_ERR_HIP: return "HIP runtime error";
        case MOE_ERR_TOO_LARGE: return "problem needs more scratch memory than the library's static array holds";
        default: return "unknown error";
    }
}

}  // extern "C"
