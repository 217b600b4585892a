/*
 * moe_sb — statically batched MoE expert GEMM for AMD MI355X (gfx950).
 *
 * C ABI of the hot path of "Static Batching of Irregular Workloads on GPUs:
 * Framework and Application to Efficient MoE Model Inference": given the
 * token sequence, the per-expert weights and this step's routing result,
 * compute for every token its product with each selected expert's weight
 * (Sec. 2.2, Sec. 4), as ONE kernel whose workgroups find their own
 * (expert, m-tile, n-tile) from a compressed task map (Sec. 3.1, Sec. 4.1).
 *
 * General rules for every call
 *   - Pointers marked DEVICE are device memory owned by the caller; pointers
 *     marked HOST are host memory.  The library allocates nothing; the only state
 *     it keeps is per-kernel, per-device launch attributes set on first use (guarded by a lock: calls
 *     may come from several host threads).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they do not synchronise unless stated.
 *   - Return value: MOE_OK (0) or a negative MOE_ERR_* code.  Nothing is
 *     enqueued when an argument error is returned.  No call throws or aborts.
 */
#ifndef MOE_SB_H
#define MOE_SB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = -1, /* null pointer, negative size, k > E, misaligned pointer */
    MOE_ERR_UNSUPPORTED = -2, /* tile shape / dtype / divisibility the kernels do not cover */
    MOE_ERR_ROUTING = -3,     /* a routing id outside [0,E) was found on the device */
    MOE_ERR_HIP = -4,         /* a HIP runtime call failed */
    MOE_ERR_TOO_LARGE = -5    /* the problem needs more scratch memory than the library's static array holds */
};

enum { MOE_DTYPE_BF16 = 0, MOE_DTYPE_FP8_E4M3 = 1 };

/* Storage order of the expert weights (moe_gemm_desc.w_layout).  KN is the layout of the problem statement:
 * W[e][k][n], n contiguous.  NK is a pre-packed alternative, W[e][n][k], k contiguous (the order in which
 * linear layers are usually stored); only some tilings have a kernel for it, see moe_w_layout_supported. */
enum { MOE_W_LAYOUT_KN = 0, MOE_W_LAYOUT_NK = 1 };

/* What the GEMM's epilogue stores (moe_gemm_desc.epilogue). */
enum { MOE_EPILOGUE_NONE = 0, MOE_EPILOGUE_SWIGLU = 1 };

/* Order of the non-empty experts in sigma (Sec. 4.1, Sec. 4.2). */
enum { MOE_ORDER_ASCENDING = 0, MOE_ORDER_SPREAD = 1, MOE_ORDER_INTERLEAVE = 2 };

/*
 * Task-map blob (all int32 words; E64 = E rounded up to a multiple of 64,
 * R = T*k routed rows, flat row id r = t*k + j).  Word offsets:
 *
 *   header       [MOE_MAP_HDR_WORDS]   see MOE_HDR_* below
 *   counts       [E64]       tokens per expert, pad 0
 *   offsets      [E64 + 64]  exclusive scan of counts; entries above E hold R
 *   sigma        [E64]       non-empty index -> real expert (Sec. 4.1), ascending, pad -1
 *   tile_prefix  [E64]       inclusive prefix sum of tiles per non-empty expert
 *                            (Alg. 1, built over non-empty experts only, Sec. 4.1);
 *                            pad INT32_MAX (Sec. 3.1 allows padding with the largest value)
 *   task_records [E64][4]    the same map packed per non-empty task i, for a decode with one memory
 *                            round trip: {tile_prefix[i], sigma[i], counts[sigma[i]], offsets[sigma[i]]};
 *                            pads {INT32_MAX, -1, 0, 0}
 *   sorted_rows  [R]         the per-expert token index arrays (Sec. 4.3) back to
 *                            back: rows of expert e are sorted_rows[offsets[e] ..
 *                            offsets[e+1]), ascending in r; token = r / k
 *   scratch      [...]       private to the library
 *
 * Tiles of expert e: nu(e) = ceil(counts[e]/tile_m(e)) * ceil(N/tile_n), tile_m(e) = tile_m unless a
 * second tiling strategy is in use (moe_build_task_map_tiled).
 * Block B (0-based) belongs to non-empty task h = #{ i : tile_prefix[i] <= B }
 * (Alg. 2), expert sigma[h] (Alg. 4), tile l = B - tile_prefix[h-1], and
 * m_tile = l % mt_e, n_tile = l / mt_e  (order 0 = "m fastest").
 */
#define MOE_MAP_MAGIC 0x3142534D /* "MSB1" */
#define MOE_MAP_HDR_WORDS 32
enum {
    MOE_HDR_MAGIC = 0,
    MOE_HDR_T = 1,
    MOE_HDR_K_TOP = 2,
    MOE_HDR_E = 3,
    MOE_HDR_N = 4,
    MOE_HDR_TILE_M = 5,
    MOE_HDR_TILE_N = 6,
    MOE_HDR_NT = 7,          /* ceil(N / tile_n) */
    MOE_HDR_M = 8,           /* number of non-empty experts */
    MOE_HDR_TOTAL_TILES = 9, /* tile_prefix[M-1], 0 when the map is empty or invalid */
    MOE_HDR_ORDER = 10,      /* 0: m-tile fastest inside an expert */
    MOE_HDR_STATUS = 11,     /* 0, or the number of routing ids outside [0,E) */
    MOE_HDR_R = 12,          /* T*k */
    MOE_HDR_E64 = 13,
    MOE_HDR_SIGMA_ORDER = 14,    /* MOE_ORDER_* the map was built with */
    MOE_HDR_TILE_M_SMALL = 15,   /* second tiling strategy (0 = none), see moe_build_task_map_tiled */
    MOE_HDR_SMALL_MAX_ROWS = 16,
    MOE_HDR_TILE_M_SLACK = 17,   /* extra rows the last m-tile of an expert may hold, see moe_build_task_map_ex */
    MOE_HDR_HEAVY_TILES = 18     /* MOE_ORDER_INTERLEAVE: tiles of the heavy experts = block index where the light part begins, else 0 */
};

/* Word offsets of the blob's fields for a given E (HOST, pure). */
size_t moe_map_off_counts(int E);
size_t moe_map_off_offsets(int E);
size_t moe_map_off_sigma(int E);
size_t moe_map_off_tile_prefix(int E);
size_t moe_map_off_task_records(int E);
size_t moe_map_off_sorted_rows(int E);

/*
 * Bytes the caller must allocate (DEVICE, 256-byte aligned) for a task map
 * that will hold up to T_max tokens.  HOST, pure.  Returns 0 on invalid
 * arguments.
 */
size_t moe_task_map_bytes(int T_max, int k, int E, int tile_m, int tile_n, int N);

/*
 * Workgroups moe_grouped_gemm launches for such a map: an upper bound on
 * total_tiles that needs no device->host copy,
 *   (floor(R/tile_m) + min(E, R)) * ceil(N/tile_n).   HOST, pure.
 */
int64_t moe_grid_upper_bound(int T, int k, int E, int tile_m, int tile_n, int N);

/*
 * Build the task map for one inference step, i.e. once the routing of the step is known
 * (Sec. 4.1; Alg. 1; Sec. 4.3 token index arrays).
 *   topk_ids  DEVICE int32 [T, k] row-major: expert chosen for token t, slot j.
 *   T >= 0 tokens (0 gives a valid empty map), 1 <= k <= E, 1 <= E <= 1024,
 *   T*k <= 2^24, tile_m in {16,32,64,128,256}, tile_n in {64,128,256}, N >= 1.
 *   task_map  DEVICE, >= moe_task_map_bytes(T,...) bytes, written entirely.  The allocation must really be
 *             that large: the kernels read a few words past sorted_rows (into the scratch part).
 * Deterministic: the same input gives the same bytes.  Ids outside [0,E) are
 * counted in header[MOE_HDR_STATUS] and force total_tiles = 0.
 */
int moe_build_task_map(const int32_t* topk_ids, int T, int k, int E, int tile_m, int tile_n, int N,
                       void* task_map, void* stream);

/*
 * Same, with the expert ordering of Sec. 4.2 made explicit.  The paper mixes busy
 * (compute-bound) and idle (memory-bound) experts along the block order and finds a placement by repeated
 * halving of the interval better than plain alternation, without giving the algorithm; here:
 *   MOE_ORDER_ASCENDING  sigma lists non-empty experts by increasing index (moe_build_task_map).
 *   MOE_ORDER_SPREAD     non-empty experts are ranked by tile count (largest first, ties by
 *                        lower index); rank r gets the key bitrev(r) over ceil(log2 M) bits;
 *                        sigma lists them by increasing key: busiest first, second busiest in
 *                        the middle, the next two at the quarter points, ... so every
 *                        contiguous run of blocks (one per XCD) mixes busy and small experts.
 *   MOE_ORDER_INTERLEAVE the way Sec. 4.2's idea is carried out here: experts whose rows fill at most a quarter of
 *                        one m-tile (4 * count <= tile_m) are light (their tiles only stream weights), the rest
 *                        heavy; sigma lists the heavy ones by falling tile count (ties by lower index), then
 *                        the light ones by rising index, and header[MOE_HDR_HEAVY_TILES] holds the block index
 *                        where the light part begins.  moe_grouped_gemm then deals every XCD a contiguous
 *                        share of the heavy blocks and one of the light blocks and runs them interleaved in
 *                        proportion, so that memory-bound tiles stream while compute-bound ones multiply.
 * Only sigma, tile_prefix and the task records depend on the order; counts, offsets and sorted_rows do not.
 * Any other `order` returns MOE_ERR_INVALID_ARG.
 */
int moe_build_task_map_ordered(const int32_t* topk_ids, int T, int k, int E, int tile_m, int tile_n, int N,
                               int order, void* task_map, void* stream);

/*
 * Same, with two tiling strategies in one batch (Alg. 3: tasks of different types / tiling
 * strategies dispatched inside one kernel; Sec. 4: large GEMMs are better served by large tiles).
 * The paper gives neither shapes nor thresholds; here an expert with at most
 * small_max_rows rows is tiled with tile_m_small rows per tile, every other expert with tile_m:
 *     nu(e) = ceil(counts[e] / tile_m(e)) * ceil(N / tile_n).
 * tile_m_small in {16,32,64,128}, tile_m_small < tile_m, 1 <= small_max_rows <= 4*tile_m_small;
 * tile_m_small = small_max_rows = 0 gives moe_build_task_map_ordered.  The pair must be passed
 * unchanged to moe_grouped_gemm (desc->tile_m_small, desc->small_max_rows).
 */
int moe_build_task_map_tiled(const int32_t* topk_ids, int T, int k, int E, int tile_m, int tile_n, int N, int order,
                             int tile_m_small, int small_max_rows, void* task_map, void* stream);

/* Grid bound for a two-strategy map (HOST, pure):
 *   (floor(R/tile_m) + min(E,R) * max(1, ceil(small_max_rows/tile_m_small))) * ceil(N/tile_n). */
int64_t moe_grid_upper_bound_tiled(int T, int k, int E, int tile_m, int tile_n, int N, int tile_m_small,
                                   int small_max_rows);

/*
 * All tiling choices of a batch in one place.  The paper leaves the tiling strategy of each task
 * to the task function (Sec. 3.2, Alg. 3); these are the strategies this library implements.
 */
typedef struct moe_tiling {
    int32_t tile_m, tile_n;   /* rows and columns of an output tile */
    int32_t order;            /* MOE_ORDER_* */
    int32_t tile_m_small, small_max_rows; /* second strategy for small experts, or 0, 0 */
    int32_t tile_m_slack;     /* 0, or: the last m-tile of a tile_m-strategy expert may hold up to
                                 tile_m + tile_m_slack rows, so that a remainder of at most
                                 tile_m_slack rows does not open a nearly empty tile of its own:
                                     m_tiles(c) = max(1, ceil((c - tile_m_slack) / tile_m))  for c > 0.
                                 Tile m of the expert starts at row m * tile_m of its segment; all
                                 tiles but the last hold tile_m rows.  0 <= tile_m_slack < tile_m.
                                 GEMM kernels exist for 256 x 256 bf16 tiles with 32 (the faster one, on
                                 16-row MFMA blocks) or 64 slack rows; moe_tiling_supported tells. */
} moe_tiling;

/*
 * The general builder: moe_build_task_map_tiled plus tile_m_slack.  Same arguments, blob and errors;
 * header word MOE_HDR_TILE_M_SLACK records the slack.  `tiling` is a HOST pointer, read before return.
 * The same moe_tiling values must reach moe_grouped_gemm through its descriptor.
 */
int moe_build_task_map_ex(const int32_t* topk_ids, int T, int k, int E, int N, const moe_tiling* tiling,
                          void* task_map, void* stream);

/*
 * A reasonable tiling for a problem shape, from the measurements behind this library (HOST, pure; the routing
 * itself is not known to the host, so the choice goes by the mean rows per expert T*k/E):
 *   fp8: up to 24 rows per expert (the decode regime) 16-row tiles, 256 wide when that gives between one and two
 *   workgroups per CU, else 128; up to 96 rows 64 x 256; above that 256 x 256;
 *   bf16: up to 48 rows per expert 128 x 128 when 256-wide tiles would leave CUs without one; else up to
 *   8 rows 16 x 256; from 48 to 96 rows 128 x 256 when there are enough n-tiles to fill
 *   the chip three times over, else 64 x 256; otherwise 256 x 256 (its launch handles tiles of at most 64 and
 *   128 rows with narrower task functions), with 32 slack rows above 192 rows per expert.  Where that choice
 *   would give fewer than three quarters of the CUs a tile under a balanced routing (few experts and a narrow N:
 *   a down projection at a few hundred tokens), the largest of 128 x 256, 128 x 128, 64 x 128 that does.
 * Always ascending order, one strategy.  The result satisfies moe_tiling_supported when N % tile_n == 0 allows
 * it (tile_n falls back to 128 or 64).  Returns MOE_ERR_INVALID_ARG on bad arguments, MOE_ERR_UNSUPPORTED when
 * no kernel fits (N not a multiple of 64).
 */
int moe_default_tiling(int dtype, int T, int k, int E, int K, int N, moe_tiling* out);

/* 1 if moe_grouped_gemm has a kernel for this dtype and tiling (order is ignored), else 0. HOST, pure. */
int moe_tiling_supported(int dtype, const moe_tiling* tiling);

/*
 * Synchronises the stream and returns MOE_ERR_ROUTING if the map recorded a
 * bad routing id, MOE_ERR_INVALID_ARG if the blob is not a map, else MOE_OK.
 */
int moe_task_map_status(const void* task_map, void* stream);

/*
 * Expand the compressed map into the full per-block table (the prior-art
 * representation of Sec. 2.1 / 3.1), using the same device decode routine the
 * GEMM kernel uses.  table: DEVICE int32 [grid][4] = {expert, m_tile, n_tile,
 * rows_in_tile}; rows_in_tile <= tile_m + tile_m_slack; entries B >= total_tiles are set to -1.  `grid` is normally
 * moe_grid_upper_bound(...).
 */
int moe_task_map_expand(const void* task_map, int E, int32_t* table, int64_t grid, void* stream);

typedef struct moe_gemm_desc {
    int32_t dtype;        /* MOE_DTYPE_* : element type of X and W */
    int32_t T, k, E;      /* must equal what the map was built with */
    int32_t K, N;         /* reduction length and output width */
    int32_t tile_m, tile_n; /* must equal what the map was built with */
    const float* x_scale; /* DEVICE fp32 [T], per-token scale  (fp8 only, else NULL) */
    const float* w_scale; /* DEVICE fp32 [E], per-expert scale (fp8 only, else NULL) */
    int32_t tile_m_small, small_max_rows; /* second tiling strategy of the map, or 0, 0 */
    int32_t tile_m_slack; /* slack rows of the map's last m-tiles, or 0 */
    int32_t epilogue;     /* MOE_EPILOGUE_* */
    int32_t w_layout;     /* MOE_W_LAYOUT_* */
    int32_t launch_mode;  /* MOE_LAUNCH_*; 0 for the library's own choice.  Results are identical in every mode. */
} moe_gemm_desc;

/* How moe_grouped_gemm maps workgroups to tiles (moe_gemm_desc.launch_mode).  The task map and the results are the
 * same in every mode; tests and measurements use the explicit modes.
 *   MOE_LAUNCH_AUTO      resident workgroups where a kernel for that exists and the grid bound is at least two
 *                        tiles per resident workgroup, else one workgroup per tile
 *   MOE_LAUNCH_PER_TILE  always one workgroup per tile
 *   MOE_LAUNCH_RESIDENT  resident workgroups (each runs a contiguous share of its XCD's tiles back to back) wherever
 *                        a kernel for that exists: 16-row tiles with E <= 256 (fp8: T + E <= 2048); elsewhere the
 *                        same as MOE_LAUNCH_PER_TILE
 *   a value >= 8         MOE_LAUNCH_RESIDENT with at most that many workgroups (rounded down to a multiple of 8)
 */
enum { MOE_LAUNCH_AUTO = 0, MOE_LAUNCH_PER_TILE = 1, MOE_LAUNCH_RESIDENT = 2 };

/*
 * The statically batched expert GEMM (Alg. 3/4 with the GEMM tile as the task
 * function; Sec. 4.3 gathered token rows; Sec. 4.4 pipeline):
 *     Y[t, j, :] = X[t, :] . W[e(t,j), :, :]        e(t,j) = topk_ids[t, j]
 *   X  DEVICE [T, K]    bf16 or e4m3 bytes, K contiguous, 16-byte aligned rows
 *   W  DEVICE [E, K, N] same element type, N contiguous  (or [E, N, K] with desc->w_layout = MOE_W_LAYOUT_NK)
 *   Y  DEVICE [T, k, N] bf16, written once per element; rows of a partial
 *      m-tile beyond the expert's count write nothing.
 *   fp8: Y = (sum over e4m3 products in fp32) * x_scale[t] * w_scale[e].
 * Accumulation is fp32; the store rounds to bf16 (nearest even).
 * Requires K % 64 == 0 (bf16) / K % 128 == 0 (fp8) and N % tile_n == 0,
 * else MOE_ERR_UNSUPPORTED.  (tile_m, tile_n, dtype) must be a supported
 * combination: see moe_tile_supported.  A map whose header does not match
 * `desc`, or whose status is non-zero, makes the kernel a no-op.
 * topk_ids is accepted for symmetry with the problem statement and may be
 * NULL: the kernel reads the routing from the map.
 *
 * desc->epilogue = MOE_EPILOGUE_SWIGLU fuses the activation of a gated expert into the same task function
 * (Sec. 3.2: the work of a tile is whatever its task function does): W holds the gate projection in columns
 * [0, N/2) and the up projection in [N/2, N), and with G = X.W_gate, U = X.W_up (fp32 sums, fp8 scaled first)
 *     Y[t, j, i] = bf16( G_i / (1 + exp(-G_i)) * U_i ),   i in [0, N/2);   Y is DEVICE [T, k, N/2].
 * The map is the one built for N (an n-tile of tile_n weight columns yields tile_n/2 outputs).  N % 64 == 0.
 */
int moe_grouped_gemm(const void* X, const void* W, const int32_t* topk_ids, const void* task_map, void* Y,
                     const moe_gemm_desc* desc, void* stream);

/*
 * The same product for launches too short to give every CU a tile (few experts, a narrow N and a long K: a down
 * projection at several hundred tokens), split along K: every tile of the map (Sec. 3.1: the map is unchanged, a
 * workgroup finds its tile as always) is run by k_parts workgroups, each over one k_parts-th of K; their fp32 sums
 * go to `workspace` and a second kernel adds them in ascending order of the parts, rounds once to bf16 and scatters
 * the rows to Y.  Same result definition and tolerance as moe_grouped_gemm; the summation order differs.
 *   workspace  DEVICE, 16-byte aligned, at least moe_splitk_workspace_bytes(T, k, N, k_parts) bytes
 *              (k_parts * T*k * N fp32); owned by the caller, contents undefined afterwards; calls that share a
 *              workspace must not overlap.
 * Supported: bf16, MOE_W_LAYOUT_KN, MOE_EPILOGUE_NONE, tile 256 x 256 without slack rows and with one tiling
 * strategy, k_parts 2 or 4 with (K / 64) % k_parts == 0 and K / 64 / k_parts >= 8, N % 256 == 0; anything else
 * returns MOE_ERR_UNSUPPORTED.  MOE_ERR_INVALID_ARG for NULL or misaligned pointers or a workspace that is too small.
 */
int moe_grouped_gemm_splitk(const void* X, const void* W, const void* task_map, void* Y, const moe_gemm_desc* desc,
                            int k_parts, void* workspace, size_t workspace_bytes, void* stream);

/*
 * moe_grouped_gemm_splitk for callers that cannot allocate device memory and have no workspace to hand in: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without the
 * workspace), same kernels, same results bit for bit; the fp32 partial sums go to a static device array inside the
 * library instead: moe_splitk_static_scratch_bytes() = 32 MiB per GPU, held by every GPU the library runs on until
 * the process ends.  The call allocates and frees nothing (its first call on a device looks the array's address up).
 *   - MOE_ERR_TOO_LARGE when moe_splitk_workspace_bytes(T, k, N, k_parts) exceeds the array (nothing is enqueued);
 *     all other errors as for moe_grouped_gemm_splitk.
 *   - All calls on one GPU share that GPU's array, which keeps the last call's contents.  Nothing in it has to start
 *     at zero: every partial sum the reduction reads was written by the product launch of the same call.  Calls that
 *     may overlap on one GPU (different streams without ordering, several host threads) race on it: order them, or
 *     use moe_grouped_gemm_splitk with a workspace each.
 */
int moe_grouped_gemm_splitk_static(const void* X, const void* W, const void* task_map, void* Y,
                                   const moe_gemm_desc* desc, int k_parts, void* stream);

/* Size of that static array in bytes.  HOST, pure. */
size_t moe_splitk_static_scratch_bytes(void);

/*
 * moe_grouped_gemm for launches whose last round of tiles is only partly filled (Sec. 3.1's map is unchanged; this
 * is a property of the launch).  With one workgroup per tile an XCD's tiles run in rounds of its 32 CUs; when the
 * last round holds t < 32 tiles the other CUs idle for a whole tile's duration.  Here those t tiles are run by
 * P workgroups each, every one over a part of K; their fp32 sums go to `workspace` and are added in ascending order
 * of the parts, rounded once to bf16 and scattered to Y.  P is the smallest of 1, 2, 4 that minimises the last
 * round's length ceil(t * P / 32) / P (e.g. t <= 8: 4 parts, a quarter; t = 16: 2 parts, a half; t = 22: 4 parts,
 * three quarters; t = 27: no split), chosen per XCD on the device, and only if every part keeps at least 8 k-tiles.
 * All other tiles run exactly as in moe_grouped_gemm (their results are bit for bit the same); the tail tiles differ
 * from it in summation order only.  Three launches on `stream`.
 *   workspace  DEVICE, 16-byte aligned, at least moe_tail_split_workspace_bytes(tile_m, tile_n) bytes
 *              (8 * 128 * rows * tile_n * 4 with rows = tile_m, 288 for 256-row tiles: 288 MiB), owned by the caller, contents undefined
 *              afterwards; calls that share it must not overlap.
 * Supported: bf16, MOE_W_LAYOUT_KN, MOE_EPILOGUE_NONE, tiles 256 x 256 (without slack rows or with 32), 128 x 256 or
 * 64 x 256 (without), one tiling strategy, K % 64 == 0, N % 256 == 0; anything else MOE_ERR_UNSUPPORTED.
 */
int moe_grouped_gemm_tail_split(const void* X, const void* W, const void* task_map, void* Y, const moe_gemm_desc* desc,
                                void* workspace, size_t workspace_bytes, void* stream);
/* HOST, pure; 0 for a tile shape without a tail-split launch. */
size_t moe_tail_split_workspace_bytes(int tile_m, int tile_n);

/* Bytes of workspace moe_grouped_gemm_splitk needs (0 for k_parts < 2 or bad sizes).  HOST, pure. */
size_t moe_splitk_workspace_bytes(int T, int k, int N, int k_parts);

/* Whether to split, for a bf16 product over 256 x 256 tiles (HOST, pure): 1 = no (use moe_grouped_gemm with
 * moe_default_tiling), else the k_parts (2 or 4) to pass to moe_grouped_gemm_splitk with a plain 256 x 256
 * tiling.  It says yes where, under a balanced
 * routing, 256 x 256 tiles would cover fewer than three quarters of the CUs, the experts hold at least 120 rows on
 * average and every part keeps at least 16 k-tiles (the fewest parts that cover
 * three quarters of the CUs, else four, else two).  MOE_ERR_INVALID_ARG (negative) on bad arguments. */
int moe_default_k_parts(int T, int k, int E, int K, int N);

/* 1 if a GEMM kernel exists for this (dtype, tile_m, tile_n), else 0.  HOST, pure. */
int moe_tile_supported(int dtype, int tile_m, int tile_n);
/* 1 if a GEMM kernel exists for this dtype, tiling and weight layout, else 0.  HOST, pure. */
int moe_w_layout_supported(int dtype, const moe_tiling* tiling, int w_layout);
/* 1 if a two-strategy GEMM kernel exists for (dtype, tile_m, tile_n) + tile_m_small.  HOST, pure. */
int moe_tile_pair_supported(int dtype, int tile_m, int tile_n, int tile_m_small);

/*
 * The last step of the MoE layer (Sec. 2.2: the products of a token with its selected experts are summed up):
 *     out[t, n] = bf16( sum_{j=0..k-1} w[t, j] * Y[t, j, n] )     (fp32, j ascending)
 *   Y            DEVICE [T, k, N] bf16 (what moe_grouped_gemm wrote), 16-byte aligned
 *   topk_weights DEVICE [T, k] fp32 router weights, or NULL for the plain sum
 *   out          DEVICE [T, N] bf16, 16-byte aligned, must not overlap Y
 * N % 8 == 0, else MOE_ERR_UNSUPPORTED.  Enqueued on `stream`; allocates nothing.
 */
int moe_combine(const void* Y, const float* topk_weights, int T, int k, int N, void* out, void* stream);

/*
 * Heterogeneous batching (Sec. 3.2, Alg. 3: tasks of different kinds -- the paper names a GEMM and a reduction -- in
 * ONE kernel): moe_grouped_gemm with a reduction task added to the batch.  The reduction is moe_combine's,
 *     out[t, n] = bf16( sum_j topk_weights[t, j] * Y_in[t, j, n] ),
 * over the finished products of an EARLIER call (another layer, another micro-batch: it must not depend on the Y
 * this call writes).  Its nu = moe_reduce_task_tiles(T, N) tiles of 4096 eight-column chunks each are appended to
 * the GEMM map's tiles: in the terms of Sec. 3.1 the batch's TilePrefix is the map's with one more entry,
 * total_tiles + nu; a block at or beyond total_tiles belongs to the reduction task and runs its task function,
 * every other block is decoded as in moe_grouped_gemm.  The reduction tiles only move memory; every XCD walks its
 * share of them spread in proportion over its share of the GEMM blocks (the placement idea of Sec. 4.2), so they
 * stream while the neighbouring workgroups multiply.
 */
typedef struct moe_reduce_task {
    const void* Y;              /* DEVICE [T, k, N] bf16, 16-byte aligned */
    const float* topk_weights;  /* DEVICE [T, k] fp32, or NULL for the plain sum */
    int32_t T, k, N;            /* N % 8 == 0 */
    void* out;                  /* DEVICE [T, N] bf16, 16-byte aligned, must not overlap Y or the GEMM's buffers */
} moe_reduce_task;

/* Tiles of such a reduction task: ceil(T * (N / 8) / 4096).  HOST, pure; 0 on invalid sizes. */
int64_t moe_reduce_task_tiles(int T, int N);

/*
 * X, W, task_map, Y, desc as for moe_grouped_gemm (same results bit for bit); `red` is a HOST pointer, read before
 * return.  out is what moe_combine(red->Y, red->topk_weights, red->T, red->k, red->N, red->out) gives, bit for bit.
 * Supported where a batched kernel exists: bf16, [E][K][N] weights, 256 x 256 tiles without slack rows or with 32,
 * one tiling strategy; anything else MOE_ERR_UNSUPPORTED.  A map that does not match `desc` makes the whole call a
 * no-op (the reduction included).  MOE_ERR_INVALID_ARG for a NULL red or bad pointers.
 */
int moe_grouped_gemm_batched(const void* X, const void* W, const void* task_map, void* Y, const moe_gemm_desc* desc,
                             const moe_reduce_task* red, void* stream);

/* Static string for a return code. */
const char* moe_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* MOE_SB_H */
