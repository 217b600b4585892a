/*
 * Oracle for the statically batched MoE expert GEMM.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, CPU-only restatement of what the hot path computes, written
 * from the paper (Static Batching of Irregular Workloads on GPUs, Sec. 3.1,
 * Sec. 4.1, Sec. 4.3; Alg. 1, 2, 4) so that it can be checked against the
 * paper by eye.  It shares no code, header, table or helper with the HIP
 * library.  Only tests, the smoke check and the CPU-baseline leg of the
 * benchmark may call it; the product path never does.
 *
 * Conventions (the paper leaves these open; each is a fixed reading):
 *   - block index B and all arrays are 0-based: the task of block B is
 *     h = #{ i : TilePrefix[i] <= B }  (the comparison Alg. 2 votes on, read with 0-based B).
 *   - nu(expert e) = ceil(c_e / tile_m(e)) * ceil(N / tile_n)   (tiles of its GEMM), where
 *     tile_m(e) is the task's tiling strategy (Sec. 3.2, Sec. 4: every task is assigned to one
 *     of a few tiling strategies fixed in advance; the paper gives neither shapes nor thresholds).  Two
 *     strategies here: experts with at most small_max_rows rows use tile_m_small, all
 *     others tile_m; small_max_rows = 0 means one strategy for every expert.
 *     A third knob of the tile_m strategy, also this library's own: with tile_m_slack > 0
 *     an expert's rows are cut into tiles of tile_m rows from the front, but as soon as
 *     what is left fits into tile_m + tile_m_slack rows it becomes the last tile, so a
 *     remainder of a few rows never gets a tile to itself.  Tile m still starts at row
 *     m * tile_m of the expert's segment.  tile_m_slack = 0 is the plain ceil(c / tile_m).
 *   - sigma lists the non-empty experts in ascending expert index (Sec. 4.1), or, with
 *     order = 1, spread out by repeated halving (our reading of the better of the two arrangements of Sec. 4.2): the non-empty experts
 *     are ranked by tile count (largest first, ties by lower index), rank r gets the key
 *     bitrev(r) over ceil(log2 M) bits, and sigma lists them by increasing key -- the
 *     busiest expert first, the second busiest in the middle, the next two at the
 *     quarter points, and so on, with the small experts filling the gaps.
 *   - inside an expert, tile index l runs m-tile fastest:
 *       m_tile = l % mt_e,  n_tile = l / mt_e.
 *   - the token index array of an expert (Sec. 4.3) is ordered by flat row id
 *     r = t*k + j (stable), which makes the map unique.
 *   - result: Y[r, n] = sum_kappa X[t, kappa] * W[e(r), kappa, n], no sum over
 *     a token's experts.
 *
 * Parity pins (tests, CPU only): hand-worked examples, brute-force full
 * per-block table vs. the Alg. 2+4 decode, count/permutation invariants, the
 * paper's balanced/best/worst closed-form counts (Sec. 5), reduction to a
 * plain matrix product checked against an independent library matmul, bf16 and
 * e4m3 format definitions checked against an independent implementation.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- formats */

/* bfloat16 = the upper 16 bits of an IEEE-754 binary32. */
float orc_bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* binary32 -> bfloat16, round to nearest, ties to even.  NaN stays NaN. */
uint16_t orc_f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lower = u & 0xffffu;
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1u;
    return (uint16_t)upper;
}

/* double -> bfloat16 with a single rounding (RNE) straight from the double. */
uint16_t orc_f64_to_bf16_rne(double d) {
    if (isnan(d)) return 0x7fc0;
    uint16_t sign = signbit(d) ? 0x8000u : 0u;
    double a = fabs(d);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7f80u);
    int ex;
    double m = frexp(a, &ex); /* a = m * 2^ex, m in [0.5,1) */
    int e = ex - 1;            /* a = (2m) * 2^e, 2m in [1,2) */
    if (e < -126) e = -126;    /* subnormal range: fixed exponent */
    /* quantum of a bf16 at exponent e is 2^(e-7) */
    double q = ldexp(1.0, e - 7);
    double n = a / q; /* exact: power-of-two scaling */
    double fl = floor(n);
    double frac = n - fl;
    if (frac > 0.5 || (frac == 0.5 && fmod(fl, 2.0) == 1.0)) fl += 1.0;
    double r = fl * q;
    (void)m;
    float rf = (float)r; /* exactly representable (<= 8 significant bits) or inf */
    uint32_t u;
    memcpy(&u, &rf, 4);
    if (r >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7f80u);
    return (uint16_t)(sign | (u >> 16));
}

/* OCP 8-bit float E4M3 (the "fn" flavour: bias 7, no infinities, only
 * S.1111.111 is NaN, max finite 448).
 *   normal:    (-1)^s * 2^(E-7) * (1 + m/8),  E in 1..15
 *   subnormal: (-1)^s * 2^(-6)  * (m/8),      E = 0                        */
float orc_e4m3_to_f32(uint8_t b) {
    int s = b >> 7, E = (b >> 3) & 15, m = b & 7;
    float v;
    if (E == 15 && m == 7) return NAN;
    if (E == 0) v = ldexpf((float)m / 8.0f, -6);
    else v = ldexpf(1.0f + (float)m / 8.0f, E - 7);
    return s ? -v : v;
}

/* ---------------------------------------------------------------- task map */

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

/* Alg. 1: inclusive prefix sum of the tile counts nu[0..n).  Written as the
 * definition (a fresh sum for every i), not as a running scan. */
void orc_tile_prefix(const int32_t* nu, int n, int32_t* tile_prefix) {
    for (int i = 0; i < n; ++i) {
        int64_t s = 0;
        for (int j = 0; j <= i; ++j) s += nu[j];
        tile_prefix[i] = (int32_t)s;
    }
}

/* The mapping of Sec. 3.1 (what Alg. 2's vote and population count arrive at), written from its definition:
 * block B belongs to the first task whose inclusive prefix lies above B -- TilePrefix is non-decreasing, so
 * that task's index equals the number of entries at or below B -- and its tile index inside the task is B
 * minus everything the tasks before it hold.  Blocks past the last entry get h = n. */
void orc_mapping(const int32_t* tile_prefix, int n, int B, int32_t* h_out, int32_t* l_out) {
    int owner = 0;
    while (owner < n && tile_prefix[owner] <= B) owner += 1;
    int32_t tiles_before = owner > 0 ? tile_prefix[owner - 1] : 0;
    *h_out = owner;
    *l_out = B - tiles_before;
}

/* Two-level TilePrefix (Sec. 3.1 mentions it for task counts beyond a few warps and omits the details; our
 * reading): the tasks are cut into groups of `group` consecutive tasks, the first level holds the last
 * TilePrefix entry of every group (a group cut short by the end of the array counts as ending at +infinity).
 * A vote over the first level gives the group of block B, Alg. 2 inside that group gives the task.
 * Must return exactly what orc_mapping returns.                                                        */
void orc_mapping_two_level(const int32_t* tile_prefix, int n, int group, int B, int32_t* h_out, int32_t* l_out) {
    int groups = (n + group - 1) / group;
    int g = 0; /* groups that lie entirely at or before B */
    for (int i = 0; i < groups; ++i) {
        int last = i * group + group - 1;
        if (last < n && B >= tile_prefix[last]) g += 1;
    }
    int begin = g * group;
    int len = n - begin < group ? n - begin : group;
    if (len < 0) len = 0;
    int32_t h = 0, l = 0;
    orc_mapping(tile_prefix + begin, len, B, &h, &l);
    /* l from the in-group vote is relative to the group's first entry only when h > 0 there */
    if (h == 0) l = B - (begin > 0 ? tile_prefix[begin - 1] : 0);
    *h_out = begin + h;
    *l_out = l;
}

/* Tiling strategy of an expert with c rows (see the conventions at the top). */
static int expert_tile_m(int c, int tile_m, int tile_m_small, int small_max_rows) {
    return (small_max_rows > 0 && c <= small_max_rows) ? tile_m_small : tile_m;
}

/* m-tiles of an expert with c rows, and the rows of its tile m_tile (conventions at the top):
 * tiles are cut from the front; what fits into tm + slack rows is the last tile. */
static int expert_m_tiles(int c, int tile_m, int tile_m_small, int small_max_rows, int slack) {
    int tm = expert_tile_m(c, tile_m, tile_m_small, small_max_rows);
    if (tm != tile_m) slack = 0; /* the slack belongs to the tile_m strategy only */
    int tiles = 0, left = c;
    while (left > 0) {
        tiles += 1;
        if (left <= tm + slack) left = 0;
        else left -= tm;
    }
    return tiles;
}
static int expert_tile_rows(int c, int tile_m, int tile_m_small, int small_max_rows, int slack, int m_tile) {
    int tm = expert_tile_m(c, tile_m, tile_m_small, small_max_rows);
    if (tm != tile_m) slack = 0;
    int left = c - m_tile * tm;
    return left <= tm + slack ? left : tm;
}

/* Bit reversal of r over nbits bits. */
static int bit_reverse(int r, int nbits) {
    int v = 0;
    for (int b = 0; b < nbits; ++b)
        if (r & (1 << b)) v |= 1 << (nbits - 1 - b);
    return v;
}

/* Sec. 4.2 order by repeated halving (reading stated at the top of this file).
 * experts[0..M) ascending non-empty experts with tile counts nu[0..M): writes sigma[0..M). */
static void spread_order(const int32_t* experts, const int32_t* nu, int M, int32_t* sigma) {
    int nbits = 0;
    while ((1 << nbits) < M) ++nbits;
    int32_t* key = (int32_t*)malloc(sizeof(int32_t) * (size_t)(M > 0 ? M : 1));
    for (int i = 0; i < M; ++i) {
        int rank = 0; /* how many experts are busier (or equally busy with a lower index) */
        for (int j = 0; j < M; ++j)
            if (nu[j] > nu[i] || (nu[j] == nu[i] && j < i)) rank += 1;
        key[i] = bit_reverse(rank, nbits);
    }
    for (int i = 0; i < M; ++i) {
        int pos = 0;
        for (int j = 0; j < M; ++j)
            if (key[j] < key[i]) pos += 1;
        sigma[pos] = experts[i];
    }
    free(key);
}

/* Sec. 4.2 wants memory-bound (few-token) experts to run at the same time as compute-bound (busy) ones.  Order 2
 * prepares that: the non-empty experts are split into heavy and light ones (light: all rows fit one m-tile and
 * fill at most a quarter of it, 4 * c <= tile_m), sigma lists the heavy ones first, by falling tile count (ties by
 * lower index), then the light ones by rising index; heavy_tiles = the tiles of the heavy part, i.e. the block
 * index at which the light part begins.  How the kernel then deals heavy and light blocks to its workgroups is
 * the kernel's business (any bijection of the block indices computes the same Y).
 * experts[0..M), counts_ne[0..M), nu[0..M): the ascending non-empty experts, their row and tile counts.       */
static int interleave_order(const int32_t* experts, const int32_t* counts_ne, const int32_t* nu, int M, int tile_m,
                            int32_t* sigma) {
    int heavy_tiles = 0, n = 0;
    char* used = (char*)calloc((size_t)(M > 0 ? M : 1), 1);
    /* heavy experts by selection: repeatedly take the unused heavy expert with the most tiles (first one on ties) */
    for (;;) {
        int best = -1;
        for (int i = 0; i < M; ++i) {
            int light = (4 * counts_ne[i] <= tile_m);
            if (used[i] || light) continue;
            if (best < 0 || nu[i] > nu[best]) best = i;
        }
        if (best < 0) break;
        used[best] = 1;
        sigma[n++] = experts[best];
        heavy_tiles += nu[best];
    }
    for (int i = 0; i < M; ++i)
        if (!used[i]) sigma[n++] = experts[i];
    free(used);
    return heavy_tiles;
}

/* Routing result -> everything the kernel needs (Sec. 4.1, 4.3):
 *   counts[E], offsets[E+1] (exclusive scan), sorted_rows[T*k] (per-expert
 *   token index arrays, stored back to back, as flat row ids r = t*k+j; the
 *   token is r / k), sigma[M] (non-empty -> real expert), tile_prefix[M].
 *   order: 0 = sigma ascending, 1 = spread (Sec. 4.2), 2 = heavy experts first, then the light ones.
 *   tile_m_small, small_max_rows: the second tiling strategy (0, 0 = none).
 *   tile_m_slack: rows the last tile of a tile_m-strategy expert may hold beyond tile_m.
 * Returns 0, or -1 if an id is outside [0,E).                               */
int orc_build_task_map(const int32_t* topk_ids, int T, int k, int E, int tile_m, int tile_n, int N, int order,
                       int tile_m_small, int small_max_rows, int tile_m_slack, int32_t* counts, int32_t* offsets, int32_t* sorted_rows, int32_t* sigma,
                       int32_t* tile_prefix, int32_t* M_out, int32_t* total_tiles_out, int32_t* heavy_tiles_out) {
    int R = T * k;
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int r = 0; r < R; ++r) {
        int e = topk_ids[r];
        if (e < 0 || e >= E) return -1;
        counts[e] += 1;
    }
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
    /* token index arrays: for each expert, the rows routed to it, ascending */
    for (int e = 0; e < E; ++e) {
        int w = offsets[e];
        for (int r = 0; r < R; ++r)
            if (topk_ids[r] == e) sorted_rows[w++] = r;
    }
    /* the non-empty experts and their tile counts */
    int M = 0;
    int32_t* nu = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E > 0 ? E : 1));
    int32_t* ne = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E > 0 ? E : 1));
    int nt = ceil_div(N, tile_n);
    for (int e = 0; e < E; ++e) {
        if (counts[e] > 0) {
            ne[M] = e;
            nu[M] = expert_m_tiles(counts[e], tile_m, tile_m_small, small_max_rows, tile_m_slack) * nt;
            M += 1;
        }
    }
    int heavy_tiles = 0;
    if (order == 1) spread_order(ne, nu, M, sigma);
    else if (order == 2) {
        int32_t* cne = (int32_t*)malloc(sizeof(int32_t) * (size_t)(M > 0 ? M : 1));
        for (int i = 0; i < M; ++i) cne[i] = counts[ne[i]];
        heavy_tiles = interleave_order(ne, cne, nu, M, tile_m, sigma);
        free(cne);
    } else for (int i = 0; i < M; ++i) sigma[i] = ne[i];
    /* tile counts in sigma order, then Alg. 1 */
    for (int i = 0; i < M; ++i)
        nu[i] = expert_m_tiles(counts[sigma[i]], tile_m, tile_m_small, small_max_rows, tile_m_slack) * nt;
    orc_tile_prefix(nu, M, tile_prefix);
    free(nu);
    free(ne);
    *M_out = M;
    *total_tiles_out = M > 0 ? tile_prefix[M - 1] : 0;
    if (heavy_tiles_out) *heavy_tiles_out = heavy_tiles;
    return 0;
}

/* Alg. 4 for block B: non-empty task h, real expert sigma(h), then the tile
 * index l split into (m_tile, n_tile), m fastest.  out = {e, m_tile, n_tile,
 * rows_in_tile}.                                                           */
void orc_decode_block(const int32_t* tile_prefix, const int32_t* sigma, int M, const int32_t* counts,
                      int tile_m, int tile_m_small, int small_max_rows, int tile_m_slack, int B, int32_t* out4) {
    int32_t h, l;
    orc_mapping(tile_prefix, M, B, &h, &l);
    int e = sigma[h];
    /* Alg. 3: the task's type decides its tiling */
    int mt = expert_m_tiles(counts[e], tile_m, tile_m_small, small_max_rows, tile_m_slack);
    int m_tile = l % mt, n_tile = l / mt;
    int rows = expert_tile_rows(counts[e], tile_m, tile_m_small, small_max_rows, tile_m_slack, m_tile);
    out4[0] = e; out4[1] = m_tile; out4[2] = n_tile; out4[3] = rows;
}

/* The prior-art full per-block table (Sec. 2.1 / 3.1: one entry per thread
 * block), by nested loops over (expert, n_tile, m_tile) with no prefix array
 * at all.  It is an independent definition of the same map.  expert_order
 * lists all E experts in visiting order (empty ones contribute no entry).
 * Returns the number of entries written (room for cap entries of 4 ints).  */
int orc_full_table(const int32_t* counts, int E, const int32_t* expert_order, int tile_m, int tile_m_small,
                   int small_max_rows, int tile_m_slack, int tile_n, int N, int32_t* table, int cap) {
    int b = 0;
    int nt = ceil_div(N, tile_n);
    for (int i = 0; i < E; ++i) {
        int e = expert_order ? expert_order[i] : i; /* experts are visited in this order; NULL = 0,1,2,... */
        int tm = expert_tile_m(counts[e], tile_m, tile_m_small, small_max_rows);
        int slack = tm == tile_m ? tile_m_slack : 0;
        for (int n_tile = 0; n_tile < nt; ++n_tile) {
            /* walk the expert's rows: a tile of tm rows at a time, the rest as one tile once it fits tm + slack */
            int first_row = 0, m_tile = 0;
            while (first_row < counts[e]) {
                if (b >= cap) return -1;
                int rest = counts[e] - first_row;
                int rows = rest <= tm + slack ? rest : tm;
                table[4 * b + 0] = e; table[4 * b + 1] = m_tile;
                table[4 * b + 2] = n_tile; table[4 * b + 3] = rows;
                b += 1;
                first_row += rows;
                m_tile += 1;
            }
        }
    }
    return b;
}

/* ---------------------------------------------------------------- result */

/* Y for a list of routed rows (rows == NULL: all T*k rows, in order).
 * X: [T,K] bf16 bits, W: [E,K,N] bf16 bits (N contiguous).
 * For row r = t*k+j with e = topk_ids[r], for every n:
 *     acc32 = ((x_0*w_0 + x_1*w_1) + x_2*w_2) + ...     (fp32, kappa ascending)
 *     acc64 = the same sum in fp64
 * Outputs (any may be NULL), each [nrows, N]:
 *     Y32  fp32 accumulator, Y64 fp64 accumulator,
 *     Ybf  bf16_rne(acc64)  (one rounding, from the fp64 sum).
 * The loop nest is (row, kappa, n) so that memory is walked contiguously;
 * each output element still adds its terms in increasing kappa.            */
void orc_grouped_gemm_bf16(const uint16_t* X, const uint16_t* W, const int32_t* topk_ids, int T, int k,
                           int E, int K, int N, const int32_t* rows, int nrows, float* Y32, double* Y64,
                           uint16_t* Ybf) {
    (void)E;
    if (rows == NULL) nrows = T * k;
#pragma omp parallel
    {
        float* a32 = (float*)malloc(sizeof(float) * (size_t)N);
        double* a64 = (double*)malloc(sizeof(double) * (size_t)N);
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < nrows; ++i) {
            int r = rows ? rows[i] : i;
            int t = r / k;
            int e = topk_ids[r];
            const uint16_t* x = X + (size_t)t * K;
            const uint16_t* w = W + (size_t)e * K * N;
            for (int n = 0; n < N; ++n) { a32[n] = 0.0f; a64[n] = 0.0; }
            for (int kap = 0; kap < K; ++kap) {
                float xv = orc_bf16_to_f32(x[kap]);
                const uint16_t* wr = w + (size_t)kap * N;
                for (int n = 0; n < N; ++n) {
                    float wv = orc_bf16_to_f32(wr[n]);
                    float p = xv * wv; /* exact: 8-bit x 8-bit significands */
                    a32[n] += p;
                    a64[n] += (double)p;
                }
            }
            for (int n = 0; n < N; ++n) {
                size_t o = (size_t)i * N + n;
                if (Y32) Y32[o] = a32[n];
                if (Y64) Y64[o] = a64[n];
                if (Ybf) Ybf[o] = orc_f64_to_bf16_rne(a64[n]);
            }
        }
        free(a32);
        free(a64);
    }
}

/* fp8 variant: X [T,K] e4m3 bytes with x_scale[T]; W [E,K,N] e4m3 bytes with
 * w_scale[E].  The sum runs over the decoded bytes; the two scales multiply
 * the finished sum once:  Y = (sum) * x_scale[t] * w_scale[e].             */
void orc_grouped_gemm_fp8(const uint8_t* X, const uint8_t* W, const float* x_scale, const float* w_scale,
                          const int32_t* topk_ids, int T, int k, int E, int K, int N, const int32_t* rows,
                          int nrows, float* Y32, double* Y64, uint16_t* Ybf) {
    (void)E;
    if (rows == NULL) nrows = T * k;
#pragma omp parallel
    {
        float* a32 = (float*)malloc(sizeof(float) * (size_t)N);
        double* a64 = (double*)malloc(sizeof(double) * (size_t)N);
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < nrows; ++i) {
            int r = rows ? rows[i] : i;
            int t = r / k;
            int e = topk_ids[r];
            const uint8_t* x = X + (size_t)t * K;
            const uint8_t* w = W + (size_t)e * K * N;
            for (int n = 0; n < N; ++n) { a32[n] = 0.0f; a64[n] = 0.0; }
            for (int kap = 0; kap < K; ++kap) {
                float xv = orc_e4m3_to_f32(x[kap]);
                const uint8_t* wr = w + (size_t)kap * N;
                for (int n = 0; n < N; ++n) {
                    float p = xv * orc_e4m3_to_f32(wr[n]); /* exact: 4-bit x 4-bit */
                    a32[n] += p;
                    a64[n] += (double)p;
                }
            }
            double s = (double)x_scale[t] * (double)w_scale[e];
            for (int n = 0; n < N; ++n) {
                size_t o = (size_t)i * N + n;
                if (Y32) Y32[o] = (a32[n] * x_scale[t]) * w_scale[e];
                if (Y64) Y64[o] = a64[n] * s;
                if (Ybf) Ybf[o] = orc_f64_to_bf16_rne(a64[n] * s);
            }
        }
        free(a32);
        free(a64);
    }
}

/* Single elements (r, n) one by one: used to sample huge problems.
 * is_fp8 selects the element decoding; scales may be NULL for bf16.        */
void orc_gemm_elements(const void* X, const void* W, const float* x_scale, const float* w_scale,
                       const int32_t* topk_ids, int k, int K, int N, int is_fp8, const int32_t* rr,
                       const int32_t* nn, int count, double* Y64) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < count; ++i) {
        int r = rr[i], n = nn[i];
        int t = r / k, e = topk_ids[r];
        double acc = 0.0;
        for (int kap = 0; kap < K; ++kap) {
            float xv, wv;
            if (is_fp8) {
                xv = orc_e4m3_to_f32(((const uint8_t*)X)[(size_t)t * K + kap]);
                wv = orc_e4m3_to_f32(((const uint8_t*)W)[((size_t)e * K + kap) * N + n]);
            } else {
                xv = orc_bf16_to_f32(((const uint16_t*)X)[(size_t)t * K + kap]);
                wv = orc_bf16_to_f32(((const uint16_t*)W)[((size_t)e * K + kap) * N + n]);
            }
            acc += (double)xv * (double)wv;
        }
        if (is_fp8) acc *= (double)x_scale[t] * (double)w_scale[e];
        Y64[i] = acc;
    }
}

/* Norm product ||X[t,:]||_2 * ||W[e,:,n]||_2 for sampled elements: the scale
 * the error tolerance is stated against (scales folded in for fp8).        */
void orc_norm_scale_elements(const void* X, const void* W, const float* x_scale, const float* w_scale,
                             const int32_t* topk_ids, int k, int K, int N, int is_fp8, const int32_t* rr,
                             const int32_t* nn, int count, double* out) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < count; ++i) {
        int r = rr[i], n = nn[i];
        int t = r / k, e = topk_ids[r];
        double sx = 0.0, sw = 0.0;
        for (int kap = 0; kap < K; ++kap) {
            double xv, wv;
            if (is_fp8) {
                xv = orc_e4m3_to_f32(((const uint8_t*)X)[(size_t)t * K + kap]);
                wv = orc_e4m3_to_f32(((const uint8_t*)W)[((size_t)e * K + kap) * N + n]);
            } else {
                xv = orc_bf16_to_f32(((const uint16_t*)X)[(size_t)t * K + kap]);
                wv = orc_bf16_to_f32(((const uint16_t*)W)[((size_t)e * K + kap) * N + n]);
            }
            sx += xv * xv;
            sw += wv * wv;
        }
        double s = sqrt(sx) * sqrt(sw);
        if (is_fp8) s *= fabs((double)x_scale[t] * (double)w_scale[e]);
        out[i] = s;
    }
}

/* ---------------------------------------------------------------- neighbours of the product */

/* Gated activation of an expert whose weight holds the gate projection in columns [0, N/2) and the up
 * projection in [N/2, N) (the fused gate and up projection of the benchmark shapes; the paper's MoE layer,
 * Sec. 2.2, leaves the expert's internals open):
 *     H[r, i] = silu(G) * U,  G = Y[r, i], U = Y[r, N/2 + i],  silu(g) = g / (1 + exp(-g)),
 * from the fp64 sums Y64 [nrows, N] of orc_grouped_gemm_*.  Outputs [nrows, N/2]: H64, and Hbf = one
 * rounding of H64 to bf16.                                                                              */
void orc_swiglu(const double* Y64, int nrows, int N, double* H64, uint16_t* Hbf) {
    int I = N / 2;
    for (int r = 0; r < nrows; ++r)
        for (int i = 0; i < I; ++i) {
            double g = Y64[(size_t)r * N + i];
            double u = Y64[(size_t)r * N + I + i];
            double h = g / (1.0 + exp(-g)) * u;
            if (H64) H64[(size_t)r * I + i] = h;
            if (Hbf) Hbf[(size_t)r * I + i] = orc_f64_to_bf16_rne(h);
        }
}

/* The sum over a token's selected experts (Sec. 2.2: the products are finally summed up), weighted by the
 * router when w != NULL:   out[t, n] = sum_j w[t, j] * Y[t, j, n],  j ascending.
 * Y: [T, k, N] bf16 bits (what the product stored).  Outputs [T, N]: out64, outbf = one rounding to bf16. */
void orc_combine(const uint16_t* Y, const float* w, int T, int k, int N, double* out64, uint16_t* outbf) {
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int j = 0; j < k; ++j) {
                double wj = w ? (double)w[(size_t)t * k + j] : 1.0;
                acc += wj * (double)orc_bf16_to_f32(Y[((size_t)t * k + j) * N + n]);
            }
            if (out64) out64[(size_t)t * N + n] = acc;
            if (outbf) outbf[(size_t)t * N + n] = orc_f64_to_bf16_rne(acc);
        }
}
