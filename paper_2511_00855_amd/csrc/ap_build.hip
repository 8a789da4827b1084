// Index construction (Algorithm 1, Steps 1-3 of Section 4.1): seed lists by an
// MFMA dense product with exact top-K selection, synchronous refinement rounds
// under the hybrid metric, detourable-route sort, inner-product pruning with
// keyword recycling, and assembly of the fixed-degree edge lists.
// Every stage is a pure function of the previous stage's arrays; nothing that
// decides an id depends on the order in which atomics arrive.
#include <stdlib.h>
#include <algorithm>
#include "ap_tiles.hpp"

int ap_fill_u32(void *p, size_t n, uint32_t v, hipStream_t st);
int ap_alloc_graph(ap_index *ix);

#define AP_A_CAP 512   // a-side list entries staged in LDS

// =================================================================== S2: seed
// scores[r][j] = <dense[node r], dense[j]> for a slab of rows and all columns.
// Tile order of the seed products.  Workgroups are handed to the 8 XCDs round-robin by their linear id, and every XCD
// has an L2 of its own: workgroup b runs on XCD b % 8 and is the (b / 8)-th of that XCD.  Each XCD gets a contiguous
// band of row tiles and walks it column tile by column tile, so the band's rows stay in that XCD's L2 and a column
// tile is fetched once per XCD instead of once per row tile.  Returns false for the padding workgroups of a band that
// is shorter than the others.
#define AP_XCDS 8
__device__ __forceinline__ bool ap_seed_tile(int64_t row_tiles, int64_t &rt, int64_t &ct) {
    const int64_t band = (row_tiles + AP_XCDS - 1) / AP_XCDS;
    const int64_t xcd = blockIdx.x % AP_XCDS, idx = blockIdx.x / AP_XCDS;
    rt = xcd * band + idx % band;
    ct = idx / band;
    return rt < row_tiles;
}
static inline unsigned ap_seed_grid(int64_t row_tiles, int64_t col_tiles) {
    return (unsigned)(AP_XCDS * ((row_tiles + AP_XCDS - 1) / AP_XCDS) * col_tiles);
}

template <int DT>
__global__ __launch_bounds__(256) void k_seed_scores(const void *dense, int32_t dim, int64_t n, const int32_t *node_ids,
                                                     int64_t row0, int64_t nrows, int64_t col0, int64_t ncols,
                                                     float *__restrict__ scores /* nrows x ncols */) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[ApTileLds<DT>::BYTES];
    __shared__ int32_t a_rows[AP_TILE], b_rows[AP_TILE];
    int64_t rt, ct;
    if (!ap_seed_tile((nrows + AP_TILE - 1) / AP_TILE, rt, ct)) return;
    const int64_t i0 = rt * AP_TILE, j0 = ct * AP_TILE;
    if (threadIdx.x < AP_TILE) {
        const int64_t r = i0 + threadIdx.x;
        a_rows[threadIdx.x] = r < nrows ? (node_ids ? node_ids[row0 + r] : (int32_t)(row0 + r)) : -1;
        const int64_t j = j0 + threadIdx.x;
        b_rows[threadIdx.x] = j < ncols ? (int32_t)(col0 + j) : -1;
    }
    ap_f32x16 acc[2][2];
    ap_tile_product<DT>(dense, dim, a_rows, b_rows, lds, acc);
    ap_tile_foreach(acc, [&](int i, int j, float v) {
        if (i0 + i < nrows && j0 + j < ncols) scores[(i0 + i) * ncols + (j0 + j)] = v;
    });
}

// Appending a tile's candidates to their rows' buffers.  A candidate is not appended on the spot (an atomic on the
// row's counter whose answer the store has to wait for, at some forty of a lane's sixty-four elements): the wave notes
// it in its own part of the LDS the product has left (place = a running count + the lane's rank among the lanes that
// passed: no atomic, no wait); afterwards the candidates are counted per row in LDS, every row that has some takes its
// places in buf with ONE atomic for the whole tile, and the candidates are written out.
// An entry: score bits | column in the tile << 32 | row in the tile << 40 | side << 48 | (later) place << 49.
// side 0: the candidate goes to the buffer of its row's document (id = its column's document); side 1, used by the
// symmetric sweep only: the score is also that of the mirrored pair, and the candidate goes to the buffer of its
// column's document (id = its row's document).
// direct(side, i, j, v): the append on the spot, for what the wave's part (wcap entries) cannot hold.
template <typename DIRECT>
__device__ __forceinline__ void ap_seed_stage(bool pass, int side, int i, int j, float v, uint64_t *stage, int32_t wcap, int32_t &nw, DIRECT direct) {
    const uint64_t m = __ballot(pass);
    if (m) {
        if (pass) {
            const int32_t slot = nw + (int32_t)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
            if (slot < wcap) stage[slot] = ((uint64_t)(uint32_t)((side << 16) | (i << 8) | j) << 32) | __float_as_uint(v);
            else direct(side, i, j, v);
        }
        nw += __popcll(m);
    }
}
// Called by every thread of the workgroup once its wave has staged nw candidates.  drop(side, i, j): a candidate that is
// not one after all (the document itself, a row or column past the end).  s_cnt[2 * rows] must be zero on entry
// ([rows] if no candidate has side 1).  Buffers and counters are indexed by row0 + (row in the tile) for side 0 and by
// row1 + (column in the tile) for side 1; the ids stored are id0 + column and id1 + row.
template <typename DROP>
__device__ __forceinline__ void ap_seed_flush(uint64_t *stage, int32_t wcap, int32_t nw, int32_t rows, bool both_sides, int32_t *s_cnt,
                                              int32_t *s_base, int32_t *__restrict__ cnt, unsigned long long *__restrict__ buf, int32_t cap,
                                              int64_t row0, int32_t id0, int64_t row1, int32_t id1, DROP drop) {
    const int lane = threadIdx.x & 63;
    const int32_t ns = nw < wcap ? nw : wcap;
    for (int32_t p = lane; p < ns; p += 64) {
        const uint64_t e = stage[p];
        const int32_t j = (int32_t)(e >> 32) & 255, i = (int32_t)(e >> 40) & 255, side = (int32_t)(e >> 48) & 1;
        if (drop(side, i, j)) { stage[p] = e | (0x7fffull << 49); continue; }
        stage[p] = e | ((uint64_t)atomicAdd(&s_cnt[side ? rows + j : i], 1) << 49);
    }
    __syncthreads();
    for (int32_t x = threadIdx.x; x < (both_sides ? 2 * rows : rows); x += blockDim.x) {
        const int32_t c = s_cnt[x];
        s_base[x] = c ? atomicAdd(&cnt[x < rows ? row0 + x : row1 + (x - rows)], c) : 0;
    }
    __syncthreads();
    for (int32_t p = lane; p < ns; p += 64) {
        const uint64_t e = stage[p];
        const int32_t j = (int32_t)(e >> 32) & 255, i = (int32_t)(e >> 40) & 255, side = (int32_t)(e >> 48) & 1, place = (int32_t)(e >> 49);
        if (place == 0x7fff) continue;
        const int32_t pos = s_base[side ? rows + j : i] + place;
        if (pos < cap) buf[(side ? row1 + j : row0 + i) * (int64_t)cap + pos] = ap_make_key(__uint_as_float((uint32_t)e), side ? id1 + i : id0 + j, 1u);
    }
}

// The same product over all columns, but instead of storing the scores, every
// score that reaches its row's threshold tau (a lower bound of the row's K-th
// best, found on a sample of the columns) is appended to the row's candidate
// buffer as a ranking key.  cnt[r] counts the appends (also those beyond cap).
// The launch covers column tiles from ct0 on.  SYM (rows = a slab of the whole corpus in order, every tile full and
// inside the corpus): tau, buf and cnt point at the slab's first row inside arrays that cover the whole corpus; tiles
// below the diagonal return at once, and a score of a tile above it is offered to its column's document as well (see
// k_seed_thresh_big).
template <int DT, bool SYM>
__global__ __launch_bounds__(256) void k_seed_thresh(const void *dense, int32_t dim, int64_t n, const int32_t *node_ids,
                                                     int64_t row0, int64_t nrows, const float *__restrict__ tau,
                                                     unsigned long long *__restrict__ buf, int32_t cap,
                                                     int32_t *__restrict__ cnt, int64_t ct0) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[ApTileLds<DT>::BYTES];
    __shared__ int32_t a_rows[AP_TILE], b_rows[AP_TILE];
    __shared__ float s_tau[AP_TILE], s_tauc[SYM ? AP_TILE : 1];
    __shared__ int32_t s_cnt[(SYM ? 2 : 1) * AP_TILE], s_base[(SYM ? 2 : 1) * AP_TILE];
    int64_t rt, ct;
    if (!ap_seed_tile((nrows + AP_TILE - 1) / AP_TILE, rt, ct)) return;
    const int64_t i0 = rt * AP_TILE, j0 = (ct0 + ct) * AP_TILE;
    if (SYM && j0 < row0 + i0) return;   // below the diagonal: its mirror image does the work
    const bool mirror = SYM && j0 > row0 + i0;   // uniform
    if (threadIdx.x < AP_TILE) {
        const int64_t r = i0 + threadIdx.x;
        s_cnt[threadIdx.x] = 0;
        if (SYM) { s_cnt[AP_TILE + threadIdx.x] = 0; s_tauc[threadIdx.x] = tau[j0 - row0 + threadIdx.x]; }
        a_rows[threadIdx.x] = r < nrows ? (node_ids ? node_ids[row0 + r] : (int32_t)(row0 + r)) : -1;
        s_tau[threadIdx.x] = r < nrows ? tau[r] : INFINITY;
        const int64_t j = j0 + threadIdx.x;
        b_rows[threadIdx.x] = j < n ? (int32_t)j : -1;
    }
    ap_f32x16 acc[2][2];
    ap_tile_product<DT>(dense, dim, a_rows, b_rows, lds, acc);
    __syncthreads();   // the product's LDS is free
    constexpr int W_CAP = ApTileLds<DT>::BYTES / 4 / 8;
    uint64_t *stage = reinterpret_cast<uint64_t *>(lds) + ap_wave_id() * W_CAP;
    auto drop = [&](int, int i, int j) { return !(i0 + i < nrows && j0 + j < n && a_rows[i] != (int32_t)(j0 + j)); };
    auto direct = [&](int side, int i, int j, float v) {
        if (!drop(side, i, j)) {
            const int64_t row = side ? j0 - row0 + j : i0 + i;
            const int32_t pos = atomicAdd(&cnt[row], 1);
            if (pos < cap) buf[row * (int64_t)cap + pos] = ap_make_key(v, side ? (int32_t)(row0 + i0 + i) : (int32_t)(j0 + j), 1u);
        }
    };
    int32_t nw = 0;
    ap_tile_foreach(acc, [&](int i, int j, float v) {
        ap_seed_stage(v >= s_tau[i], 0, i, j, v, stage, W_CAP, nw, direct);
        if (SYM) ap_seed_stage(mirror && v >= s_tauc[j], 1, i, j, v, stage, W_CAP, nw, direct);
    });
    ap_seed_flush(stage, W_CAP, nw, AP_TILE, SYM, s_cnt, s_base, cnt, buf, cap, i0, (int32_t)j0, j0 - row0, (int32_t)(row0 + i0), drop);
}

// The thresholded sweep for bf16 rows on 256x256 tiles (the product above): the same appends as k_seed_thresh.
// 4 x 4 waves of 64 x 64 each: measured faster than 2 x 4 waves of 128 x 64 or 2 x 2 of 128 x 128 (fewer LDS reads per
// MFMA, but fewer waves to overlap them with), and 12 % faster than the 128 x 128 tiles of k_seed_thresh.
#ifndef AP_BIG_WM
#define AP_BIG_WM 4
#define AP_BIG_WN 4
#endif
// RUN: every tile of the launch is two runs of 256 consecutive documents inside the corpus (no node list, no ragged
// edge, dim a multiple of 64); the host launches the edges of a sweep with RUN = false.  The launch covers row tiles
// rt0 .. rt0 + nrt and column tiles from ct0 on.
// SYM (with RUN, rows = the whole corpus, row0 = 0): the product is symmetric, so only the tiles on and above the
// diagonal are computed (a launch's tiles below it return at once), and a score of an off-diagonal tile is offered
// twice: to its row's document against that document's threshold, and to its column's document against that one's.
// The mirrored pair would have got the same bits: the same products summed over k in the same order.
template <int WM, int WN, bool RUN, bool SYM>
__global__ __launch_bounds__(WM * WN * 64) void k_seed_thresh_big(const void *dense, int32_t dim, int64_t n, const int32_t *node_ids,
                                                                  int64_t row0, int64_t nrows, const float *__restrict__ tau,
                                                                  unsigned long long *__restrict__ buf, int32_t cap,
                                                                  int32_t *__restrict__ cnt, int64_t rt0, int64_t nrt, int64_t ct0) {
    static_assert(RUN || !SYM, "the symmetric sweep is for runs of consecutive documents");
    extern __shared__ __attribute__((aligned(16))) unsigned char big_lds[];
    __shared__ int32_t a_rows[AP_BIG], b_rows[AP_BIG];
    __shared__ __attribute__((aligned(16))) float s_tau[AP_BIG];
    __shared__ float s_tauc[SYM ? AP_BIG : 1];          // SYM: the thresholds of the tile's column documents
    __shared__ int32_t s_cnt[(SYM ? 2 : 1) * AP_BIG], s_base[(SYM ? 2 : 1) * AP_BIG];   // the tile's candidates per buffer, and where each buffer's go
    int64_t rt, ct;
    if (!ap_seed_tile(nrt, rt, ct)) return;
    const int64_t i0 = (rt0 + rt) * AP_BIG, j0 = (ct0 + ct) * AP_BIG;
    if (SYM && j0 < i0) return;   // below the diagonal: its mirror image does the work
    for (int32_t x = threadIdx.x; x < AP_BIG; x += blockDim.x) {
        s_cnt[x] = 0;
        if (SYM) { s_cnt[AP_BIG + x] = 0; s_tauc[x] = tau[j0 + x]; }
        const int64_t r = i0 + x;
        a_rows[x] = r < nrows ? (node_ids ? node_ids[row0 + r] : (int32_t)(row0 + r)) : -1;
        s_tau[x] = r < nrows ? tau[r] : INFINITY;
        const int64_t j = j0 + x;
        b_rows[x] = j < n ? (int32_t)j : -1;
    }
    ap_f32x16 acc[ApBig<WM, WN>::FA][ApBig<WM, WN>::FB];
    if (RUN) {
        const int32_t a_first = (int32_t)(row0 + i0), b_first = (int32_t)j0;
        ap_big_gemm_bf16<WM, WN, true>(dense, dim, a_rows, b_rows, a_first, b_first, reinterpret_cast<uint16_t *>(big_lds), acc);
        // A lane holds 4 consecutive rows x (FB x 32 columns apart) per 8-row group: the rows' thresholds come as one
        // 16-byte LDS read, and an element costs a compare and a (rarely taken) branch.  Only a tile whose row and
        // column runs overlap can pair a document with itself.
        const bool diagonal = a_first < b_first + AP_BIG && b_first < a_first + AP_BIG;
        const bool mirror = SYM && !diagonal;   // uniform: the scores also go to the column documents
        const int lane = threadIdx.x & 63, wave = ap_wave_id();
        const int wm = wave / WN, wn = wave % WN;
        constexpr int W_CAP = AP_BIG_LDS_BYTES / (WM * WN) / 8;   // entries of a wave's part of the LDS
        uint64_t *stage = reinterpret_cast<uint64_t *>(big_lds) + wave * W_CAP;
        auto drop = [&](int, int i, int j) { return diagonal && a_first + i == b_first + j; };
        auto direct = [&](int side, int i, int j, float v) {
            if (!drop(side, i, j)) {
                const int64_t row = side ? j0 + j : i0 + i;
                const int32_t pos = atomicAdd(&cnt[row], 1);
                if (pos < cap) buf[row * (int64_t)cap + pos] = ap_make_key(v, side ? a_first + i : b_first + j, 1u);
            }
        };
        float tc[ApBig<WM, WN>::FB];   // the thresholds of this lane's columns
#pragma unroll
        for (int b = 0; b < ApBig<WM, WN>::FB; b++) tc[b] = SYM ? s_tauc[wn * (AP_BIG / WN) + b * 32 + (lane & 31)] : INFINITY;
        int32_t nw = 0;   // uniform: candidates of this wave so far
#pragma unroll
        for (int a = 0; a < ApBig<WM, WN>::FA; a++)
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const int ib = wm * (AP_BIG / WM) + a * 32 + 8 * q + 4 * (lane >> 5);
                const float4 t4 = *reinterpret_cast<const float4 *>(&s_tau[ib]);
                const float tt[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
                for (int b = 0; b < ApBig<WM, WN>::FB; b++)
#pragma unroll
                    for (int rr = 0; rr < 4; rr++) {
                        const float v = acc[a][b][4 * q + rr];
                        const int j = wn * (AP_BIG / WN) + b * 32 + (lane & 31);
                        ap_seed_stage(v >= tt[rr], 0, ib + rr, j, v, stage, W_CAP, nw, direct);
                        if (SYM) ap_seed_stage(mirror && v >= tc[b], 1, ib + rr, j, v, stage, W_CAP, nw, direct);
                    }
            }
        ap_seed_flush(stage, W_CAP, nw, AP_BIG, SYM, s_cnt, s_base, cnt, buf, cap, i0, b_first, j0, a_first, drop);
    } else {
        ap_big_gemm_bf16<WM, WN, false>(dense, dim, a_rows, b_rows, 0, 0, reinterpret_cast<uint16_t *>(big_lds), acc);
        constexpr int W_CAP = AP_BIG_LDS_BYTES / (WM * WN) / 8;
        uint64_t *stage = reinterpret_cast<uint64_t *>(big_lds) + ap_wave_id() * W_CAP;
        auto drop = [&](int, int i, int j) { return !(i0 + i < nrows && j0 + j < n && a_rows[i] != (int32_t)(j0 + j)); };
        auto direct = [&](int, int i, int j, float v) {
            if (!drop(0, i, j)) {
                const int32_t pos = atomicAdd(&cnt[i0 + i], 1);
                if (pos < cap) buf[(i0 + i) * (int64_t)cap + pos] = ap_make_key(v, (int32_t)(j0 + j), 1u);
            }
        };
        int32_t nw = 0;
        ap_big_foreach<WM, WN>(acc, [&](int i, int j, float v) { ap_seed_stage(v >= s_tau[i], 0, i, j, v, stage, W_CAP, nw, direct); });
        ap_seed_flush(stage, W_CAP, nw, AP_BIG, false, s_cnt, s_base, cnt, buf, cap, i0, (int32_t)j0, (int64_t)0, 0, drop);
    }
}

// One block per row: exact top-K of the row (excluding the node itself), sorted.
// Row r of `scores` has ncols entries; its result goes to row out_row0 + r.
__global__ __launch_bounds__(256) void k_select_rows(const float *__restrict__ scores, int64_t ncols, int32_t K,
                                                     const int32_t *node_ids, int64_t row0, int32_t exclude_self, int64_t out_row0,
                                                     int32_t *__restrict__ out_ids, float *__restrict__ out_sc) {
    __shared__ uint32_t hist[256];
    __shared__ uint64_t sel[256];
    __shared__ int32_t misc[4];
    __shared__ uint64_t pre;
    const int64_t r = blockIdx.x;
    const int32_t self = exclude_self ? (node_ids ? node_ids[row0 + r] : (int32_t)(row0 + r)) : -1;
    for (int i = threadIdx.x; i < 256; i += blockDim.x) sel[i] = 0;
    __syncthreads();
    const int32_t got = ap_radix_select(scores + r * ncols, ncols, self, K, hist, sel, misc, &pre);
    ap_bitonic_desc(sel, 256);
    for (int32_t i = threadIdx.x; i < K; i += blockDim.x) {
        if (out_ids) out_ids[(out_row0 + r) * K + i] = i < got ? ap_key_id(sel[i]) : -1;
        out_sc[(out_row0 + r) * K + i] = i < got ? ap_key_score(sel[i]) : -INFINITY;
    }
}

// tau[r] = K-th best score of row r of a [nrows x K] sorted score table.
// ulps (a debug setting, normally 0) raises the threshold by that many representable values.
__global__ void k_take_tau(const float *__restrict__ sc, int64_t nrows, int32_t K, uint32_t ulps, float *__restrict__ tau) {
    const int64_t r = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (r < nrows) {
        const float t = sc[r * K + K - 1];
        tau[r] = (ulps && t - t == 0.f) ? ap_ord2f(ap_f2ord(t) + ulps) : t;
    }
}

// One block per row: exact top-K among the row's buffered candidate keys.
// Rows whose buffer overflowed are reported in overflow_rows and left to the caller, and so are rows that hold fewer
// than `need` = min(K, n - 1) keys: the threshold came from another kernel's product of the same rows, and a score
// that kernel rounded one ulp higher would silently shorten the list.
__global__ __launch_bounds__(256) void k_select_buf(const unsigned long long *__restrict__ buf, int32_t cap,
                                                    const int32_t *__restrict__ cnt, int32_t K, int32_t need, int64_t out_row0,
                                                    int32_t *__restrict__ out_ids, float *__restrict__ out_sc,
                                                    int32_t *__restrict__ n_overflow, int32_t *__restrict__ overflow_rows) {
    __shared__ uint32_t hist[256];
    __shared__ uint64_t sel[256];
    __shared__ int32_t misc[4];
    __shared__ uint64_t pre;
    const int64_t r = blockIdx.x;
    const int32_t c = cnt[r];
    if (c > cap || c < need) {   // uniform for the block
        if (threadIdx.x == 0) overflow_rows[atomicAdd(n_overflow, 1)] = (int32_t)r;
        return;
    }
    for (int i = threadIdx.x; i < 256; i += blockDim.x) sel[i] = 0;
    __syncthreads();
    const unsigned long long *row = buf + r * (int64_t)cap;
    const int32_t got = ap_radix_select_keys([&](int64_t j) -> uint64_t { return row[j]; }, c, c, K, hist, sel, misc, &pre);
    ap_bitonic_desc(sel, 256);
    for (int32_t i = threadIdx.x; i < K; i += blockDim.x) {
        out_ids[(out_row0 + r) * K + i] = i < got ? ap_key_id(sel[i]) : -1;
        out_sc[(out_row0 + r) * K + i] = i < got ? ap_key_score(sel[i]) : -INFINITY;
    }
}

// Exact path: full score rows of a slab, then selection.  Rows [row0, row0+nrows) of the node list.
static hipError_t seed_exact_rows(const ap_index *ix, const int32_t *node_ids, int64_t row0, int64_t nrows, int32_t K,
                                  float *scratch, int64_t scratch_rows, int32_t *out_ids, float *out_sc, hipStream_t st) {
    const int64_t n = ix->docs.n;
    hipError_t e = hipSuccess;
    for (int64_t r0 = row0; r0 < row0 + nrows && e == hipSuccess; r0 += scratch_rows) {
        const int64_t nr = std::min(scratch_rows, row0 + nrows - r0);
        dim3 grid(ap_seed_grid((nr + AP_TILE - 1) / AP_TILE, (n + AP_TILE - 1) / AP_TILE));
        ix->seed_flops += (unsigned long long)(((nr + AP_TILE - 1) / AP_TILE) * ((n + AP_TILE - 1) / AP_TILE)) * 2ull * AP_TILE * AP_TILE * (unsigned long long)ix->docs.dim;
        if (ix->dtype == AP_F32)
            hipLaunchKernelGGL(k_seed_scores<AP_F32>, grid, dim3(256), 0, st, ix->docs.dense, ix->docs.dim, n, node_ids, r0, nr, (int64_t)0, n, scratch);
        else
            hipLaunchKernelGGL(k_seed_scores<AP_BF16>, grid, dim3(256), 0, st, ix->docs.dense, ix->docs.dim, n, node_ids, r0, nr, (int64_t)0, n, scratch);
        e = hipGetLastError();
        if (e != hipSuccess) break;
        hipLaunchKernelGGL(k_select_rows, dim3((unsigned)nr), dim3(256), 0, st, scratch, n, K, node_ids, r0, 1, r0, out_ids, out_sc);
        e = hipGetLastError();
    }
    return e;
}

// rows list[r] of a [*, K] table take the values of row r of a compact one
__global__ void k_scatter_rows(const int32_t *__restrict__ list, int64_t nlist, int32_t K, const int32_t *__restrict__ ids,
                               const float *__restrict__ sc, int32_t *__restrict__ out_ids, float *__restrict__ out_sc) {
    const int64_t t = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (t < nlist * K) {
        const int64_t r = t / K, i = t % K;
        out_ids[(int64_t)list[r] * K + i] = ids[t];
        out_sc[(int64_t)list[r] * K + i] = sc[t];
    }
}

// S2 for a whole corpus of bf16 rows: the sweep with half the products.  D D^T is symmetric, so only the tiles on and
// above the diagonal are multiplied and every score is offered to both of its documents (k_seed_thresh_big<.., SYM>).
// For that every document's candidate buffer has to exist at once, so the buffers are short (cap entries, by the
// memory that is free) and the thresholds tight: tau = the m-th best of cs sampled columns with m < K, chosen so that
// a row expects about 0.45 cap candidates.  Such a tau is not a guaranteed lower bound of the row's K-th best: a row
// that ends up with fewer than K candidates (a few in ten thousand) or more than cap is redone by the exact path,
// like an overflowing row of the one-sided sweep.  The lists are the exact ones either way.
// *done = false (and AP_OK): not applicable here (shape, memory); the caller takes the one-sided sweep.
static int ap_seed_knn_symmetric(const ap_index *ix, int32_t K, int32_t *out_ids, float *out_sc, hipStream_t st, bool *done) {
    *done = false;
    const bool big = ix->dtype == AP_BF16;             // bf16 rows: 256x256 tiles; f32 rows: 128x128 tiles
    const int64_t E = big ? AP_BIG : AP_TILE;
    const int64_t n = ix->docs.n, T = n / E;
    if ((big && ix->docs.dim % AP_BK16 != 0) || T < 2 || n > ((int64_t)1 << 30)) return AP_OK;
    size_t free_b = 0, total_b = 0;
    if (hipMemGetInfo(&free_b, &total_b) != hipSuccess) return AP_OK;
    int64_t cap = 4096;
    while (cap > 512 && (double)n * (double)cap * 8.0 > 0.62 * (double)free_b) cap >>= 1;
    if ((double)n * (double)cap * 8.0 > 0.62 * (double)free_b) return AP_OK;
    const double mean = 0.45 * (double)cap;
    int64_t m = std::min<int64_t>(K, 24);
    int64_t cs = (int64_t)((double)m * (double)n / mean) + 1;
    const int64_t cs_min = g_ap_debug.seed_sample_cols > 0 ? std::max<int64_t>(K + 1, g_ap_debug.seed_sample_cols) : 4096;
    if (cs < cs_min || g_ap_debug.seed_sample_cols > 0) {   // a fixed sample: the rank that gives the same expectation
        cs = cs_min;
        m = std::min<int64_t>(K, std::max<int64_t>(m, (int64_t)(mean * (double)cs / (double)n) + 1));
    }
    cs = (cs + AP_TILE - 1) / AP_TILE * AP_TILE;
    if (n < 2 * cs) return AP_OK;
    if (g_ap_debug.seed_buffer_cap > 0) cap = g_ap_debug.seed_buffer_cap;   // forces overflows
    const int64_t RS = 8192;
    float *scratch = nullptr, *tau = nullptr, *tmp_sc = nullptr;
    unsigned long long *buf = nullptr;
    int32_t *cnt = nullptr, *ovf = nullptr;
    int rc = ap_dev_alloc(&buf, (size_t)n * (size_t)cap);
    if (rc != AP_OK) { (void)hipGetLastError(); ap_set_error("%s", ""); return AP_OK; }   // no room for the buffers after all: the one-sided sweep
    rc = ap_dev_alloc(&scratch, (size_t)RS * (size_t)cs);
    if (rc == AP_OK) rc = ap_dev_alloc(&tau, (size_t)n);
    if (rc == AP_OK) rc = ap_dev_alloc(&tmp_sc, (size_t)RS * (size_t)m);
    if (rc == AP_OK) rc = ap_dev_alloc(&cnt, (size_t)n);
    if (rc == AP_OK) rc = ap_dev_alloc(&ovf, (size_t)n + 1);
    hipError_t e = hipSuccess;
    int32_t *re_ids = nullptr; float *re_sc = nullptr, *ex_scratch = nullptr;
    if (rc == AP_OK) {
        // thresholds of all rows
        for (int64_t row0 = 0; row0 < n && e == hipSuccess; row0 += RS) {
            const int64_t nrows = std::min(RS, n - row0);
            dim3 gs(ap_seed_grid((nrows + AP_TILE - 1) / AP_TILE, cs / AP_TILE));
            ix->seed_flops += (unsigned long long)(((nrows + AP_TILE - 1) / AP_TILE) * (cs / AP_TILE)) * 2ull * AP_TILE * AP_TILE * (unsigned long long)ix->docs.dim;
            if (big)
                hipLaunchKernelGGL(k_seed_scores<AP_BF16>, gs, dim3(256), 0, st, ix->docs.dense, ix->docs.dim, n, (const int32_t *)nullptr, row0, nrows,
                                   (int64_t)0, cs, scratch);
            else
                hipLaunchKernelGGL(k_seed_scores<AP_F32>, gs, dim3(256), 0, st, ix->docs.dense, ix->docs.dim, n, (const int32_t *)nullptr, row0, nrows,
                                   (int64_t)0, cs, scratch);
            hipLaunchKernelGGL(k_select_rows, dim3((unsigned)nrows), dim3(256), 0, st, scratch, cs, (int32_t)m, (const int32_t *)nullptr, row0, 1,
                               (int64_t)0, (int32_t *)nullptr, tmp_sc);
            hipLaunchKernelGGL(k_take_tau, dim3((unsigned)((nrows + 255) / 256)), dim3(256), 0, st, tmp_sc, nrows, (int32_t)m,
                               (uint32_t)g_ap_debug.seed_tau_ulps, tau + row0);
            e = hipGetLastError();
        }
        if (e == hipSuccess) rc = ap_fill_u32(cnt, (size_t)n, 0u, st);
        if (rc == AP_OK) rc = ap_fill_u32(ovf, 1, 0u, st);
    }
    if (rc == AP_OK && e == hipSuccess) {
        ap_progress("seed lists: thresholds of %lld rows (rank %lld of %lld sampled columns), buffers of %lld", (long long)n, (long long)m,
                    (long long)cs, (long long)cap);
        // tiles multiplied: those on and above the diagonal, and the ragged last row and column of tiles
        ix->seed_flops += (unsigned long long)(T * (T + 1) / 2 + (n % E != 0 ? 2 * T + 1 : 0)) * 2ull * (unsigned long long)(E * E) * (unsigned long long)ix->docs.dim;
        if (big) {
            const dim3 tb(AP_BIG_WM * AP_BIG_WN * 64);
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_seed_thresh_big<AP_BIG_WM, AP_BIG_WN, true, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, AP_BIG_LDS_BYTES);
            if (e == hipSuccess)
                e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_seed_thresh_big<AP_BIG_WM, AP_BIG_WN, false, false>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, AP_BIG_LDS_BYTES);
            // the square of full tiles, a slab of 32 row tiles a launch: each XCD keeps four row tiles and walks the column
            // tiles from the slab's own first column on
            for (int64_t s0 = 0; s0 < T && e == hipSuccess; s0 += 32) {
                const int64_t nrt = std::min<int64_t>(32, T - s0), nct = T - s0;
                hipLaunchKernelGGL((k_seed_thresh_big<AP_BIG_WM, AP_BIG_WN, true, true>), dim3(ap_seed_grid(nrt, nct)), tb, AP_BIG_LDS_BYTES, st,
                                   ix->docs.dense, ix->docs.dim, n, (const int32_t *)nullptr, (int64_t)0, n, tau, buf, (int32_t)cap, cnt, s0, nrt, s0);
                e = hipGetLastError();
                if ((s0 / 32) % 64 == 63) {
                    if (e == hipSuccess) e = hipStreamSynchronize(st);
                    ap_progress("seed lists: %lld of %lld row tiles", (long long)(s0 + nrt), (long long)T);
                }
            }
            if (e == hipSuccess && n % AP_BIG != 0) {
                // the ragged last column tile for the full row tiles, and the ragged last rows against every column: one-sided
                hipLaunchKernelGGL((k_seed_thresh_big<AP_BIG_WM, AP_BIG_WN, false, false>), dim3(ap_seed_grid(T, 1)), tb, AP_BIG_LDS_BYTES, st,
                                   ix->docs.dense, ix->docs.dim, n, (const int32_t *)nullptr, (int64_t)0, n, tau, buf, (int32_t)cap, cnt, (int64_t)0, T, T);
                hipLaunchKernelGGL((k_seed_thresh_big<AP_BIG_WM, AP_BIG_WN, false, false>), dim3(ap_seed_grid(1, T + 1)), tb, AP_BIG_LDS_BYTES, st,
                                   ix->docs.dense, ix->docs.dim, n, (const int32_t *)nullptr, (int64_t)0, n, tau, buf, (int32_t)cap, cnt, T, (int64_t)1, (int64_t)0);
                e = hipGetLastError();
            }
        } else {
            // f32 rows: the same on 128x128 tiles, a slab of 64 row tiles (eight per XCD) a launch
            for (int64_t s0 = 0; s0 < T && e == hipSuccess; s0 += 64) {
                const int64_t nrt = std::min<int64_t>(64, T - s0), nct = T - s0, r0 = s0 * AP_TILE;
                hipLaunchKernelGGL((k_seed_thresh<AP_F32, true>), dim3(ap_seed_grid(nrt, nct)), dim3(256), 0, st, ix->docs.dense, ix->docs.dim, n,
                                   (const int32_t *)nullptr, r0, nrt * AP_TILE, tau + r0, buf + r0 * cap, (int32_t)cap, cnt + r0, s0);
                e = hipGetLastError();
            }
            if (e == hipSuccess && n % AP_TILE != 0) {
                const int64_t r0 = T * AP_TILE;
                hipLaunchKernelGGL((k_seed_thresh<AP_F32, false>), dim3(ap_seed_grid(T, 1)), dim3(256), 0, st, ix->docs.dense, ix->docs.dim, n,
                                   (const int32_t *)nullptr, (int64_t)0, r0, tau, buf, (int32_t)cap, cnt, T);
                hipLaunchKernelGGL((k_seed_thresh<AP_F32, false>), dim3(ap_seed_grid(1, T + 1)), dim3(256), 0, st, ix->docs.dense, ix->docs.dim, n,
                                   (const int32_t *)nullptr, r0, n - r0, tau + r0, buf + r0 * cap, (int32_t)cap, cnt + r0, (int64_t)0);
                e = hipGetLastError();
            }
        }
        int32_t n_ovf = 0;
        if (e == hipSuccess) {
            hipLaunchKernelGGL(k_select_buf, dim3((unsigned)n), dim3(256), 0, st, buf, (int32_t)cap, cnt, K, (int32_t)std::min<int64_t>(K, n - 1),
                               (int64_t)0, out_ids, out_sc, ovf, ovf + 1);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipMemcpyAsync(&n_ovf, ovf, sizeof(int32_t), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e == hipSuccess && n_ovf > 0) {   // rows left short or overflowing: the exact path
            ap_progress("seed lists: %d rows redone by the exact path", (int)n_ovf);
            (void)hipFree(buf); buf = nullptr;
            int64_t ex_rows = std::max<int64_t>(AP_TILE, (((int64_t)1 << 28) / n) / AP_TILE * AP_TILE);
            ex_rows = std::min<int64_t>(ex_rows, ((int64_t)n_ovf + AP_TILE - 1) / AP_TILE * AP_TILE);
            rc = ap_dev_alloc(&ex_scratch, (size_t)ex_rows * (size_t)n);
            if (rc == AP_OK) rc = ap_dev_alloc(&re_ids, (size_t)n_ovf * (size_t)K);
            if (rc == AP_OK) rc = ap_dev_alloc(&re_sc, (size_t)n_ovf * (size_t)K);
            if (rc == AP_OK) {
                e = seed_exact_rows(ix, ovf + 1, 0, n_ovf, K, ex_scratch, ex_rows, re_ids, re_sc, st);
                if (e == hipSuccess) {
                    const int64_t tot = (int64_t)n_ovf * K;
                    hipLaunchKernelGGL(k_scatter_rows, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, ovf + 1, (int64_t)n_ovf, K, re_ids, re_sc,
                                       out_ids, out_sc);
                    e = hipGetLastError();
                }
                if (e == hipSuccess) e = hipStreamSynchronize(st);
            }
        }
    }
    void *ptrs[] = {scratch, tau, tmp_sc, buf, cnt, ovf, ex_scratch, re_ids, re_sc};
    for (void *q : ptrs) if (q) (void)hipFree(q);
    if (rc != AP_OK) return rc;
    if (e != hipSuccess) { ap_set_error("seed k-NN failed: %s", hipGetErrorString(e)); return AP_EHIP; }
    *done = true;
    return AP_OK;
}

// S2.  Small corpora: every score row is materialised and the K best are
// selected from it.  Large corpora: the N x N scores are never stored: a
// sample of the columns gives each row a lower bound tau of its K-th best
// score, then one sweep over all columns appends only the scores >= tau to a
// per-row candidate buffer, from which the exact top-K is selected.  A row
// whose buffer overflows (not observed; the buffer holds twice the expected
// number of candidates) is redone by the exact path.
int ap_seed_knn_impl(const ap_index *ix, const int32_t *node_ids, int64_t nn, int32_t K, int32_t *out_ids,
                         float *out_sc, hipStream_t st) {
    const int64_t n = ix->docs.n;
    int64_t cs = std::max<int64_t>(16384, (n + 63) / 64);
    if (g_ap_debug.seed_sample_cols > 0) cs = std::max<int64_t>(K + 1, g_ap_debug.seed_sample_cols);
    cs = (cs + AP_TILE - 1) / AP_TILE * AP_TILE;
    // rows per launch of the exact path: a score slab of ~1 GiB
    int64_t ex_rows = std::max<int64_t>(AP_TILE, (((int64_t)1 << 28) / n) / AP_TILE * AP_TILE);
    ex_rows = std::min<int64_t>(ex_rows, (nn + AP_TILE - 1) / AP_TILE * AP_TILE);
    hipError_t e = hipSuccess;
    int rc = AP_OK;
    if (n < 2 * cs) {
        float *scratch = nullptr;
        AP_TRY(ap_dev_alloc(&scratch, (size_t)ex_rows * (size_t)n));
        e = seed_exact_rows(ix, node_ids, 0, nn, K, scratch, ex_rows, out_ids, out_sc, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        (void)hipFree(scratch);
        if (e != hipSuccess) { ap_set_error("seed k-NN failed: %s", hipGetErrorString(e)); return AP_EHIP; }
        return AP_OK;
    }
    if (!node_ids && !g_ap_debug.seed_one_sided) {   // the whole corpus: the symmetric sweep where it applies
        bool done = false;
        rc = ap_seed_knn_symmetric(ix, K, out_ids, out_sc, st, &done);
        if (rc != AP_OK || done) return rc;
    }
    const int64_t RS = std::min<int64_t>(8192, (nn + AP_TILE - 1) / AP_TILE * AP_TILE);
    // expected candidates per row = K * n / cs (tau is the K-th best of cs sampled columns)
    int64_t cap = 1024;
    while (cap < 2 * ((int64_t)K * n / cs + K)) cap <<= 1;
    if (g_ap_debug.seed_buffer_cap > 0) cap = g_ap_debug.seed_buffer_cap;   // forces overflows
    float *scratch = nullptr, *tau = nullptr, *tmp_sc = nullptr, *ex_scratch = nullptr;
    unsigned long long *buf = nullptr;
    int32_t *cnt = nullptr, *ovf = nullptr;   // ovf[0] = number of overflowed rows, ovf[1..] = their indices
    rc = ap_dev_alloc(&scratch, (size_t)RS * (size_t)cs);
    if (rc == AP_OK) rc = ap_dev_alloc(&tau, (size_t)RS);
    if (rc == AP_OK) rc = ap_dev_alloc(&tmp_sc, (size_t)RS * K);
    if (rc == AP_OK) rc = ap_dev_alloc(&buf, (size_t)RS * (size_t)cap);
    if (rc == AP_OK) rc = ap_dev_alloc(&cnt, (size_t)RS);
    if (rc == AP_OK) rc = ap_dev_alloc(&ovf, (size_t)RS + 1);
    for (int64_t row0 = 0; rc == AP_OK && row0 < nn && e == hipSuccess; row0 += RS) {
        const int64_t nrows = std::min(RS, nn - row0);
        const int64_t ytiles = (nrows + AP_TILE - 1) / AP_TILE;
        dim3 gs(ap_seed_grid(ytiles, cs / AP_TILE)), gf(ap_seed_grid(ytiles, (n + AP_TILE - 1) / AP_TILE));
        {   // FLOPs of the sample product and of the sweep (tiles of 128 for f32 rows, of 256 for bf16 rows)
            const unsigned long long d2 = 2ull * (unsigned long long)ix->docs.dim;
            ix->seed_flops += (unsigned long long)(ytiles * (cs / AP_TILE)) * AP_TILE * AP_TILE * d2;
            if (ix->dtype == AP_F32) ix->seed_flops += (unsigned long long)(ytiles * ((n + AP_TILE - 1) / AP_TILE)) * AP_TILE * AP_TILE * d2;
            else ix->seed_flops += (unsigned long long)(((nrows + AP_BIG - 1) / AP_BIG) * ((n + AP_BIG - 1) / AP_BIG)) * AP_BIG * AP_BIG * d2;
        }
        if (ix->dtype == AP_F32)
            hipLaunchKernelGGL(k_seed_scores<AP_F32>, gs, dim3(256), 0, st, ix->docs.dense, ix->docs.dim, n, node_ids, row0, nrows, (int64_t)0, cs, scratch);
        else
            hipLaunchKernelGGL(k_seed_scores<AP_BF16>, gs, dim3(256), 0, st, ix->docs.dense, ix->docs.dim, n, node_ids, row0, nrows, (int64_t)0, cs, scratch);
        hipLaunchKernelGGL(k_select_rows, dim3((unsigned)nrows), dim3(256), 0, st, scratch, cs, K, node_ids, row0, 1, (int64_t)0,
                           (int32_t *)nullptr, tmp_sc);
        hipLaunchKernelGGL(k_take_tau, dim3((unsigned)((nrows + 255) / 256)), dim3(256), 0, st, tmp_sc, nrows, K,
                           (uint32_t)g_ap_debug.seed_tau_ulps, tau);
        rc = ap_fill_u32(cnt, (size_t)nrows, 0u, st);
        if (rc == AP_OK) rc = ap_fill_u32(ovf, 1, 0u, st);
        if (rc != AP_OK) break;
        if (ix->dtype == AP_F32)
            hipLaunchKernelGGL((k_seed_thresh<AP_F32, false>), gf, dim3(256), 0, st, ix->docs.dense, ix->docs.dim, n, node_ids, row0, nrows, tau, buf, (int32_t)cap, cnt, (int64_t)0);
        else {
            // the inner tiles (runs of consecutive documents, all inside the corpus) take the lean instantiation, the ragged
            // last row tile and last column tile the general one
            const int64_t row_tiles = (nrows + AP_BIG - 1) / AP_BIG, col_tiles = (n + AP_BIG - 1) / AP_BIG;
            const bool runs = node_ids == nullptr && ix->docs.dim % AP_BK16 == 0;
            const int64_t full_rt = runs ? nrows / AP_BIG : 0, full_ct = runs ? n / AP_BIG : 0;
            auto sweep = [&](bool lean, int64_t rt0, int64_t nrt, int64_t ct0, int64_t nct) {
                if (nrt <= 0 || nct <= 0 || e != hipSuccess) return;
                const dim3 gb(ap_seed_grid(nrt, nct));
                const dim3 tb(AP_BIG_WM * AP_BIG_WN * 64);
                if (lean) {
                    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_seed_thresh_big<AP_BIG_WM, AP_BIG_WN, true, false>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, AP_BIG_LDS_BYTES);
                    if (e == hipSuccess)
                        hipLaunchKernelGGL((k_seed_thresh_big<AP_BIG_WM, AP_BIG_WN, true, false>), gb, tb, AP_BIG_LDS_BYTES, st, ix->docs.dense, ix->docs.dim, n,
                                           node_ids, row0, nrows, tau, buf, (int32_t)cap, cnt, rt0, nrt, ct0);
                } else {
                    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_seed_thresh_big<AP_BIG_WM, AP_BIG_WN, false, false>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, AP_BIG_LDS_BYTES);
                    if (e == hipSuccess)
                        hipLaunchKernelGGL((k_seed_thresh_big<AP_BIG_WM, AP_BIG_WN, false, false>), gb, tb, AP_BIG_LDS_BYTES, st, ix->docs.dense, ix->docs.dim, n,
                                           node_ids, row0, nrows, tau, buf, (int32_t)cap, cnt, rt0, nrt, ct0);
                }
                if (e == hipSuccess) e = hipGetLastError();
            };
            sweep(true, 0, full_rt, 0, full_ct);
            sweep(false, 0, full_rt, full_ct, col_tiles - full_ct);          // ragged last column tile
            sweep(false, full_rt, row_tiles - full_rt, 0, col_tiles);        // ragged last row tile (or everything)
            if (e != hipSuccess) break;
        }
        hipLaunchKernelGGL(k_select_buf, dim3((unsigned)nrows), dim3(256), 0, st, buf, (int32_t)cap, cnt, K,
                           (int32_t)std::min<int64_t>(K, n - 1), row0, out_ids, out_sc, ovf, ovf + 1);
        e = hipGetLastError();
        if (e != hipSuccess) break;
        int32_t n_ovf = 0;
        e = hipMemcpyAsync(&n_ovf, ovf, sizeof(int32_t), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) break;
        if ((row0 / RS) % 64 == 63) ap_progress("seed lists: %lld of %lld rows", (long long)(row0 + nrows), (long long)nn);
        if (n_ovf > 0) {   // redo the slab by the exact path
            if (!ex_scratch) rc = ap_dev_alloc(&ex_scratch, (size_t)ex_rows * (size_t)n);
            if (rc != AP_OK) break;
            e = seed_exact_rows(ix, node_ids, row0, nrows, K, ex_scratch, ex_rows, out_ids, out_sc, st);
        }
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    void *ptrs[] = {scratch, tau, tmp_sc, buf, cnt, ovf, ex_scratch};
    for (void *p : ptrs) if (p) (void)hipFree(p);
    if (rc != AP_OK) return rc;
    if (e != hipSuccess) { ap_set_error("seed k-NN failed: %s", hipGetErrorString(e)); return AP_EHIP; }
    return AP_OK;
}

extern "C" int ap_stage_seed_knn(const ap_index *ix, const int32_t *node_ids, int64_t nn, int32_t K, int32_t *out_ids,
                                 float *out_scores, void *stream) {
    AP_REQUIRE(ix && out_ids && out_scores, "NULL argument");
    AP_REQUIRE(K >= 1 && K <= 256, "K = %d must be in [1, 256]", K);
    if (!node_ids) nn = ix->docs.n;
    AP_REQUIRE(nn >= 0, "nn is negative");
    if (nn == 0) return AP_OK;
    return ap_seed_knn_impl(ix, node_ids, nn, K, out_ids, out_scores, (hipStream_t)stream);
}

extern "C" int ap_stage_entry_points(const ap_index *ix, int32_t E, int32_t *out_entry, void *stream) {
    AP_REQUIRE(ix && out_entry, "NULL argument");
    AP_REQUIRE(E >= 1 && E <= 256, "E = %d must be in [1, 256]", E);
    hipStream_t st = (hipStream_t)stream;
    float *sc = nullptr;
    AP_TRY(ap_dev_alloc(&sc, (size_t)E));
    hipLaunchKernelGGL(k_select_rows, dim3(1), dim3(256), 0, st, ix->self_sim, ix->docs.n, E, (const int32_t *)nullptr,
                       (int64_t)0, 0, (int64_t)0, out_entry, sc);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(sc);
    if (e != hipSuccess) { ap_set_error("entry point selection failed: %s", hipGetErrorString(e)); return AP_EHIP; }
    return AP_OK;
}

// =================================================================== S3: refinement round
#define AP_HT 4096
#define AP_MAXC 1280   // K + S*S <= 256 + 32*32

__device__ __forceinline__ bool ap_ht_insert(int32_t *ht, int32_t v) {
    uint32_t h = ((uint32_t)v * 2654435761u) >> 20;  // 12 bits
    for (;;) {
        const int32_t old = atomicCAS(&ht[h], -1, v);
        if (old == -1) return true;
        if (old == v) return false;
        h = (h + 1) & (AP_HT - 1);
    }
}
__device__ __forceinline__ bool ap_ht_has(const int32_t *ht, int32_t v) {
    uint32_t h = ((uint32_t)v * 2654435761u) >> 20;
    for (;;) {
        const int32_t cur = ht[h];
        if (cur == -1) return false;
        if (cur == v) return true;
        h = (h + 1) & (AP_HT - 1);
    }
}

#define AP_RT_SPB 10   // look-up tables of the node's own lists: 1024 + 512 slots, at most a quarter full
#define AP_RT_TXB 9
template <int DT, int NV>
__global__ __launch_bounds__(512) void k_refine(ApVecs D, const uint2 *__restrict__ rec, const uint4 *__restrict__ meta, float wd,
                                                float ws, float wf, int32_t K, int32_t S, int32_t P,
                                                const int32_t *__restrict__ knn, const int32_t *__restrict__ sp_ids,
                                                const float *__restrict__ sp_sc, const int32_t *__restrict__ node_ids,
                                                int64_t nn, int64_t x0, int32_t *__restrict__ out_ids, float *__restrict__ out_sc,
                                                int32_t *__restrict__ out_sp_ids, float *__restrict__ out_sp_sc,
                                                unsigned long long *__restrict__ n_sims) {
    __shared__ int32_t ht[AP_HT];
    __shared__ int32_t cand[AP_MAXC];
    __shared__ uint64_t keys[2048];   // the candidates' fused keys, sorted in place afterwards (AP_MAXC padded to a power of two)
    __shared__ float comp[3][AP_MAXC];
    __shared__ int32_t l_sp_idx[AP_A_CAP], l_tx_idx[AP_A_CAP];
    __shared__ float l_sp_val[AP_A_CAP], l_tx_val[AP_A_CAP];
    __shared__ uint64_t oldk[3][32];
    __shared__ __attribute__((aligned(16))) uint64_t qtab[(1 << AP_RT_SPB) + (1 << AP_RT_TXB)];
    __shared__ int32_t s_cnt, s_seed[2];
    const int64_t x = x0 + blockIdx.x;   // the launch covers nodes x0 .. x0 + gridDim.x of the nn
    const int64_t u = node_ids ? (int64_t)node_ids[x] : x;
    const int lane = threadIdx.x & 63, wave = ap_wave_id();
    const ApLists a = ap_stage_lists(D, u, l_sp_idx, l_sp_val, l_tx_idx, l_tx_val, AP_A_CAP);
    float qa[NV * ApDense<DT>::EPC];
    ap_load_aside<DT, NV, DT>(D.dense, u, D.dim, qa);
    for (int i = threadIdx.x; i < AP_HT; i += blockDim.x) ht[i] = -1;
    // the node's own lists as bucket tables with a hash multiplier of their own (the usual case: one 16-byte read per
    // look-up, as in the search); lists that are longer, or that no multiplier fits, are searched where they lie
    bool use_tab = a.sp_n <= (1 << AP_RT_SPB) / 4 && a.tx_n <= (1 << AP_RT_TXB) / 4;   // uniform
    uint32_t msp = 0, mtx = 0;
    if (threadIdx.x == 0) s_cnt = 0;
    __syncthreads();
    if (use_tab && wave == 0) {
        const int32_t s0 = ap_bucket_build<4>(a.sp_idx, a.sp_val, a.sp_n, qtab, AP_RT_SPB);
        const int32_t s1 = ap_bucket_build<2>(a.tx_idx, a.tx_val, a.tx_n, qtab + (1 << AP_RT_SPB), AP_RT_TXB);
        if (lane == 0) { s_seed[0] = s0; s_seed[1] = s1; }
    }
    __syncthreads();
    if (use_tab) {
        const int32_t seed0 = ap_uniform_i32(s_seed[0]), seed1 = ap_uniform_i32(s_seed[1]);
        use_tab = seed0 >= 0 && seed1 >= 0;
        if (use_tab) { msp = ap_seed_mult(seed0); mtx = ap_seed_mult(seed1); }
    }
    // candidates: own list, and the first S neighbours of the first S neighbours
    const int32_t sl = S < K ? S : K;
    const int32_t slots = K + sl * sl;
    for (int32_t s = threadIdx.x; s < slots; s += blockDim.x) {
        int32_t v;
        if (s < K) v = knn[u * K + s];
        else {
            const int32_t i = (s - K) / sl, j = (s - K) % sl;
            const int32_t p = knn[u * K + i];
            v = p < 0 ? -1 : knn[(int64_t)p * K + j];
        }
        if (v >= 0 && v != (int32_t)u && ap_ht_insert(ht, v)) cand[atomicAdd(&s_cnt, 1)] = v;
    }
    __syncthreads();
    const int32_t cnt = ap_uniform_i32(s_cnt);
    if (threadIdx.x == 0 && n_sims) atomicAdd(n_sims, (unsigned long long)cnt);   // measurement: similarities of this node and round
    // where each candidate's record lies and how long it is: fetched for all candidates at once, and parked in the space
    // the candidates' component scores take later, so that the scoring loop starts its loads without a round trip of its own
    if (use_tab) {
        for (int32_t t = threadIdx.x; t < cnt; t += blockDim.x) {
            const uint4 m = meta[cand[t]];
            comp[0][t] = __uint_as_float(m.x); comp[1][t] = __uint_as_float(m.y);
        }
        __syncthreads();
    }
    for (int32_t i = wave; i < cnt; i += (int32_t)(blockDim.x >> 6)) {
        const int32_t v = ap_uniform_i32(cand[i]);
        float sd, ss, sf;
        if (use_tab) {
            uint4 raw[NV];
            ap_dense_load_raw<DT, NV>(D, v, raw);   // the dense row is always needed here: its loads go first
            const uint32_t mx = ap_uniform_u32(__float_as_uint(comp[0][i])), my = ap_uniform_u32(__float_as_uint(comp[1][i]));
            const uint2 *r = rec + mx;
            const int32_t spn = (int32_t)(my & 0xffffu), txn = (int32_t)(my >> 16);
            int32_t si[2], ti[1];
            float sv[2], tv[1];
            ap_rec_load<2, 1>(r, spn, txn, si, sv, ti, tv);
            sd = ap_dense_dot_raw<DT, NV>(D, qa, raw);
            ap_rec_reduce_bucket<2, 1, AP_RT_SPB, AP_RT_TXB>(r, (const AP_LDS uint64_t *)qtab, (const AP_LDS uint64_t *)(qtab + (1 << AP_RT_SPB)),
                                                             msp, mtx, spn, txn, si, sv, ti, tv, ss, sf);
        } else {
            ap_hybrid_wave<DT, NV>(D, qa, a, v, sd, ss, sf);
        }
        if (lane == 0) {
            keys[i] = ap_make_key(ap_fuse(wd, ws, wf, sd, ss, sf), v, 1u);
            comp[0][i] = sd; comp[1][i] = ss; comp[2][i] = sf;
        }
    }
    // top-K under the fused score: the keys (all different: a key carries its id) sorted in LDS.  Ranking every key
    // against every other took a third of the kernel's vector instructions.
    int32_t n2 = 64;
    while (n2 < cnt) n2 <<= 1;   // uniform; cnt <= AP_MAXC <= 2048
    for (int32_t t = cnt + threadIdx.x; t < n2; t += blockDim.x) keys[t] = 0ull;
    ap_bitonic_desc(keys, n2);   // begins and ends with a barrier
    for (int32_t t = threadIdx.x; t < K; t += blockDim.x) {
        const uint64_t key = t < cnt ? keys[t] : 0ull;
        out_ids[x * K + t] = t < cnt ? ap_key_id(key) : -1;
        out_sc[x * K + t] = t < cnt ? ap_key_score(key) : -INFINITY;
    }
    // per-path lists: the best P by each single similarity among this round's candidates and the previous list (entries
    // scored again this round excepted).  One wave per path, on its own: every lane keeps its share of the keys in
    // registers and the P best are drawn one after the other by wave-wide maxima (no block-wide pass, no barrier).
    if (wave < 3) {
        const int p = wave;
        uint64_t ok = 0;
        bool have = false;
        if (lane < P) {
            const int32_t id = sp_ids[((int64_t)p * D.n + u) * P + lane];
            if (id >= 0 && !ap_ht_has(ht, id)) { have = true; ok = ap_make_key(sp_sc[((int64_t)p * D.n + u) * P + lane], id, 1u); }
        }
        const uint64_t hm = __ballot(have);
        const int32_t nold = (int32_t)__popcll(hm);
        if (have) oldk[p][__popcll(hm & ((1ull << lane) - 1ull))] = ok;
        ap_wave_sync();
        constexpr int PER = (AP_MAXC + 32 + 63) / 64;
        uint64_t mine[PER];
#pragma unroll
        for (int j = 0; j < PER; j++) {
            const int32_t t = j * 64 + lane;
            mine[j] = t < cnt ? ap_make_key(comp[p][t], cand[t], 1u) : (t < cnt + nold ? oldk[p][t - cnt] : 0ull);
        }
        uint64_t prev = ~0ull;
        for (int32_t r = 0; r < P; r++) {
            uint64_t best = 0;
#pragma unroll
            for (int j = 0; j < PER; j++)
                if (mine[j] < prev && mine[j] > best) best = mine[j];
            for (int o = 32; o > 0; o >>= 1) {
                const uint64_t other = __shfl_xor(best, o, 64);
                best = other > best ? other : best;
            }
            if (lane == 0) {
                out_sp_ids[((int64_t)p * nn + x) * P + r] = best ? ap_key_id(best) : -1;
                out_sp_sc[((int64_t)p * nn + x) * P + r] = best ? ap_key_score(best) : -INFINITY;
            }
            prev = best;   // 0 once exhausted: nothing ranks after it
        }
    }
}

extern "C" int ap_stage_refine(const ap_index *ix, int32_t K, int32_t S, int32_t P, const int32_t *knn_ids,
                               const int32_t *sp_ids, const float *sp_sc, const int32_t *node_ids, int64_t nn,
                               int32_t *out_ids, float *out_sc, int32_t *out_sp_ids, float *out_sp_sc, void *stream) {
    AP_REQUIRE(ix && knn_ids && sp_ids && sp_sc && out_ids && out_sc && out_sp_ids && out_sp_sc, "NULL argument");
    AP_REQUIRE(K >= 1 && K <= 256 && S >= 0 && S <= 32 && P >= 1 && P <= 32, "need 1<=K<=256, 0<=S<=32, 1<=P<=32");
    if (!node_ids) nn = ix->docs.n;
    if (nn <= 0) return AP_OK;
    const float *w = ix->params.build_w;
    const int64_t slice = AP_MAX_LAUNCH_THREADS / 512;   // a launch holds fewer than 2^32 threads
    for (int64_t x0 = 0; x0 < nn; x0 += slice) {
        const int64_t cn = std::min<int64_t>(slice, nn - x0);
        AP_DISPATCH_DENSE(ix->dtype, ix->docs.dim,
                          hipLaunchKernelGGL((k_refine<DT, NV>), dim3((unsigned)cn), dim3(512), 0, (hipStream_t)stream, ix->docs,
                                             ix->rec, ix->meta, w[0], w[1], w[2], K, S, P, knn_ids, sp_ids, sp_sc, node_ids, nn, x0, out_ids,
                                             out_sc, out_sp_ids, out_sp_sc, ix->counters));
        AP_CHECK_HIP(hipGetLastError());
    }
    return AP_OK;
}

// =================================================================== S4: neighbourhood similarities
// Dense part: G = X X^T for the K gathered rows of one neighbourhood (MFMA).
template <int DT>
__global__ __launch_bounds__(256) void k_gram_dense(const void *dense, int32_t dim, int32_t K, const int32_t *__restrict__ knn,
                                                    const int32_t *__restrict__ node_ids, int64_t x0,
                                                    float *__restrict__ pm /* chunk x K x K */) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[ApTileLds<DT>::BYTES];
    __shared__ int32_t a_rows[AP_TILE], b_rows[AP_TILE];
    const int64_t x = blockIdx.y;
    const int64_t u = node_ids ? (int64_t)node_ids[x0 + x] : x0 + x;
    const int32_t tiles = (K + AP_TILE - 1) / AP_TILE;
    const int32_t i0 = (blockIdx.x / tiles) * AP_TILE, j0 = (blockIdx.x % tiles) * AP_TILE;
    if (threadIdx.x < AP_TILE) {
        a_rows[threadIdx.x] = i0 + threadIdx.x < K ? knn[u * K + i0 + threadIdx.x] : -1;
        b_rows[threadIdx.x] = j0 + threadIdx.x < K ? knn[u * K + j0 + threadIdx.x] : -1;
    }
    ap_f32x16 acc[2][2];
    ap_tile_product<DT>(dense, dim, a_rows, b_rows, lds, acc);
    float *out = pm + x * (int64_t)K * K;
    ap_tile_foreach(acc, [&](int i, int j, float v) {
        if (i0 + i < K && j0 + j < K) out[(int64_t)(i0 + i) * K + (j0 + j)] = v;
    });
}

// Sparse and lexical parts of the neighbourhood similarities, and the fusion with the dense part: sorted lists are
// merged, one lane per pair.
// A 256-thread block takes a 16 x 16 tile of one neighbourhood's matrix (tiles on or below the diagonal; the matrix is
// symmetric and mirrored on output).  The packed records of the tile's 16 row and 16 column documents (sparse
// entries then lexical entries, ascending term ids) are copied to LDS, and thread (r, c) walks the two sorted lists
// of its pair with two cursors: about |a| + |b| steps, one 8-byte LDS read per step, products added in ascending
// term order.  Every lane works on a pair of its own, so an instruction serves 64 pairs; a wave-per-pair look-up
// scheme spends most of its instructions on terms the other list does not hold.
#define AP_GT 16                 // tile edge
#define AP_GT_ENTRIES 6144       // LDS budget of a tile: 32 records of ~165 entries; a tile that needs more reads global memory

// Straight-line body: every lane of the wave runs the same instructions until the last lane's lists are used up; a
// lane that is done keeps re-reading its last entries and adds nothing.
template <typename P>
__device__ __forceinline__ float ap_merge_dot(P a, int32_t na, P b, int32_t nb) {
    float acc = 0.f;
    bool live = na > 0 && nb > 0;
    int32_t pa = 0, pb = 0;
    uint64_t ea = live ? a[0] : 0ull, eb = live ? b[0] : 1ull;
    while (__any(live)) {
        const uint32_t ta = (uint32_t)ea, tb = (uint32_t)eb;
        const float prod = __uint_as_float((uint32_t)(ea >> 32)) * __uint_as_float((uint32_t)(eb >> 32));
        acc = (live && ta == tb) ? acc + prod : acc;
        pa += (live && ta <= tb) ? 1 : 0;
        pb += (live && tb <= ta) ? 1 : 0;
        live = live && pa < na && pb < nb;
        if (live) { ea = a[pa]; eb = b[pb]; }
    }
    return acc;
}

// The same walk over two lists in LDS that each end in a sentinel entry (weight 0) and one entry of padding: nothing is
// masked and no cursor is clamped.  The a side's sentinel term is 0xffffffff and a's cursor moves on "a's term <= b's
// term" compared UNSIGNED; the b side's is 0x7fffffff and b's cursor moves on "b's term <= a's term" compared SIGNED.
// Real terms lie in [0, 0x7fffffff), where the two orders agree; a's sentinel is the largest value of the unsigned
// order and b's the largest of the signed one, so a cursor that has reached its sentinel never moves again, whatever
// the other side shows, and the two sentinels never match each other or a term.  The walk tests "is any lane's pair
// still live" once per AP_GT_UNROLL steps: a lane whose pair is done idles on its sentinels.  a_end and b_end are the LDS byte
// addresses of the sentinels; same products in the same order as ap_merge_dot.
#define AP_GT_SENT 2
#define AP_GT_UNROLL 8   // steps per liveness test (prune stage of 200,000 documents: 2: 396 ms, 4: 361 ms, 8: 350 ms, 16: 351 ms)
#define AP_GT_SENT_A 0xffffffffull
#define AP_GT_SENT_B 0x7fffffffull
__device__ __forceinline__ float ap_merge_dot_lds(uint32_t a, uint32_t a_end, uint32_t b, uint32_t b_end) {
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));   // a plain vector value: loads from LDS as it is
    typedef const AP_LDS u32x2 *LP;
    auto at = [](uint32_t p) { return *(LP)(uintptr_t)p; };
    float acc = 0.f;
    // Each list's current entry and the one after it are in registers; a step reads the entry that follows the new
    // "next" position, which the step after it may select: the LDS round trip has a step's instructions to hide behind.
    u32x2 ea = at(a), eb = at(b), ea1 = at(a + 8u), eb1 = at(b + 8u);
    while (__any(a < a_end && b < b_end)) {
#pragma unroll
        for (int u = 0; u < AP_GT_UNROLL; u++) {
            const bool adva = ea.x <= eb.x, advb = (int32_t)eb.x <= (int32_t)ea.x;
            // adds exactly 0 when the terms differ (taking "both cursors move" for the match test saves the compare and
            // is no faster: the scalar AND of the two masks sits in the dependency chain)
            acc = fmaf(ea.x == eb.x ? __uint_as_float(ea.y) : 0.f, __uint_as_float(eb.y), acc);
            a = adva ? a + 8u : a; b = advb ? b + 8u : b;
            const u32x2 la = at(a + 8u), lb = at(b + 8u);
            ea.x = adva ? ea1.x : ea.x; ea.y = adva ? ea1.y : ea.y;
            eb.x = advb ? eb1.x : eb.x; eb.y = advb ? eb1.y : eb.y;
            ea1 = la; eb1 = lb;
        }
    }
    return acc;
}

__global__ __launch_bounds__(256) void k_gram_merge(const uint2 *__restrict__ rec, const uint4 *__restrict__ meta, float wd, float ws,
                                                    float wf, int32_t K, const int32_t *__restrict__ knn,
                                                    const int32_t *__restrict__ node_ids, int64_t x0, float *__restrict__ pm) {
    __shared__ uint64_t ent[AP_GT_ENTRIES];
    __shared__ int32_t d_id[2 * AP_GT], d_off[2 * AP_GT], d_sn[2 * AP_GT], d_tn[2 * AP_GT];
    __shared__ uint32_t d_first[2 * AP_GT];
    __shared__ int32_t s_total;
    const int64_t x = blockIdx.y;
    const int64_t u = node_ids ? (int64_t)node_ids[x0 + x] : x0 + x;
    // tile number -> (row block I, column block J), J <= I
    int32_t I = 0, rem = (int32_t)blockIdx.x;
    while (rem > I) { rem -= I + 1; I++; }
    const int32_t J = rem;
    const int tid = threadIdx.x, lane = tid & 63;
    if (tid < 64) {   // slots 0..15: row documents, 16..31: column documents
        int32_t id = -1, sn = 0, tn = 0;
        uint32_t first = 0;
        if (lane < 2 * AP_GT) {
            const int32_t pos = (lane < AP_GT ? I * AP_GT + lane : J * AP_GT + lane - AP_GT);
            if (pos < K) id = knn[u * K + pos];
            if (id >= 0) { const uint4 m = meta[id]; first = m.x; sn = (int32_t)(m.y & 0xffffu); tn = (int32_t)(m.y >> 16); }
        }
        const int32_t room = lane < 2 * AP_GT ? sn + tn + 2 * AP_GT_SENT : 0;   // a record in LDS: sparse entries, sentinels, lexical entries, sentinels
        int32_t incl = room;
        for (int o = 1; o < 64; o <<= 1) {
            const int32_t up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        if (lane < 2 * AP_GT) { d_id[lane] = id; d_off[lane] = incl - room; d_sn[lane] = sn; d_tn[lane] = tn; d_first[lane] = first; }
        if (lane == 2 * AP_GT - 1) s_total = incl;
    }
    __syncthreads();
    const bool in_lds = s_total <= AP_GT_ENTRIES;   // uniform
    const uint64_t *grec = reinterpret_cast<const uint64_t *>(rec);
    if (in_lds) {
        for (int d = 0; d < 2 * AP_GT; d++) {
            const int32_t sn = d_sn[d], len = sn + d_tn[d], off = d_off[d];
            const uint64_t *src = grec + d_first[d];
            for (int32_t e = tid; e < len; e += 256) ent[off + e + (e >= sn ? AP_GT_SENT : 0)] = src[e];
            if (tid < AP_GT_SENT) {   // slots 0..15 are a sides of the walks, 16..31 b sides
                const uint64_t sent = d < AP_GT ? AP_GT_SENT_A : AP_GT_SENT_B;
                ent[off + sn + tid] = sent; ent[off + len + AP_GT_SENT + tid] = sent;
            }
        }
        __syncthreads();
    }
    const int r = tid / AP_GT, c = tid % AP_GT;
    const int32_t i = I * AP_GT + r, j = J * AP_GT + c;
    if (i >= K || j >= K || j > i) return;
    float *out = pm + x * (int64_t)K * K;
    const int32_t a = d_id[r], b = d_id[AP_GT + c];
    float val = -INFINITY;
    if (a >= 0 && b >= 0) {
        float qs, qt;
        if (in_lds) {
            const uint32_t base = (uint32_t)(uintptr_t)(const AP_LDS uint64_t *)ent;
            const uint32_t la = base + 8u * (uint32_t)d_off[r], lb = base + 8u * (uint32_t)d_off[AP_GT + c];
            const uint32_t sa = 8u * (uint32_t)d_sn[r], sb = 8u * (uint32_t)d_sn[AP_GT + c];
            qs = ap_merge_dot_lds(la, la + sa, lb, lb + sb);
            const uint32_t ta = la + sa + 8u * AP_GT_SENT, tb = lb + sb + 8u * AP_GT_SENT;
            qt = ap_merge_dot_lds(ta, ta + 8u * (uint32_t)d_tn[r], tb, tb + 8u * (uint32_t)d_tn[AP_GT + c]);
        } else {
            const uint64_t *ga = grec + d_first[r], *gb = grec + d_first[AP_GT + c];
            qs = ap_merge_dot(ga, d_sn[r], gb, d_sn[AP_GT + c]);
            qt = ap_merge_dot(ga + d_sn[r], d_tn[r], gb + d_sn[AP_GT + c], d_tn[AP_GT + c]);
        }
        val = fmaf(wd, out[(int64_t)i * K + j], fmaf(wf, qt, ws * qs));
    }
    out[(int64_t)i * K + j] = val;
    out[(int64_t)j * K + i] = val;
}

// =================================================================== S4 + S5: detour sort, IP prune, keyword flags
// Detourable routes (Section 3.3): A -> X -> Y detours A -> Y iff
// min(sim(A,X), sim(X,Y)) > sim(A,Y).  Neighbours are stably sorted by their
// number of such routes, then walked in that order (Algorithm 1): v joins SE
// when |SE| < R and sim(w,v) < sim(v,v) for every w in SE; otherwise it is
// recycled as a keyword edge if its keyword flag is set, i.e. if it shares a
// keyword with A and no current member of SE covers all the shared keywords.
#define AP_T_CAP 512

__device__ __forceinline__ bool ap_list_has(const int32_t *idx, int64_t beg, int64_t end, int32_t t) {
    int64_t lo = beg, hi = end;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (idx[mid] < t) lo = mid + 1; else hi = mid;
    }
    return lo < end && idx[lo] == t;
}

// Where t stands in a list of n ascending ids in LDS, -1 if it is not there.
__device__ __forceinline__ int32_t ap_list_find_lds(const int32_t *idx, int32_t n, int32_t t) {
    int32_t lo = 0, hi = n;
    while (lo < hi) {
        const int32_t mid = (lo + hi) >> 1;
        if (idx[mid] < t) lo = mid + 1; else hi = mid;
    }
    return lo < n && idx[lo] == t ? lo : -1;
}

__global__ __launch_bounds__(256) void k_detour_prune(ApVecs D, const float *__restrict__ self_sim, int32_t K, int32_t R,
                                                      int32_t ke_cap, const int32_t *__restrict__ knn,
                                                      const float *__restrict__ knn_sc, const int32_t *__restrict__ node_ids,
                                                      int64_t x0, int64_t xout0, const float *__restrict__ pm,
                                                      int32_t *__restrict__ o_count, int32_t *__restrict__ o_sorted,
                                                      int32_t *__restrict__ o_se, int32_t *__restrict__ o_ke,
                                                      int32_t *__restrict__ o_ke_count, int32_t *__restrict__ o_flag,
                                                      int32_t mode) {
    __shared__ int32_t ids[256], cnt[256], order[256], se_pos[128], flag[256];
    __shared__ float simA[256];
    __shared__ int32_t T[AP_T_CAP];
    __shared__ int32_t a_tx[AP_T_CAP];   // the node's own keywords: every step of the walk searches them
    // Per keyword of the node, the members of SE that hold it (bit i = the i-th member; |SE| <= R <= 128).  "Some member
    // holds every shared keyword" is then an AND over the shared keywords' words instead of a search of every
    // member's list for every shared keyword.
    __shared__ unsigned long long kwm[AP_T_CAP][2];
    const int64_t x = blockIdx.x;               // index inside the chunk (pm)
    const int64_t xo = xout0 + x;               // index in the output arrays
    const int64_t u = node_ids ? (int64_t)node_ids[x0 + x] : x0 + x;
    const float *P = pm + x * (int64_t)K * K;
    const int t = threadIdx.x;
    if (t < K) { ids[t] = knn[u * K + t]; simA[t] = knn_sc[u * K + t]; flag[t] = 0; }
    const int64_t a_beg = D.tx_indptr[u], a_end = D.tx_indptr[u + 1];
    const bool a_in_lds = a_end - a_beg <= AP_T_CAP;   // uniform
    if (a_in_lds) for (int32_t e = t; e < (int32_t)(a_end - a_beg); e += 256) { a_tx[e] = D.tx_idx[a_beg + e]; kwm[e][0] = 0ull; kwm[e][1] = 0ull; }
    __syncthreads();
    if (t < K) {
        int32_t c = 0;
        if (ids[t] >= 0) {
            const float sy = simA[t];
            for (int32_t xx = 0; xx < K; xx++) {
                if (xx == t || ids[xx] < 0) continue;
                const float a = simA[xx], b = P[(int64_t)xx * K + t];
                c += (a < b ? a : b) > sy;
            }
        }
        cnt[t] = c;
    }
    __syncthreads();
    if (t < K) {
        int32_t r = 0;
        if (ids[t] >= 0) {
            if (mode == AP_PRUNE_IP_ONLY) {   // ablation: no detour sort, the list as ranked by similarity
                for (int32_t z = 0; z < t; z++) r += ids[z] >= 0;
            } else {
                for (int32_t z = 0; z < K; z++) r += ids[z] >= 0 && (cnt[z] < cnt[t] || (cnt[z] == cnt[t] && z < t));
            }
        } else {
            for (int32_t z = 0; z < K; z++) r += ids[z] >= 0 || z < t;
        }
        order[r] = t;
    }
    __syncthreads();
    if (t < K) {
        if (o_count) o_count[xo * K + t] = cnt[t];
        if (o_sorted) o_sorted[xo * K + t] = ids[order[t]];
    }
    if (t >= 64) return;   // the walk is sequential in v; one wave does it
    const int lane = t;
    const int64_t ab = D.tx_indptr[u], ae = D.tx_indptr[u + 1];
    int32_t nse = 0, nke = 0;
    for (int32_t r = 0; r < K; r++) {
        const int32_t pv = order[r], v = ids[pv];
        if (v < 0) break;   // holes are sorted last
        if (nse == 0 && !a_in_lds) { if (lane == 0) se_pos[0] = pv; nse = 1; ap_wave_sync(); continue; }
        // T = K(A) n K(v): the shared keywords themselves, or (node's list in LDS) their places in the node's list
        const int64_t vb = D.tx_indptr[v], ve = D.tx_indptr[v + 1];
        int32_t nt_all = 0;
        for (int64_t e0 = vb; e0 < ve; e0 += 64) {
            const int64_t e = e0 + lane;
            const int32_t term = e < ve ? D.tx_idx[e] : -1;
            int32_t at = -1;
            if (term >= 0) at = a_in_lds ? ap_list_find_lds(a_tx, (int32_t)(ae - ab), term) : (ap_list_has(D.tx_idx, ab, ae, term) ? 0 : -1);
            const bool in = at >= 0;
            const uint64_t m = __ballot(in);
            if (in) { const int32_t pos = nt_all + __popcll(m & ((1ull << lane) - 1ull)); if (pos < AP_T_CAP) T[pos] = a_in_lds ? at : term; }
            nt_all += __popcll(m);
        }
        ap_wave_sync();
        const int32_t nt = nt_all < AP_T_CAP ? nt_all : AP_T_CAP;
        if (nse == 0) {   // the first member of SE: its keywords are noted, nothing is tested
            if (lane == 0) se_pos[0] = pv;
            for (int32_t k = lane; k < nt; k += 64) kwm[T[k]][0] |= 1ull;
            nse = 1;
            ap_wave_sync();
            continue;
        }
        int32_t fl = 0;
        if (nt_all > 0 && a_in_lds) {
            // a member holds every shared keyword iff its bit survives the AND of those keywords' words
            unsigned long long w0 = ~0ull, w1 = ~0ull;
            for (int32_t k = lane; k < nt; k += 64) { w0 &= kwm[T[k]][0]; w1 &= kwm[T[k]][1]; }
            for (int32_t o = 32; o > 0; o >>= 1) { w0 &= __shfl_xor(w0, o); w1 &= __shfl_xor(w1, o); }
            fl = (w0 | w1) ? 0 : 1;
        } else if (nt_all > 0) {
            // does some member of SE hold every shared keyword?
            bool covered = false;
            for (int32_t i = lane; i < nse; i += 64) {
                const int32_t y = ids[se_pos[i]];
                const int64_t yb = D.tx_indptr[y], ye = D.tx_indptr[y + 1];
                bool all_in = true;
                for (int32_t k = 0; k < nt && all_in; k++) all_in = ap_list_has(D.tx_idx, yb, ye, T[k]);
                if (all_in && nt_all > AP_T_CAP) {   // rare: the shared set overflowed T; test the rest directly
                    for (int64_t e = vb; e < ve && all_in; e++) {
                        const int32_t term = D.tx_idx[e];
                        if (ap_list_has(D.tx_idx, ab, ae, term)) all_in = ap_list_has(D.tx_idx, yb, ye, term);
                    }
                }
                covered = covered || all_in;
            }
            fl = __ballot(covered) ? 0 : 1;
        }
        // IP test against every member of SE
        bool bad = false;
        const float sv = self_sim[v];
        if (mode != AP_PRUNE_RNG_ONLY)   // ablation: without the test SE is the first R of the detour order
            for (int32_t i = lane; i < nse; i += 64) bad = bad || !(P[(int64_t)se_pos[i] * K + pv] < sv);
        const bool ok = nse < R && !__ballot(bad);
        if (lane == 0) {
            flag[pv] = fl;
            if (ok) se_pos[nse] = pv;
            else if (fl && nke < ke_cap && o_ke) o_ke[xo * ke_cap + nke] = v;
        }
        if (ok && a_in_lds) for (int32_t k = lane; k < nt; k += 64) kwm[T[k]][nse >> 6] |= 1ull << (nse & 63);
        if (ok) nse++;
        else if (fl && nke < ke_cap) nke++;
        ap_wave_sync();
    }
    ap_wave_sync();
    for (int32_t i = lane; i < R; i += 64) if (o_se) o_se[xo * R + i] = i < nse ? ids[se_pos[i]] : -1;
    for (int32_t i = nke + lane; i < ke_cap; i += 64) if (o_ke) o_ke[xo * ke_cap + i] = -1;
    if (lane == 0 && o_ke_count) o_ke_count[xo] = nke;
    for (int32_t i = lane; i < K; i += 64) if (o_flag) o_flag[xo * K + i] = flag[i];
}

int ap_prune_impl(const ap_index *ix, int32_t K, int32_t R, const int32_t *knn_ids, const float *knn_sc,
                      const int32_t *node_ids, int64_t nn, float *pm_out, int32_t *count, int32_t *sorted_ids,
                      int32_t *se, int32_t *ke, int32_t *ke_count, int32_t *flag, hipStream_t st) {
    const int64_t per = (int64_t)K * K;
    int64_t chunk = pm_out ? nn : std::min<int64_t>(nn, std::max<int64_t>(1, ((int64_t)1 << 28) / per));
    float *scratch = nullptr;
    if (!pm_out) AP_TRY(ap_dev_alloc(&scratch, (size_t)chunk * (size_t)per));
    const float *w = ix->params.build_w;
    const int32_t tiles = (K + AP_TILE - 1) / AP_TILE;
    hipError_t e = hipSuccess;
    for (int64_t x0 = 0; x0 < nn && e == hipSuccess; x0 += chunk) {
        const int64_t cn = std::min(chunk, nn - x0);
        float *pm = pm_out ? pm_out + x0 * per : scratch;
        for (int64_t y0 = 0; y0 < cn && e == hipSuccess; y0 += 32768) {   // grid.y limit
            const int64_t yn = std::min<int64_t>(32768, cn - y0);
            dim3 g1((unsigned)(tiles * tiles), (unsigned)yn);
            if (ix->dtype == AP_F32)
                hipLaunchKernelGGL(k_gram_dense<AP_F32>, g1, dim3(256), 0, st, ix->docs.dense, ix->docs.dim, K, knn_ids, node_ids, x0 + y0, pm + y0 * per);
            else
                hipLaunchKernelGGL(k_gram_dense<AP_BF16>, g1, dim3(256), 0, st, ix->docs.dense, ix->docs.dim, K, knn_ids, node_ids, x0 + y0, pm + y0 * per);
            e = hipGetLastError();
            if (e != hipSuccess) break;
            const int32_t tb = (K + AP_GT - 1) / AP_GT;
            dim3 g2((unsigned)(tb * (tb + 1) / 2), (unsigned)yn);
            hipLaunchKernelGGL(k_gram_merge, g2, dim3(256), 0, st, ix->rec, ix->meta, w[0], w[1], w[2], K, knn_ids, node_ids, x0 + y0, pm + y0 * per);
            e = hipGetLastError();
        }
        if (e != hipSuccess) break;
        hipLaunchKernelGGL(k_detour_prune, dim3((unsigned)cn), dim3(256), 0, st, ix->docs, ix->self_sim, K, R, R / 2, knn_ids,
                           knn_sc, node_ids, x0, x0, pm, count, sorted_ids, se, ke, ke_count, flag, ix->params.prune_mode);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (scratch) (void)hipFree(scratch);
    if (e != hipSuccess) { ap_set_error("prune stage failed: %s", hipGetErrorString(e)); return AP_EHIP; }
    return AP_OK;
}

extern "C" int ap_stage_prune(const ap_index *ix, int32_t K, int32_t R, const int32_t *knn_ids, const float *knn_sc,
                              const int32_t *node_ids, int64_t nn, float *pm, int32_t *count, int32_t *sorted_ids,
                              int32_t *se, int32_t *ke, int32_t *ke_count, int32_t *flag, void *stream) {
    AP_REQUIRE(ix && knn_ids && knn_sc, "NULL argument");
    AP_REQUIRE(K >= 1 && K <= 256 && R >= 2 && R <= 128, "need 1<=K<=256, 2<=R<=128");
    if (!node_ids) nn = ix->docs.n;
    if (nn <= 0) return AP_OK;
    return ap_prune_impl(ix, K, R, knn_ids, knn_sc, node_ids, nn, pm, count, sorted_ids, se, ke, ke_count, flag, (hipStream_t)stream);
}

// =================================================================== S6: assembly
// Reverse neighbours of u: nodes x with u among the first q entries of SE(x),
// ordered by (position of u in SE(x), x); the first q that are not already
// forward neighbours of u.  Found in q rounds of an order-independent atomic
// minimum over all (x, pos) edges: round r keeps, per target, the smallest key
// above the one kept in round r-1.
__global__ void k_rev_round(const int32_t *__restrict__ se, int64_t n, int32_t R, int32_t q, int32_t round,
                            unsigned long long *__restrict__ rev /* n x q, ~0 = none */) {
    const int64_t total = n * q;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t xnode = e / q;
        const int32_t pos = (int32_t)(e % q);
        const int32_t u = se[xnode * R + pos];
        if (u < 0 || u == xnode) continue;
        const unsigned long long key = (((unsigned long long)pos << 32) | (unsigned long long)xnode) + 1ull;
        unsigned long long prev = 0;
        if (round > 0) {
            prev = rev[(int64_t)u * q + round - 1];
            if (prev == ~0ull) continue;
        }
        if (key <= prev) continue;
        bool fwd = false;                 // x already a forward neighbour of u?
        for (int32_t i = 0; i < q; i++) fwd = fwd || se[(int64_t)u * R + i] == (int32_t)xnode;
        if (!fwd) atomicMin(&rev[(int64_t)u * q + round], key);
    }
}

// One wave per node, following the order: SE[0:q], reverse neighbours, the
// per-path lists taken round-robin (dense, sparse, lexical) up to R/2, then
// padding from the rest of SE and from the detour-sorted list.
__global__ __launch_bounds__(256) void k_assemble(int64_t n, int32_t R, int32_t K, int32_t P, const int32_t *__restrict__ se,
                                                  const int32_t *__restrict__ sorted_ids, const int32_t *__restrict__ sp_ids,
                                                  const unsigned long long *__restrict__ rev, int64_t u0, int32_t *__restrict__ out) {
    __shared__ int32_t rows[4][128];
    const int lane = threadIdx.x & 63, wave = ap_wave_id();
    const int64_t u = u0 + (int64_t)blockIdx.x * 4 + wave;
    if (u >= n) return;
    int32_t *row = rows[wave];
    int32_t len = 0;
    const int32_t q = R / 4, h = R / 2;
    auto present = [&](int32_t v) -> bool {
        bool hit = false;
        for (int32_t i = lane; i < len; i += 64) hit = hit || row[i] == v;
        return __ballot(hit) != 0;
    };
    auto push = [&](int32_t v) -> bool {   // wave-uniform
        if (v < 0 || v == (int32_t)u || present(v)) return false;
        if (lane == 0) row[len] = v;
        len++;
        ap_wave_sync();
        return true;
    };
    for (int32_t i = 0; i < q; i++) push(se[u * R + i]);
    for (int32_t i = 0, added = 0; i < q && added < q; i++) {
        const unsigned long long key = rev[u * q + i];
        if (key == ~0ull) break;
        if (push((int32_t)((key - 1ull) & 0xffffffffull))) added++;
    }
    {
        int32_t ptr[3] = {0, 0, 0}, added = 0, turn = 0, idle = 0;
        while (added < h && idle < 3) {
            bool took = false;
            while (ptr[turn] < P) {
                const int32_t v = sp_ids[((int64_t)turn * n + u) * P + ptr[turn]];
                ptr[turn]++;
                if (push(v)) { added++; took = true; break; }
            }
            idle = took ? 0 : idle + 1;
            turn = (turn + 1) % 3;
        }
    }
    for (int32_t i = q; i < R && len < R; i++) push(se[u * R + i]);
    for (int32_t i = 0; i < K && len < R; i++) push(sorted_ids[u * K + i]);
    ap_wave_sync();
    for (int32_t i = lane; i < R; i += 64) out[u * R + i] = i < len ? row[i] : -1;
}

int ap_assemble_impl(const ap_index *ix, int32_t R, int32_t K, int32_t P, const int32_t *se, const int32_t *sorted_ids,
                         const int32_t *sp_ids, int32_t *out_graph, hipStream_t st) {
    const int64_t n = ix->docs.n;
    const int32_t q = R / 4;
    unsigned long long *rev = nullptr;
    AP_TRY(ap_dev_alloc(&rev, (size_t)n * (size_t)q));
    int rc = ap_fill_u32(rev, (size_t)n * q * 2, 0xffffffffu, st);
    hipError_t e = hipSuccess;
    if (rc == AP_OK) {
        const int64_t total = n * q;
        const unsigned blocks = (unsigned)std::min<int64_t>((total + 255) / 256, 65536);
        for (int32_t r = 0; r < q && e == hipSuccess; r++) {
            hipLaunchKernelGGL(k_rev_round, dim3(blocks), dim3(256), 0, st, se, n, R, q, r, rev);
            e = hipGetLastError();
        }
        if (e == hipSuccess) {
            const int64_t slice = AP_MAX_LAUNCH_THREADS / 64;   // four nodes per 256 threads
            for (int64_t u0 = 0; u0 < n && e == hipSuccess; u0 += slice) {
                const int64_t cn = std::min<int64_t>(slice, n - u0);
                hipLaunchKernelGGL(k_assemble, dim3((unsigned)((cn + 3) / 4)), dim3(256), 0, st, n, R, K, P, se, sorted_ids, sp_ids, rev, u0, out_graph);
                e = hipGetLastError();
            }
        }
        if (e == hipSuccess) e = hipStreamSynchronize(st);
    }
    (void)hipFree(rev);
    if (rc != AP_OK) return rc;
    if (e != hipSuccess) { ap_set_error("assemble stage failed: %s", hipGetErrorString(e)); return AP_EHIP; }
    return AP_OK;
}

extern "C" int ap_stage_assemble(const ap_index *ix, int32_t R, int32_t K, int32_t P, const int32_t *se,
                                 const int32_t *sorted_ids, const int32_t *sp_ids, int32_t *out_graph, void *stream) {
    AP_REQUIRE(ix && se && sorted_ids && sp_ids && out_graph, "NULL argument");
    AP_REQUIRE(R >= 4 && R % 4 == 0 && R <= 128 && K >= 1 && K <= 256 && P >= 1 && P <= 32, "need R%%4==0, 4<=R<=128, 1<=K<=256, 1<=P<=32");
    return ap_assemble_impl(ix, R, K, P, se, sorted_ids, sp_ids, out_graph, (hipStream_t)stream);
}

// =================================================================== the whole build
// Fused scores of existing lists (used when no refinement round runs).
template <int DT, int NV>
__global__ __launch_bounds__(256) void k_rescore_lists(ApVecs D, float wd, float ws, float wf, int32_t K, int64_t u0,
                                                       const int32_t *__restrict__ knn, float *__restrict__ sc) {
    __shared__ int32_t l_sp_idx[AP_A_CAP], l_tx_idx[AP_A_CAP];
    __shared__ float l_sp_val[AP_A_CAP], l_tx_val[AP_A_CAP];
    const int64_t u = u0 + blockIdx.x;
    const int lane = threadIdx.x & 63, wave = ap_wave_id();
    const ApLists a = ap_stage_lists(D, u, l_sp_idx, l_sp_val, l_tx_idx, l_tx_val, AP_A_CAP);
    float qa[NV * ApDense<DT>::EPC];
    ap_load_aside<DT, NV, DT>(D.dense, u, D.dim, qa);
    __syncthreads();
    for (int32_t i = wave; i < K; i += 4) {
        const int32_t v = knn[u * K + i];
        float s = -INFINITY;
        if (v >= 0) { float sd, ss, sf; ap_hybrid_wave<DT, NV>(D, qa, a, v, sd, ss, sf); s = ap_fuse(wd, ws, wf, sd, ss, sf); }
        if (lane == 0) sc[u * K + i] = s;
    }
}

// Fused scores (construction weights) of the first nn rows of existing lists.
int ap_rescore_lists(const ap_index *ix, int64_t nn, int32_t K, const int32_t *knn, float *sc, hipStream_t st) {
    if (nn <= 0) return AP_OK;
    const float *w = ix->params.build_w;
    const int64_t slice = AP_MAX_LAUNCH_THREADS / 256;
    for (int64_t u0 = 0; u0 < nn; u0 += slice) {
        const int64_t cn = std::min<int64_t>(slice, nn - u0);
        AP_DISPATCH_DENSE(ix->dtype, ix->docs.dim,
                          hipLaunchKernelGGL((k_rescore_lists<DT, NV>), dim3((unsigned)cn), dim3(256), 0, st, ix->docs, w[0], w[1], w[2],
                                             K, u0, knn, sc));
        AP_CHECK_HIP(hipGetLastError());
    }
    return AP_OK;
}

struct BuildBufs {
    int32_t *knn[2] = {nullptr, nullptr};
    float *knn_sc[2] = {nullptr, nullptr};
    int32_t *spi[2] = {nullptr, nullptr};
    float *sps[2] = {nullptr, nullptr};
    int32_t *se = nullptr, *sorted = nullptr;
    void release() {
        void *p[] = {knn[0], knn[1], knn_sc[0], knn_sc[1], spi[0], spi[1], sps[0], sps[1], se, sorted};
        for (void *x : p) if (x) (void)hipFree(x);
    }
};

static int build_impl(ap_index *ix, hipStream_t st, BuildBufs &b) {
    const ap_build_params &p = ix->params;
    const int64_t n = ix->corpus.n;   // ix->docs is only filled in by the ingest step below
    const int32_t K = p.knn_k, R = p.degree, P = p.sp_len;
    ApStageEvents marks;
    AP_CHECK_HIP(marks.create());
    hipEvent_t *ev = marks.ev;
    auto mark = [&](int i) { return hipEventRecord(ev[i], st); };
    AP_CHECK_HIP(mark(0));
    AP_TRY(ap_ingest_impl(ix, st));
    AP_CHECK_HIP(mark(1));
    for (int i = 0; i < 2; i++) {
        AP_TRY(ap_dev_alloc(&b.knn[i], (size_t)n * K));
        AP_TRY(ap_dev_alloc(&b.knn_sc[i], (size_t)n * K));
        AP_TRY(ap_dev_alloc(&b.spi[i], (size_t)3 * n * P));
        AP_TRY(ap_dev_alloc(&b.sps[i], (size_t)3 * n * P));
    }
    AP_TRY(ap_dev_alloc(&b.se, (size_t)n * R));
    AP_TRY(ap_dev_alloc(&b.sorted, (size_t)n * K));
    AP_TRY(ap_alloc_graph(ix));
    ap_progress("ingest done; seed lists of %lld documents", (long long)n);
    AP_TRY(ap_seed_knn_impl(ix, nullptr, n, K, b.knn[0], b.knn_sc[0], st));
    ap_progress("seed lists done; %d refinement rounds, pruning, assembly", p.nd_rounds);
    AP_CHECK_HIP(mark(2));
    AP_TRY(ap_fill_u32(b.spi[0], (size_t)3 * n * P, 0xffffffffu, st));          // id -1
    AP_TRY(ap_fill_u32(b.sps[0], (size_t)3 * n * P, 0xff800000u, st));          // -inf
    int cur = 0;
    for (int32_t t = 0; t < p.nd_rounds; t++) {
        AP_TRY(ap_stage_refine(ix, K, p.nd_sample, P, b.knn[cur], b.spi[cur], b.sps[cur], nullptr, n, b.knn[1 - cur],
                               b.knn_sc[1 - cur], b.spi[1 - cur], b.sps[1 - cur], st));
        cur = 1 - cur;
    }
    if (p.nd_rounds == 0) AP_TRY(ap_rescore_lists(ix, n, K, b.knn[cur], b.knn_sc[cur], st));
    AP_CHECK_HIP(mark(3));
    AP_TRY(ap_prune_impl(ix, K, R, b.knn[cur], b.knn_sc[cur], nullptr, n, nullptr, nullptr, b.sorted, b.se, ix->kw, ix->kw_count,
                      nullptr, st));
    AP_CHECK_HIP(mark(4));
    AP_TRY(ap_assemble_impl(ix, R, K, P, b.se, b.sorted, b.spi[cur], ix->graph, st));
    AP_TRY(ap_stage_entry_points(ix, p.n_entry, ix->entry, st));
    AP_CHECK_HIP(mark(5));
    AP_CHECK_HIP(hipStreamSynchronize(st));
    float total = 0.f;
    for (int i = 0; i < 5; i++) {
        float ms = 0.f;
        AP_CHECK_HIP(hipEventElapsedTime(&ms, ev[i], ev[i + 1]));
        ix->timings[i] = ms * 1e-3f;
        total += ms * 1e-3f;
    }
    ix->timings[5] = total;
    ix->has_graph = true;
    // kept for later insertions
    ix->st_se = b.se; ix->st_sorted = b.sorted; ix->st_spi = b.spi[cur]; ix->st_sps = b.sps[cur];
    b.se = nullptr; b.sorted = nullptr; b.spi[cur] = nullptr; b.sps[cur] = nullptr;
    return AP_OK;
}

extern "C" int ap_build_index(const ap_corpus *corpus, const ap_build_params *params, void *stream, ap_index **out) {
    AP_REQUIRE(out != nullptr, "out is NULL");
    *out = nullptr;
    AP_TRY(ap_validate_corpus(corpus));
    AP_TRY(ap_validate_params(params));
    AP_REQUIRE(corpus->n >= 2, "need at least two documents to build a graph");
    ap_index *ix = new (std::nothrow) ap_index();
    if (!ix) { ap_set_error("out of host memory"); return AP_ENOMEM; }
    ix->corpus = *corpus;
    ix->params = *params;
    if (ix->params.sp_len == 0) ix->params.sp_len = (ix->params.degree + 5) / 6;
    ix->dtype = corpus->dense_dtype;
    BuildBufs b;
    const int rc = build_impl(ix, (hipStream_t)stream, b);
    (void)hipStreamSynchronize((hipStream_t)stream);
    b.release();
    if (rc != AP_OK) { ap_free_index(ix); return rc; }
    *out = ix;
    return AP_OK;
}
