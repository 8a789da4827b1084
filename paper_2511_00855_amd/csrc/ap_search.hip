// S7-S9: batched best-first search on the semantic edges (Algorithm 2 without
// its keyword and entity branches), one workgroup per query.
//
// Per query, in LDS: the candidate pool (one sorted array of 64-bit keys that
// plays both `cand` and `topk` of Algorithm 2; bit 0 of a key = "not yet
// expanded"), the keys of the neighbours scored in this iteration, and the
// query's two sparse lists.  The query's dense slice stays in registers.  The
// visited set is an exact bitset (one bit per document) in a per-index global
// workspace.
#include <stdlib.h>
#include "ap_common.hpp"

#define AP_Q_CAP 128  // query list entries staged in LDS

int ap_fill_u32(void *p, size_t n, uint32_t v, hipStream_t st);
int ap_validate_queries(const ap_queries *q);

struct ApSearchArgs {
    ApVecs D, Q;
    const int32_t *graph;
    const int32_t *entry;
    const float *w;     // per query (stride 3) or the index default (stride 0)
    int32_t w_stride;
    int32_t R, E, k, L, max_iters, width, cmax;
    uint32_t *visited;
    size_t words;       // visited words per query
    int32_t *out_ids;
    float *out_scores;
    int32_t *counts;    // nq x 2: similarities evaluated, iterations
};

// Number of entries of the descending array keys[0..n) that rank before `key`.
__device__ __forceinline__ int32_t ap_rank_in(const uint64_t *keys, int32_t n, uint64_t key) {
    int32_t lo = 0, hi = n;
    while (lo < hi) {
        const int32_t mid = (lo + hi) >> 1;
        if (keys[mid] > key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Scores the c candidates of this iteration: wave w takes candidates
// w, w+4, ... in groups of G whose loads are all in flight together.
template <int DT, int NV, int G, typename IP, typename VP>
__device__ __forceinline__ void ap_score_candidates(const ApVecs &D, const float *qa, IP sp_idx, VP sp_val, int32_t sp_n,
                                                    IP tx_idx, VP tx_val, int32_t tx_n, float wd, float ws, float wf,
                                                    const int32_t *cand, const int64_t *s_spb, const int32_t *s_spn,
                                                    const int64_t *s_txb, const int32_t *s_txn, int32_t c, uint64_t *newk) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int32_t i0 = wave; i0 < c; i0 += 4 * G) {
        int32_t v[G], spn[G], txn[G];
        int64_t spb[G], txb[G];
        int32_t ng = 0;
#pragma unroll
        for (int g = 0; g < G; g++) {
            const int32_t i = i0 + 4 * g;
            if (i < c) { v[g] = cand[i]; spb[g] = s_spb[i]; spn[g] = s_spn[i]; txb[g] = s_txb[i]; txn[g] = s_txn[i]; ng = g + 1; }
        }
        float sd[G], ss[G], sf[G];
        ap_hybrid_batch<DT, NV, G, 2, 1>(D, qa, sp_idx, sp_val, sp_n, tx_idx, tx_val, tx_n, ng, v, spb, spn, txb, txn, sd, ss, sf);
        if (lane == 0) {
#pragma unroll
            for (int g = 0; g < G; g++)
                if (g < ng) newk[i0 + 4 * g] = ap_make_key(ap_fuse(wd, ws, wf, sd[g], ss[g], sf[g]), v[g], 1u);
        }
    }
}

template <int DT, int NV, int AP_SEARCH_G>
__global__ __launch_bounds__(256) void k_search(ApSearchArgs g) {
    extern __shared__ uint64_t smem64[];
    uint64_t *poolA = smem64;
    uint64_t *poolB = poolA + g.L;
    uint64_t *newk = poolB + g.L;            // keys of this iteration's candidates, unordered
    uint64_t *newS = newk + g.cmax;          // the same, sorted
    int64_t *s_spb = reinterpret_cast<int64_t *>(newS + g.cmax);
    int64_t *s_txb = s_spb + g.cmax;
    int32_t *s_spn = reinterpret_cast<int32_t *>(s_txb + g.cmax);
    int32_t *s_txn = s_spn + g.cmax;
    int32_t *cand = s_txn + g.cmax;
    int32_t *l_sp_idx = cand + g.cmax;
    float *l_sp_val = reinterpret_cast<float *>(l_sp_idx + AP_Q_CAP);
    int32_t *l_tx_idx = reinterpret_cast<int32_t *>(l_sp_val + AP_Q_CAP);
    float *l_tx_val = reinterpret_cast<float *>(l_tx_idx + AP_Q_CAP);
    __shared__ int32_t s_cnt, s_np;
    __shared__ int32_t s_par[8];

    const int64_t q = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const ApLists a = ap_stage_lists(g.Q, q, l_sp_idx, l_sp_val, l_tx_idx, l_tx_val, AP_Q_CAP);
    const bool in_lds = a.sp_n <= AP_Q_CAP && a.tx_n <= AP_Q_CAP;   // uniform
    float qa[NV * ApDense<DT>::EPC];
    ap_load_aside<DT, NV, AP_F32>(g.Q.dense, q, g.D.dim, qa);
    const float wd = g.w[q * g.w_stride + 0], ws = g.w[q * g.w_stride + 1], wf = g.w[q * g.w_stride + 2];
    uint32_t *vis = g.visited + (size_t)q * g.words;
    if (threadIdx.x == 0) s_cnt = 0;
    __syncthreads();

    // S7: entry points
    for (int32_t i = threadIdx.x; i < g.E; i += blockDim.x) {
        const int32_t v = g.entry[i];
        if (v >= 0) {
            const uint32_t bit = 1u << (v & 31);
            const uint32_t old = atomicOr(&vis[v >> 5], bit);
            if (!(old & bit)) cand[atomicAdd(&s_cnt, 1)] = v;
        }
    }
    __syncthreads();
    uint64_t *cur = poolA, *nxt = poolB;
    int32_t len = 0, it = 0, nscored = 0;
    for (;;) {
        const int32_t c = s_cnt;
        nscored += c;
        // where each candidate's lists are: one round of loads for all of them
        for (int32_t i = threadIdx.x; i < c; i += blockDim.x) {
            const int32_t v = cand[i];
            const int64_t sb = g.D.sp_indptr[v], tb = g.D.tx_indptr[v];
            s_spb[i] = sb; s_spn[i] = (int32_t)(g.D.sp_indptr[v + 1] - sb);
            s_txb[i] = tb; s_txn[i] = (int32_t)(g.D.tx_indptr[v + 1] - tb);
        }
        __syncthreads();
        if (in_lds)
            ap_score_candidates<DT, NV, AP_SEARCH_G>(g.D, qa, (const AP_LDS int32_t *)l_sp_idx, (const AP_LDS float *)l_sp_val,
                                                     a.sp_n, (const AP_LDS int32_t *)l_tx_idx, (const AP_LDS float *)l_tx_val,
                                                     a.tx_n, wd, ws, wf, cand, s_spb, s_spn, s_txb, s_txn, c, newk);
        else
            ap_score_candidates<DT, NV, AP_SEARCH_G>(g.D, qa, a.sp_idx, a.sp_val, a.sp_n, a.tx_idx, a.tx_val, a.tx_n, wd, ws, wf,
                                                     cand, s_spb, s_spn, s_txb, s_txn, c, newk);
        __syncthreads();
        // sort the new keys by ranking them among themselves; only those that
        // rank before the pool's last entry (when the pool is full) can enter
        const uint64_t worst = len == g.L ? cur[g.L - 1] : 0ull;
        for (int32_t t = threadIdx.x; t < c; t += blockDim.x) {
            const uint64_t key = newk[t];
            int32_t r = 0;
            for (int32_t j = 0; j < c; j++) r += newk[j] > key;
            newS[r] = key;
        }
        __syncthreads();
        int32_t cin = ap_rank_in(newS, c, worst);   // new keys that rank before `worst` (all of them while the pool has room)
        if (cin > 0) {
            for (int32_t t = threadIdx.x; t < cin; t += blockDim.x) {
                const uint64_t key = newS[t];
                const int32_t r = t + ap_rank_in(cur, len, key);
                if (r < g.L) nxt[r] = key;
            }
            for (int32_t t = threadIdx.x; t < len; t += blockDim.x) {
                const uint64_t key = cur[t];
                const int32_t r = t + ap_rank_in(newS, cin, key);
                if (r < g.L) nxt[r] = key;
            }
            len = len + cin < g.L ? len + cin : g.L;
            { uint64_t *t = cur; cur = nxt; nxt = t; }
            __syncthreads();
        }
        if (g.max_iters > 0 && it >= g.max_iters) break;
        // S8: pick the best `width` unexpanded entries (wave 0), mark them expanded
        if (wave == 0) {
            int32_t found = 0;
            for (int32_t base = 0; base < len && found < g.width; base += 64) {
                const int32_t i = base + lane;
                const bool un = i < len && (cur[i] & 1ull);
                const uint64_t mask = __ballot(un);
                const int32_t rank = __popcll(mask & ((1ull << lane) - 1ull));
                if (un && found + rank < g.width) {
                    s_par[found + rank] = ap_key_id(cur[i]);
                    cur[i] &= ~1ull;
                }
                found += __popcll(mask);
            }
            if (lane == 0) { s_np = found < g.width ? found : g.width; s_cnt = 0; }
        }
        __syncthreads();
        const int32_t np = s_np;
        if (np == 0) break;
        // neighbours of the parents that were never seen before
        for (int32_t i = threadIdx.x; i < np * g.R; i += blockDim.x) {
            const int32_t v = g.graph[(int64_t)s_par[i / g.R] * g.R + (i % g.R)];
            if (v >= 0) {
                const uint32_t bit = 1u << (v & 31);
                const uint32_t old = atomicOr(&vis[v >> 5], bit);
                if (!(old & bit)) cand[atomicAdd(&s_cnt, 1)] = v;
            }
        }
        __syncthreads();
        it++;
    }
    if (threadIdx.x == 0) { g.counts[q * 2] = nscored; g.counts[q * 2 + 1] = it; }
    // S9
    for (int32_t i = threadIdx.x; i < g.k; i += blockDim.x) {
        g.out_ids[q * g.k + i] = i < len ? ap_key_id(cur[i]) : -1;
        g.out_scores[q * g.k + i] = i < len ? ap_key_score(cur[i]) : -INFINITY;
    }
}

extern "C" int ap_search_batch(ap_index *ix, const ap_queries *q, const float *per_query_w,
                               const ap_search_params *p, int32_t *out_ids, float *out_scores, void *stream) {
    AP_REQUIRE(ix && p, "NULL argument");
    if (!ix->has_graph) { ap_set_error("index has no graph: build or import one first"); return AP_ESTATE; }
    AP_TRY(ap_validate_queries(q));
    AP_REQUIRE(q->nq == 0 || (out_ids && out_scores), "NULL output");
    AP_REQUIRE(p->beam >= 1 && p->beam <= 4096, "beam = %d must be in [1, 4096]", p->beam);
    AP_REQUIRE(p->k >= 1 && p->k <= p->beam, "k = %d must be in [1, beam]", p->k);
    AP_REQUIRE(p->search_width >= 1 && p->search_width <= 8, "search_width = %d must be in [1, 8]", p->search_width);
    AP_REQUIRE(p->max_iters >= 0, "max_iters must be >= 0");
    if (q->nq == 0) return AP_OK;
    hipStream_t st = (hipStream_t)stream;
    ApSearchArgs g;
    g.D = ix->docs;
    g.Q = ApVecs{q->nq, ix->docs.dim, q->dense, q->sp_indptr, q->sp_idx, q->sp_val, q->tx_indptr, q->tx_idx, q->tx_cnt};
    g.graph = ix->graph;
    g.entry = ix->entry;
    g.w = per_query_w ? per_query_w : ix->w_dev;
    g.w_stride = per_query_w ? 3 : 0;
    g.R = ix->params.degree;
    g.E = ix->params.n_entry;
    g.k = p->k; g.L = p->beam; g.max_iters = p->max_iters; g.width = p->search_width;
    g.cmax = g.E > g.width * g.R ? g.E : g.width * g.R;
    g.words = ((size_t)ix->docs.n + 31) / 32;
    const size_t need = g.words * (size_t)q->nq;
    if (need > ix->visited_words) {
        if (ix->visited) { AP_CHECK_HIP(hipStreamSynchronize(st)); (void)hipFree(ix->visited); ix->visited = nullptr; ix->visited_words = 0; }
        AP_TRY(ap_dev_alloc(&ix->visited, need));
        ix->visited_words = need;
    }
    if ((size_t)q->nq * 2 > ix->search_counts_cap) {
        if (ix->search_counts) { AP_CHECK_HIP(hipStreamSynchronize(st)); (void)hipFree(ix->search_counts); ix->search_counts = nullptr; ix->search_counts_cap = 0; }
        AP_TRY(ap_dev_alloc(&ix->search_counts, (size_t)q->nq * 2));
        ix->search_counts_cap = (size_t)q->nq * 2;
    }
    if (!ix->ev_search[0]) {
        AP_CHECK_HIP(hipEventCreate(&ix->ev_search[0]));
        AP_CHECK_HIP(hipEventCreate(&ix->ev_search[1]));
    }
    g.visited = ix->visited;
    g.out_ids = out_ids;
    g.out_scores = out_scores;
    g.counts = ix->search_counts;
    ix->last_nq = q->nq;
    AP_TRY(ap_fill_u32(ix->visited, need, 0u, st));
    const size_t smem = (size_t)(2 * g.L + 2 * g.cmax) * 8 + (size_t)g.cmax * (8 + 8 + 4 + 4 + 4) + 4 * AP_Q_CAP * 4;
    AP_CHECK_HIP(hipEventRecord(ix->ev_search[0], st));
    AP_REQUIRE(smem <= 160 * 1024, "beam and search_width need %zu bytes of LDS (limit 160 KiB)", smem);
    hipError_t le = hipSuccess;
    static const int rows_in_flight = [] { const char *e = getenv("AP_SEARCH_ROWS_IN_FLIGHT"); return e ? atoi(e) : 1; }();
#define AP_LAUNCH_SEARCH(GG)                                                                                     \
    do {                                                                                                         \
        if (smem > 48 * 1024)                                                                                    \
            le = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_search<DT, NV, GG>),                      \
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);                     \
        if (le == hipSuccess) hipLaunchKernelGGL((k_search<DT, NV, GG>), dim3((unsigned)q->nq), dim3(256), smem, st, g); \
    } while (0)
    AP_DISPATCH_DENSE(ix->dtype, ix->docs.dim, {
        if (rows_in_flight <= 1) AP_LAUNCH_SEARCH(1);
        else if (rows_in_flight == 2) AP_LAUNCH_SEARCH(2);
        else if (rows_in_flight == 3) AP_LAUNCH_SEARCH(3);
        else AP_LAUNCH_SEARCH(4);
    });
#undef AP_LAUNCH_SEARCH
    AP_CHECK_HIP(le);
    AP_CHECK_HIP(hipGetLastError());
    AP_CHECK_HIP(hipEventRecord(ix->ev_search[1], st));
    return AP_OK;
}

extern "C" int ap_search_stats(const ap_index *ix, int32_t *out_counts, int32_t nq, float *kernel_ms, void *stream) {
    AP_REQUIRE(ix, "index is NULL");
    if (!ix->ev_search[1] || ix->last_nq == 0) { ap_set_error("no search has run on this index"); return AP_ESTATE; }
    AP_CHECK_HIP(hipEventSynchronize(ix->ev_search[1]));
    if (kernel_ms) AP_CHECK_HIP(hipEventElapsedTime(kernel_ms, ix->ev_search[0], ix->ev_search[1]));
    if (out_counts) {
        AP_REQUIRE(nq == ix->last_nq, "nq = %d does not match the last search (%d)", nq, ix->last_nq);
        AP_CHECK_HIP(hipMemcpyAsync(out_counts, ix->search_counts, (size_t)nq * 2 * sizeof(int32_t), hipMemcpyDeviceToDevice,
                                    (hipStream_t)stream));
    }
    return AP_OK;
}
