// S7-S9: batched best-first search on the semantic edges (Algorithm 2 without
// its keyword and entity branches), one workgroup per query.
//
// Per query, in LDS: the candidate pool (one sorted array of 64-bit keys that
// plays both `cand` and `topk` of Algorithm 2; bit 0 of a key = "not yet
// expanded"), the keys of the neighbours scored in this iteration, and the
// query's two sparse lists.  The query's dense slice stays in registers.  The
// visited set is an exact bitset (one bit per document) in a per-index global
// workspace.
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
};

// Ranks every new key and every pool key in the union and writes the best L
// of them, sorted, to `nxt`.  Keys are distinct (distinct documents), so the
// ranks are a permutation.
__device__ __forceinline__ void ap_pool_merge(const uint64_t *cur, int32_t len, const uint64_t *newk, int32_t c,
                                              uint64_t *nxt, int32_t L) {
    for (int32_t t = threadIdx.x; t < c; t += blockDim.x) {
        const uint64_t key = newk[t];
        int32_t r = 0;
        for (int32_t j = 0; j < c; j++) r += newk[j] > key;
        int32_t lo = 0, hi = len;  // pool keys ranking before `key`
        while (lo < hi) {
            const int32_t mid = (lo + hi) >> 1;
            if (cur[mid] > key) lo = mid + 1; else hi = mid;
        }
        r += lo;
        if (r < L) nxt[r] = key;
    }
    for (int32_t t = threadIdx.x; t < len; t += blockDim.x) {
        const uint64_t key = cur[t];
        int32_t r = t;
        for (int32_t j = 0; j < c; j++) r += newk[j] > key;
        if (r < L) nxt[r] = key;
    }
}

template <int DT, int NV>
__global__ __launch_bounds__(256) void k_search(ApSearchArgs g) {
    extern __shared__ uint64_t smem64[];
    uint64_t *poolA = smem64;
    uint64_t *poolB = poolA + g.L;
    uint64_t *newk = poolB + g.L;
    int32_t *cand = reinterpret_cast<int32_t *>(newk + g.cmax);
    int32_t *l_sp_idx = cand + g.cmax;
    float *l_sp_val = reinterpret_cast<float *>(l_sp_idx + AP_Q_CAP);
    int32_t *l_tx_idx = reinterpret_cast<int32_t *>(l_sp_val + AP_Q_CAP);
    float *l_tx_val = reinterpret_cast<float *>(l_tx_idx + AP_Q_CAP);
    __shared__ int32_t s_cnt, s_np;
    __shared__ int32_t s_par[8];

    const int64_t q = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const ApLists a = ap_stage_lists(g.Q, q, l_sp_idx, l_sp_val, l_tx_idx, l_tx_val, AP_Q_CAP);
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
    int32_t len = 0, it = 0;
    for (;;) {
        // score the c fresh candidates, one wave per candidate
        const int32_t c = s_cnt;
        for (int32_t i = wave; i < c; i += 4) {
            const int32_t v = cand[i];
            float sd, ss, sf;
            ap_hybrid_wave<DT, NV>(g.D, qa, a, v, sd, ss, sf);
            if (lane == 0) newk[i] = ap_make_key(ap_fuse(wd, ws, wf, sd, ss, sf), v, 1u);
        }
        __syncthreads();
        ap_pool_merge(cur, len, newk, c, nxt, g.L);
        len = len + c < g.L ? len + c : g.L;
        { uint64_t *t = cur; cur = nxt; nxt = t; }
        __syncthreads();
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
    AP_REQUIRE(p->beam >= 1 && p->beam <= 1024, "beam = %d must be in [1, 1024]", p->beam);
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
    g.visited = ix->visited;
    g.out_ids = out_ids;
    g.out_scores = out_scores;
    AP_TRY(ap_fill_u32(ix->visited, need, 0u, st));
    const size_t smem = (size_t)(2 * g.L + g.cmax) * 8 + (size_t)g.cmax * 4 + 4 * AP_Q_CAP * 4;
    AP_DISPATCH_DENSE(ix->dtype, ix->docs.dim,
                      hipLaunchKernelGGL((k_search<DT, NV>), dim3((unsigned)q->nq), dim3(256), smem, st, g));
    AP_CHECK_HIP(hipGetLastError());
    return AP_OK;
}
