// Knowledge-graph augmentation: logical edges (Section 3.4; Algorithm 1's last
// step) and the entity branches of the search (Section 4.2.3; Algorithm 2).
//
// The caller supplies, per document, the entities it mentions, and the
// relations between entities (both CSR, ascending).  Construction derives the
// entity-to-document mapping and, per document x, its logical edges: triples
// (s, y, t) with s an entity of x, (s, t) a relation, t not an entity of x and
// y != x a document that mentions t, in ascending (s, t, y) order, at most
// le_cap of them.  The search carries with every pool entry the entity that
// ties it to the query's entities and the number of relations in between
// (hop); a tie raises the score by w_k / hop.
//
// The paper applies this to small, high-value shards; the search here is a
// plain one-workgroup-per-query kernel (sorted pool in LDS, one insertion at a
// time), not the tuned kernel of the ordinary search.
#include <string.h>
#include <algorithm>
#include "ap_common.hpp"

int ap_validate_queries(const ap_queries *q);

// ------------------------------------------------------------------ construction
__global__ void k_ent_count(const int64_t *__restrict__ de_ip, const int32_t *__restrict__ de, int64_t n, int32_t n_ent, int64_t total,
                            unsigned long long *__restrict__ cnt, int32_t *__restrict__ bad) {
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < n; x += (int64_t)gridDim.x * blockDim.x) {
        if (!ap_row_ok(de_ip, x, total)) { atomicAdd(bad, 1); continue; }
        for (int64_t p = de_ip[x]; p < de_ip[x + 1]; p++) {
            const int32_t e = de[p];
            if (e < 0 || e >= n_ent || (p > de_ip[x] && de[p - 1] >= e)) { atomicAdd(bad, 1); continue; }
            atomicAdd(&cnt[e], 1ull);
        }
    }
}

// relations must name entities, ascending per row, no self-relation
__global__ void k_kg_check(const int64_t *__restrict__ kg_ip, const int32_t *__restrict__ kg, int32_t n_ent, int64_t total,
                           int32_t *__restrict__ bad) {
    for (int64_t s = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; s < n_ent; s += (int64_t)gridDim.x * blockDim.x) {
        if (!ap_row_ok(kg_ip, s, total)) { atomicAdd(bad, 1); continue; }
        for (int64_t p = kg_ip[s]; p < kg_ip[s + 1]; p++) {
            const int32_t t = kg[p];
            if (t < 0 || t >= n_ent || t == s || (p > kg_ip[s] && kg[p - 1] >= t)) atomicAdd(bad, 1);
        }
    }
}

// Exclusive prefix sum of cnt[0..m) into out[0..m] by one workgroup: each thread sums a contiguous chunk, the
// chunk totals are scanned in LDS, each thread writes its chunk.
__global__ __launch_bounds__(1024) void k_exclusive_scan(const unsigned long long *__restrict__ cnt, int64_t m, int64_t *__restrict__ out) {
    __shared__ unsigned long long part[1024];
    const int64_t chunk = (m + 1023) / 1024;
    const int64_t lo = threadIdx.x * chunk, hi = lo + chunk < m ? lo + chunk : m;
    unsigned long long s = 0;
    for (int64_t i = lo; i < hi; i++) s += cnt[i];
    part[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long run = 0;
        for (int i = 0; i < 1024; i++) { const unsigned long long v = part[i]; part[i] = run; run += v; }
        out[m] = (int64_t)run;
    }
    __syncthreads();
    unsigned long long run = part[threadIdx.x];
    for (int64_t i = lo; i < hi; i++) { out[i] = (int64_t)run; run += cnt[i]; }
}

__global__ void k_ent_fill(const int64_t *__restrict__ de_ip, const int32_t *__restrict__ de, int64_t n, const int64_t *__restrict__ en_ip,
                           unsigned long long *__restrict__ cursor, int32_t *__restrict__ tmp) {
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < n; x += (int64_t)gridDim.x * blockDim.x)
        for (int64_t p = de_ip[x]; p < de_ip[x + 1]; p++) {
            const int32_t e = de[p];
            tmp[en_ip[e] + (int64_t)atomicAdd(&cursor[e], 1ull)] = (int32_t)x;
        }
}

// The documents of an entity arrive in any order; each finds its place by counting the smaller ones (ids are distinct).
__global__ void k_ent_rank(const int64_t *__restrict__ en_ip, int32_t n_ent, const int32_t *__restrict__ tmp, int32_t *__restrict__ en) {
    const int64_t total = en_ip[n_ent];
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        int32_t lo = 0, hi = n_ent;                 // the entity whose segment holds position i
        while (hi - lo > 1) { const int32_t mid = (lo + hi) >> 1; if (en_ip[mid] <= i) lo = mid; else hi = mid; }
        const int64_t b = en_ip[lo], e = en_ip[lo + 1];
        const int32_t x = tmp[i];
        int64_t r = 0;
        for (int64_t j = b; j < e; j++) r += tmp[j] < x;
        en[b + r] = x;
    }
}

__global__ void k_logical_edges(const int64_t *__restrict__ de_ip, const int32_t *__restrict__ de, const int64_t *__restrict__ kg_ip,
                                const int32_t *__restrict__ kg, const int64_t *__restrict__ en_ip, const int32_t *__restrict__ en,
                                int64_t n, int32_t cap, int32_t *__restrict__ le, int32_t *__restrict__ le_count) {
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < n; x += (int64_t)gridDim.x * blockDim.x) {
        int32_t *row = le + x * cap * 3;
        int32_t c = 0;
        const int64_t vb = de_ip[x], ve = de_ip[x + 1];
        for (int64_t ps = vb; ps < ve && c < cap; ps++) {
            const int32_t s = de[ps];
            for (int64_t pt = kg_ip[s]; pt < kg_ip[s + 1] && c < cap; pt++) {
                const int32_t t = kg[pt];
                bool mine = false;
                for (int64_t q = vb; q < ve; q++) mine = mine || de[q] == t;
                if (mine) continue;
                for (int64_t py = en_ip[t]; py < en_ip[t + 1] && c < cap; py++) {
                    const int32_t y = en[py];
                    if (y == (int32_t)x) continue;
                    row[3 * c] = s; row[3 * c + 1] = y; row[3 * c + 2] = t; c++;
                }
            }
        }
        le_count[x] = c;
        for (int32_t i = c; i < cap; i++) { row[3 * i] = -1; row[3 * i + 1] = -1; row[3 * i + 2] = -1; }
    }
}

static void kg_release(ap_index *ix) {
    void *p[] = {ix->kg_en_ip, ix->kg_en, ix->kg_le, ix->kg_le_count};
    for (void *x : p) if (x) (void)hipFree(x);
    ix->kg_en_ip = nullptr; ix->kg_en = nullptr; ix->kg_le = nullptr; ix->kg_le_count = nullptr;
    ix->kg_n_ent = 0;
}

extern "C" int ap_set_knowledge_graph(ap_index *ix, int32_t n_ent, const int64_t *doc_ent_indptr, const int32_t *doc_ent,
                                      const int64_t *kg_indptr, const int32_t *kg_idx, int32_t le_cap, void *stream) {
    AP_REQUIRE(ix && doc_ent_indptr && doc_ent && kg_indptr && kg_idx, "NULL argument");
    AP_REQUIRE(n_ent >= 1 && n_ent < (1 << 23), "n_ent = %d must be in [1, 2^23)", n_ent);
    AP_REQUIRE(le_cap >= 1 && le_cap <= 128, "le_cap = %d must be in [1, 128]", le_cap);
    hipStream_t st = (hipStream_t)stream;
    const int64_t n = ix->corpus.n;
    kg_release(ix);
    int64_t total = 0, kg_total = 0;
    AP_CHECK_HIP(hipMemcpyAsync(&total, doc_ent_indptr + n, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    AP_CHECK_HIP(hipMemcpyAsync(&kg_total, kg_indptr + n_ent, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    AP_CHECK_HIP(hipStreamSynchronize(st));
    AP_REQUIRE(total >= 0 && total < ((int64_t)1 << 31), "doc_ent_indptr[n] = %lld is out of range", (long long)total);
    AP_REQUIRE(kg_total >= 0 && kg_total < ((int64_t)1 << 31), "kg_indptr[n_ent] = %lld is out of range", (long long)kg_total);
    unsigned long long *cnt = nullptr;
    int32_t *tmp = nullptr, *bad = nullptr;
    int rc = ap_dev_alloc(&cnt, (size_t)n_ent);
    if (rc == AP_OK) rc = ap_dev_alloc(&tmp, (size_t)total);
    if (rc == AP_OK) rc = ap_dev_alloc(&bad, 1);
    if (rc == AP_OK) rc = ap_dev_alloc(&ix->kg_en_ip, (size_t)n_ent + 1);
    if (rc == AP_OK) rc = ap_dev_alloc(&ix->kg_en, (size_t)total);
    if (rc == AP_OK) rc = ap_dev_alloc(&ix->kg_le, (size_t)n * le_cap * 3);
    if (rc == AP_OK) rc = ap_dev_alloc(&ix->kg_le_count, (size_t)n);
    if (rc == AP_OK) rc = ap_fill_u32(cnt, (size_t)n_ent * 2, 0u, st);
    if (rc == AP_OK) rc = ap_fill_u32(bad, 1, 0u, st);
    hipError_t e = hipSuccess;
    int32_t h_bad = 0;
    if (rc == AP_OK) {
        const unsigned gd = (unsigned)std::min<int64_t>((n + 255) / 256, 4096), ge = (unsigned)std::min<int64_t>(((int64_t)n_ent + 255) / 256, 4096);
        hipLaunchKernelGGL(k_ent_count, dim3(gd), dim3(256), 0, st, doc_ent_indptr, doc_ent, n, n_ent, total, cnt, bad);
        hipLaunchKernelGGL(k_kg_check, dim3(ge), dim3(256), 0, st, kg_indptr, kg_idx, n_ent, kg_total, bad);
        e = hipGetLastError();
        if (e == hipSuccess) e = hipMemcpyAsync(&h_bad, bad, sizeof(h_bad), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e == hipSuccess && h_bad == 0) {
            hipLaunchKernelGGL(k_exclusive_scan, dim3(1), dim3(1024), 0, st, cnt, (int64_t)n_ent, ix->kg_en_ip);
            rc = ap_fill_u32(cnt, (size_t)n_ent * 2, 0u, st);
            if (rc == AP_OK) {
                hipLaunchKernelGGL(k_ent_fill, dim3(gd), dim3(256), 0, st, doc_ent_indptr, doc_ent, n, ix->kg_en_ip, cnt, tmp);
                const unsigned gt = (unsigned)std::min<int64_t>((total + 255) / 256 + 1, 8192);
                hipLaunchKernelGGL(k_ent_rank, dim3(gt), dim3(256), 0, st, ix->kg_en_ip, n_ent, tmp, ix->kg_en);
                hipLaunchKernelGGL(k_logical_edges, dim3(gd), dim3(256), 0, st, doc_ent_indptr, doc_ent, kg_indptr, kg_idx, ix->kg_en_ip,
                                   ix->kg_en, n, le_cap, ix->kg_le, ix->kg_le_count);
                e = hipGetLastError();
                if (e == hipSuccess) e = hipStreamSynchronize(st);
            }
        }
    }
    void *p[] = {cnt, tmp, bad};
    for (void *x : p) if (x) (void)hipFree(x);
    if (rc == AP_OK && e != hipSuccess) { ap_set_error("knowledge-graph set-up failed: %s", hipGetErrorString(e)); rc = AP_EHIP; }
    if (rc == AP_OK && h_bad != 0) {
        ap_set_error("%d rows or entity ids are malformed (row offsets not ascending from 0 to the total, ids out of range or not "
                     "ascending within their row, or an entity related to itself)", h_bad);
        rc = AP_EINVAL;
    }
    if (rc != AP_OK) { kg_release(ix); return rc; }
    ix->kg_n_ent = n_ent; ix->kg_le_cap = le_cap; ix->kg_total = total;
    ix->kg_de_ip = doc_ent_indptr; ix->kg_de = doc_ent; ix->kg_ip = kg_indptr; ix->kg_idx = kg_idx;
    return AP_OK;
}

extern "C" int ap_export_logical_edges(const ap_index *ix, int32_t *le, int32_t *le_count, int64_t *en_indptr, int32_t *en_idx, void *stream) {
    AP_REQUIRE(ix, "index is NULL");
    if (!ix->kg_le) { ap_set_error("no knowledge graph was set on this index"); return AP_ESTATE; }
    hipStream_t st = (hipStream_t)stream;
    const size_t n = (size_t)ix->corpus.n;
    if (le) AP_CHECK_HIP(hipMemcpyAsync(le, ix->kg_le, n * ix->kg_le_cap * 3 * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    if (le_count) AP_CHECK_HIP(hipMemcpyAsync(le_count, ix->kg_le_count, n * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    if (en_indptr) AP_CHECK_HIP(hipMemcpyAsync(en_indptr, ix->kg_en_ip, ((size_t)ix->kg_n_ent + 1) * sizeof(int64_t), hipMemcpyDeviceToDevice, st));
    if (en_idx) AP_CHECK_HIP(hipMemcpyAsync(en_idx, ix->kg_en, (size_t)ix->kg_total * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    return AP_OK;
}

// ------------------------------------------------------------------ search
struct ApKgArgs {
    ApVecs D, Q;
    const int32_t *graph, *entry;
    const float *w;
    int32_t w_stride, R, E, k, L, max_iters, cmax;
    int32_t q0;         // the launch covers queries q0 .. q0 + gridDim.x
    uint32_t *visited;  // one bitset per query of the launch
    size_t words;
    int32_t *out_ids;
    float *out_scores;
    int32_t *counts;
    const uint2 *rec;
    const uint4 *meta;
    const int64_t *de_ip; const int32_t *de; const int64_t *kg_ip; const int32_t *kg; const int64_t *en_ip; const int32_t *en;
    const int32_t *le, *le_count;
    int32_t le_cap;
    const int32_t *q_ent;
    int32_t ent_stride, max_hops, n_ent;
    float w_k;
    const uint32_t *deleted;   // one bit per document, NULL when nothing was ever deleted
};

// annotation of a pool entry: (entity + 1) << 8 | hop; 0 = no entity
__device__ __forceinline__ uint32_t ap_ann(int32_t ent, int32_t hop) { return ent < 0 ? 0u : ((uint32_t)(ent + 1) << 8) | (uint32_t)hop; }

// smallest entity of document o related to entity eu, -1 if none (V(o) is ascending)
__device__ __forceinline__ int32_t ap_related_entity(const ApKgArgs &g, int32_t o, int32_t eu) {
    for (int64_t p = g.de_ip[o]; p < g.de_ip[o + 1]; p++) {
        const int32_t t = g.de[p];
        for (int64_t r = g.kg_ip[eu]; r < g.kg_ip[eu + 1]; r++)
            if (g.kg[r] == t) return t;
    }
    return -1;
}

#define AP_KG_SPB 8
#define AP_KG_TXB 7
template <int DT, int NV>
__global__ __launch_bounds__(256) void k_search_kg(ApKgArgs g) {
    extern __shared__ __attribute__((aligned(16))) uint64_t smem64[];
    uint64_t *cur = smem64;                                  // the pool, best first
    uint64_t *newk = cur + g.L;                              // keys of this iteration's candidates
    uint64_t *qtab = newk + g.cmax + ((g.L + g.cmax) & 1);   // the query's look-up tables (16-byte aligned: read two slots at a time)
    uint4 *s_meta = reinterpret_cast<uint4 *>(qtab + (1 << AP_KG_SPB) + (1 << AP_KG_TXB));
    uint32_t *cura = reinterpret_cast<uint32_t *>(s_meta + g.cmax);   // annotations of the pool entries
    uint32_t *canda = cura + g.L;                                      // annotations of the candidates
    int32_t *cand = reinterpret_cast<int32_t *>(canda + g.cmax);
    __shared__ int32_t s_cnt, s_par, s_pann, s_seed[2], s_len, s_skip;
    const int64_t q = (int64_t)g.q0 + blockIdx.x;
    const int lane = threadIdx.x & 63, wave = ap_wave_id();
    ApLists a;
    {
        const int64_t sb = g.Q.sp_indptr[q], tb = g.Q.tx_indptr[q];
        a.sp_n = (int32_t)(g.Q.sp_indptr[q + 1] - sb); a.tx_n = (int32_t)(g.Q.tx_indptr[q + 1] - tb);
        a.sp_idx = g.Q.sp_idx + sb; a.sp_val = g.Q.sp_val + sb; a.tx_idx = g.Q.tx_idx + tb; a.tx_val = g.Q.tx_val + tb;
    }
    // the query's lists as bucket tables with a hash multiplier of their own, as in the plain search; lists that are
    // too long for them, or that no multiplier fits, are searched where they lie
    bool use_tab = a.sp_n <= (1 << AP_KG_SPB) / 4 && a.tx_n <= (1 << AP_KG_TXB) / 4;   // uniform
    uint32_t msp = 0, mtx = 0;
    if (use_tab && wave == 0) {
        const int32_t s0 = ap_bucket_build(a.sp_idx, a.sp_val, a.sp_n, qtab, AP_KG_SPB);
        const int32_t s1 = ap_bucket_build(a.tx_idx, a.tx_val, a.tx_n, qtab + (1 << AP_KG_SPB), AP_KG_TXB);
        if (lane == 0) { s_seed[0] = s0; s_seed[1] = s1; }
    }
    __syncthreads();
    if (use_tab) {
        const int32_t seed0 = ap_uniform_i32(s_seed[0]), seed1 = ap_uniform_i32(s_seed[1]);
        use_tab = seed0 >= 0 && seed1 >= 0;
        if (use_tab) { msp = ap_seed_mult(seed0); mtx = ap_seed_mult(seed1); }
    }
    float qa[NV * ApDense<DT>::EPC];
    ap_load_aside<DT, NV, AP_F32>(g.Q.dense, q, g.D.dim, qa);
    const float wd = g.w[q * g.w_stride + 0], ws = g.w[q * g.w_stride + 1], wf = g.w[q * g.w_stride + 2];
    float qnorm;
    {
        float p = 0.f;
#pragma unroll
        for (int i = 0; i < NV * ApDense<DT>::EPC; i++) p = fmaf(qa[i], qa[i], p);
        qnorm = sqrtf(ap_wave_sum(p));
    }
    uint32_t *vis = g.visited + (size_t)blockIdx.x * g.words;
    if (threadIdx.x == 0) { s_len = 0; s_skip = 0; }
    if (threadIdx.x == 0) {
        // the documents that mention the query's entities, in the order of the entities then ascending id, at most E
        int32_t c = 0;
        for (int32_t j = 0; j < g.ent_stride && c < g.E; j++) {
            const int32_t e = g.q_ent[q * g.ent_stride + j];
            if (e < 0 || e >= g.n_ent) continue;
            for (int64_t p = g.en_ip[e]; p < g.en_ip[e + 1] && c < g.E; p++) {
                const int32_t v = g.en[p];
                const uint32_t bit = 1u << (v & 31);
                if (vis[v >> 5] & bit) continue;
                vis[v >> 5] |= bit;
                cand[c] = v; canda[c] = ap_ann(e, 0); c++;
            }
        }
        s_cnt = c;
    }
    __syncthreads();
    if (s_cnt == 0) {   // no entity given, or nobody mentions them: the usual entry points (uniform branch)
        __syncthreads();
        for (int32_t i = threadIdx.x; i < g.E; i += blockDim.x) {
            const int32_t v = g.entry[i];
            if (v >= 0) {
                const uint32_t bit = 1u << (v & 31);
                const uint32_t old = atomicOr(&vis[v >> 5], bit);
                if (!(old & bit)) { const int32_t pos = atomicAdd(&s_cnt, 1); cand[pos] = v; canda[pos] = 0u; }
            }
        }
        __syncthreads();
    }
    int32_t len = 0, it = 0, nscored = 0;   // len is kept by wave 0, the only one that touches the pool
    int32_t fu = 0;                          // (wave 0) every pool entry before this position has been expanded
    int32_t nskipped = 0;
    for (;;) {
        const int32_t c = s_cnt;
        nscored += c;
        for (int32_t i = threadIdx.x; i < c; i += blockDim.x) s_meta[i] = g.meta[cand[i]];
        __syncthreads();
        // as in the plain search: when the pool is full and even the largest dense part the norms allow (plus the
        // candidate's reward) could not lift a candidate past the pool's last entry, its dense row is not read
        const bool pool_full = s_len == g.L;
        const float worst_score = pool_full ? ap_key_score(cur[g.L - 1]) : 0.f;
        for (int32_t i = wave; i < c; i += 4) {
            const uint4 m = s_meta[i];
            const uint2 *r = g.rec + ap_uniform_u32(m.x);
            const int32_t spn = __builtin_amdgcn_readfirstlane((int32_t)(m.y & 0xffffu));
            const int32_t txn = __builtin_amdgcn_readfirstlane((int32_t)(m.y >> 16));
            const int32_t v = __builtin_amdgcn_readfirstlane(cand[i]);
            int32_t si[2], ti[1];
            float sv[2], tv[1], ss, sf;
            ap_rec_load<2, 1>(r, spn, txn, si, sv, ti, tv);
            if (use_tab)
                ap_rec_reduce_bucket<2, 1, AP_KG_SPB, AP_KG_TXB>(r, (const AP_LDS uint64_t *)qtab, (const AP_LDS uint64_t *)(qtab + (1 << AP_KG_SPB)),
                                                                 msp, mtx, spn, txn, si, sv, ti, tv, ss, sf);
            else
                ap_rec_reduce_lists<2, 1>(r, a, spn, txn, si, sv, ti, tv, ss, sf);
            const uint32_t an = canda[i];
            const float reward = (an != 0u && (an & 0xffu) != 0u) ? g.w_k / (float)(an & 0xffu) : 0.f;   // the reward of a tie: w_k / hop
            {
                const float dmax = fabsf(wd) * qnorm * __uint_as_float(ap_uniform_u32(m.z)) * 1.0001f;
                const float part = fmaf(wf, sf, ws * ss);
                const float ub = part + dmax + fabsf(reward) + 1e-5f * (fabsf(ws * ss) + fabsf(wf * sf) + dmax + fabsf(reward));
                if (pool_full && ub < worst_score) {
                    if (lane == 0) newk[i] = (uint64_t)(uint32_t)(i + 1);   // ranks after every real key (score bits 0)
                    nskipped++;
                    continue;
                }
            }
            const float sd = ap_dense_dot<DT, NV>(g.D, qa, v);
            float s = ap_fuse(wd, ws, wf, sd, ss, sf);
            if (an != 0u && (an & 0xffu) != 0u) s = s + reward;
            if (lane == 0) newk[i] = ap_make_key(s, v, 1u);
        }
        __syncthreads();
        // one insertion at a time into the sorted pool (any order of arrival leaves the same best L)
        if (wave == 0) {
            for (int32_t j = 0; j < c; j++) {
                const uint64_t key = newk[j];
                if (len == g.L && key < cur[len - 1]) continue;
                int32_t pos = 0;
                for (int32_t base = 0; base < len; base += 64) {
                    const int32_t i = base + lane;
                    pos += __popcll(__ballot(i < len && cur[i] > key));
                }
                const int32_t last = len < g.L ? len : g.L - 1;   // entries [pos, last) move one place towards the end
                for (int32_t hi = last; hi > pos; hi -= 64) {
                    const int32_t lo = hi - 64 > pos ? hi - 64 : pos;
                    const int32_t i = lo + lane;
                    uint64_t hk = 0; uint32_t ha = 0;
                    if (i < hi) { hk = cur[i]; ha = cura[i]; }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    if (i < hi) { cur[i + 1] = hk; cura[i + 1] = ha; }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                }
                if (lane == 0) { cur[pos] = key; cura[pos] = canda[j]; }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                len = len < g.L ? len + 1 : g.L;
                fu = fu < pos ? fu : pos;
            }
            // the best entry not yet expanded becomes the parent
            int32_t found = -1;
            if (!(g.max_iters > 0 && it >= g.max_iters)) {
                for (int32_t base = fu & ~63; base < len && found < 0; base += 64) {
                    const int32_t i = base + lane;
                    const uint64_t mask = __ballot(i < len && (cur[i] & 1ull));
                    if (mask) found = base + (int32_t)__builtin_ctzll(mask);
                }
                fu = found >= 0 ? found + 1 : len;
            }
            if (lane == 0) {
                if (found >= 0) { s_par = ap_key_id(cur[found]); s_pann = (int32_t)cura[found]; cur[found] &= ~1ull; }
                else s_par = -1;
                s_cnt = 0;
                s_len = len;
            }
        }
        __syncthreads();
        const int32_t u = s_par;
        if (u < 0) break;
        const uint32_t pann = (uint32_t)s_pann;
        const int32_t eu = pann ? (int32_t)(pann >> 8) - 1 : -1, hu = (int32_t)(pann & 0xffu);
        const bool logical = eu >= 0 && hu < g.max_hops;
        const int32_t nle = logical ? g.le_count[u] : 0;
        for (int32_t i = threadIdx.x; i < g.R + nle; i += blockDim.x) {
            int32_t v = -1;
            if (i < g.R) v = g.graph[(int64_t)u * g.R + i];
            else {
                const int32_t *t3 = g.le + ((int64_t)u * g.le_cap + (i - g.R)) * 3;
                if (t3[0] == eu) v = t3[1];
            }
            if (v >= 0) {
                const uint32_t bit = 1u << (v & 31);
                const uint32_t old = atomicOr(&vis[v >> 5], bit);
                if (!(old & bit)) {
                    uint32_t an = 0u;
                    if (eu >= 0) { const int32_t t = ap_related_entity(g, v, eu); if (t >= 0) an = ap_ann(t, hu + 1); }
                    const int32_t pos = atomicAdd(&s_cnt, 1);
                    cand[pos] = v; canda[pos] = an;
                }
            }
        }
        __syncthreads();
        it++;
    }
    if (lane == 0) atomicAdd(&s_skip, nskipped);
    __syncthreads();
    if (threadIdx.x == 0) { g.counts[q * 3] = nscored; g.counts[q * 3 + 1] = it; g.counts[q * 3 + 2] = s_skip; }
    // the best k pool entries; mark-deleted documents were searched through like any other and are left out here
    if (wave == 0) {
        int32_t o = 0;
        for (int32_t base = 0; base < len && o < g.k; base += 64) {
            const int32_t i = base + lane;
            bool live = i < len;
            if (live && g.deleted) { const int32_t v = ap_key_id(cur[i]); live = !((g.deleted[v >> 5] >> (v & 31)) & 1u); }
            const uint64_t mask = __ballot(live);
            const int32_t at = o + __popcll(mask & ((1ull << lane) - 1ull));
            if (live && at < g.k) {
                g.out_ids[q * g.k + at] = ap_key_id(cur[i]);
                g.out_scores[q * g.k + at] = ap_key_score(cur[i]);
            }
            o += __popcll(mask);
        }
        o = o < g.k ? o : g.k;
        for (int32_t i = o + lane; i < g.k; i += 64) { g.out_ids[q * g.k + i] = -1; g.out_scores[q * g.k + i] = -INFINITY; }
    }
}

extern "C" int ap_search_batch_entities(ap_index *ix, const ap_queries *q, const float *per_query_w, const ap_search_params *p,
                                        const int32_t *q_ent, int32_t ent_stride, float w_k, int32_t max_hops, int32_t *out_ids,
                                        float *out_scores, void *stream) {
    AP_REQUIRE(ix && p, "NULL argument");
    AP_TRY(ap_validate_queries(q));
    if (!ix->has_graph) { ap_set_error("index has no graph: build or import one first"); return AP_ESTATE; }
    if (!ix->kg_le) { ap_set_error("no knowledge graph was set on this index (ap_set_knowledge_graph)"); return AP_ESTATE; }
    AP_REQUIRE(q->nq == 0 || (q_ent && out_ids && out_scores), "NULL argument");
    AP_REQUIRE(ent_stride >= 1 && ent_stride <= 16, "ent_stride = %d must be in [1, 16]", ent_stride);
    AP_REQUIRE(p->beam >= 1 && p->beam <= AP_MAX_BEAM, "beam = %d must be in [1, %d]", p->beam, AP_MAX_BEAM);
    AP_REQUIRE(p->k >= 1 && p->k <= p->beam, "k = %d must be in [1, beam]", p->k);
    AP_REQUIRE(p->search_width == 1, "the knowledge-graph search expands one parent per iteration (search_width = 1)");
    AP_REQUIRE(p->max_iters >= 0, "max_iters must be >= 0");
    AP_REQUIRE(max_hops >= 0 && max_hops <= 255, "max_hops = %d must be in [0, 255]", max_hops);
    AP_REQUIRE(w_k == w_k && w_k - w_k == 0.f, "w_k must be finite");
    if (q->nq == 0) return AP_OK;
    hipStream_t st = (hipStream_t)stream;
    const int32_t nq = q->nq;
    ApKgArgs g;
    g.D = ix->docs;
    g.Q = ApVecs{nq, ix->docs.dim, q->dense, q->sp_indptr, q->sp_idx, q->sp_val, q->tx_indptr, q->tx_idx, q->tx_cnt};
    g.graph = ix->graph; g.entry = ix->entry;
    g.w = per_query_w ? per_query_w : ix->w_dev;
    g.w_stride = per_query_w ? 3 : 0;
    g.R = ix->params.degree; g.E = ix->params.n_entry;
    g.k = p->k; g.L = p->beam; g.max_iters = p->max_iters;
    g.cmax = std::max(g.E, g.R + ix->kg_le_cap);
    g.words = ((size_t)ix->docs.n + 31) / 32;
    ApSearchWs ws;
    AP_TRY(ap_search_reserve(ix, nq, st, &ws));
    g.visited = ws.visited; g.out_ids = out_ids; g.out_scores = out_scores; g.counts = ws.counts;
    g.rec = ix->rec; g.meta = ix->meta;
    g.de_ip = ix->kg_de_ip; g.de = ix->kg_de; g.kg_ip = ix->kg_ip; g.kg = ix->kg_idx; g.en_ip = ix->kg_en_ip; g.en = ix->kg_en;
    g.le = ix->kg_le; g.le_count = ix->kg_le_count; g.le_cap = ix->kg_le_cap;
    g.q_ent = q_ent; g.ent_stride = ent_stride; g.max_hops = max_hops; g.w_k = w_k;
    g.n_ent = ix->kg_n_ent; g.deleted = ix->deleted;
    const size_t smem = (size_t)(g.L + g.cmax) * 8 + ((1 << AP_KG_SPB) + (1 << AP_KG_TXB)) * 8 + 8 + (size_t)g.cmax * 16 +
                        (size_t)(g.L + 2 * g.cmax) * 4;
    AP_REQUIRE(smem <= 160 * 1024, "beam needs %zu bytes of LDS (limit 160 KiB)", smem);
    for (int32_t q0 = 0; q0 < nq; q0 += ws.slab) {   // slabs of queries share the workspace
        const int32_t qn = std::min(ws.slab, nq - q0);
        g.q0 = q0;
        AP_TRY(ap_fill_u32(ws.visited, g.words * (size_t)qn, 0u, st));
        if (q0 == 0) AP_CHECK_HIP(hipEventRecord(ws.ev0, st));
        hipError_t le = hipSuccess;
        AP_DISPATCH_DENSE(ix->dtype, ix->docs.dim, {
            if (smem > 48 * 1024)
                le = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_search_kg<DT, NV>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (le == hipSuccess) hipLaunchKernelGGL((k_search_kg<DT, NV>), dim3((unsigned)qn), dim3(256), smem, st, g);
        });
        AP_CHECK_HIP(le);
        AP_CHECK_HIP(hipGetLastError());
    }
    AP_CHECK_HIP(hipEventRecord(ix->ev_search[1], st));
    return AP_OK;
}
