// Insertion of new documents into a built index (Section 4.1, "Updates of
// the hybrid index"): the K nearest neighbours of each new document are the
// best of two candidate sets -- what a search of the existing index on its
// semantic edges returns for the new document, and the K-lists the new
// documents get among themselves -- and pruning, keyword recycling and
// edge-list assembly then run as in the construction.
//
// The caller hands over the enlarged corpus (the first n0 documents are the
// indexed ones, unchanged; the rest are new) and gets a new index; the old one
// stays valid.  S0 is recomputed over the enlarged corpus, so all lexical
// weights follow the statistics of the new corpus, exactly as a rebuild would.
#include <string.h>
#include <algorithm>
#include <new>
#include "ap_common.hpp"

extern "C" int ap_stage_refine(const ap_index *ix, int32_t K, int32_t S, int32_t P, const int32_t *knn_ids,
                               const int32_t *sp_ids, const float *sp_sc, const int32_t *node_ids, int64_t nn,
                               int32_t *out_ids, float *out_sc, int32_t *out_sp_ids, float *out_sp_sc, void *stream);
extern "C" int ap_stage_entry_points(const ap_index *index, int32_t E, int32_t *out_entry, void *stream);
extern "C" void ap_free_index(ap_index *ix);

// ids >= 0 move up by `shift` (lists computed on the new documents alone use local ids)
__global__ void k_shift_ids(int32_t *__restrict__ ids, size_t n, int32_t shift) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        if (ids[i] >= 0) ids[i] += shift;
}

__global__ void k_iota(int32_t *__restrict__ out, int64_t n, int32_t first) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        out[i] = first + (int32_t)i;
}

__global__ void k_bf16_to_f32(const uint16_t *__restrict__ in, float *__restrict__ out, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        out[i] = __uint_as_float((uint32_t)in[i] << 16);
}

// Best K of two ranked lists over disjoint ids, by (score descending, id ascending).  One block per row; thread t
// holds entry t of the first list or entry t-K of the second and counts the keys that rank before its own.
__global__ __launch_bounds__(512) void k_merge_ranked(int32_t K, const int32_t *__restrict__ a_ids, const float *__restrict__ a_sc,
                                                      const int32_t *__restrict__ b_ids, const float *__restrict__ b_sc,
                                                      int64_t x0, int32_t *__restrict__ out_ids, float *__restrict__ out_sc) {
    __shared__ uint64_t keys[512];
    const int64_t x = x0 + blockIdx.x;
    const int32_t t = threadIdx.x;
    uint64_t key = 0;
    if (t < 2 * K) {
        const int32_t id = t < K ? a_ids[x * K + t] : b_ids[x * K + t - K];
        const float s = t < K ? a_sc[x * K + t] : b_sc[x * K + t - K];
        if (id >= 0) key = ap_make_key(s, id, 1u);
    }
    keys[t] = key;
    __syncthreads();
    int32_t total = 0, r = 0;
    for (int32_t j = 0; j < 2 * K; j++) { total += keys[j] != 0ull; r += keys[j] > key; }
    if (key != 0ull && r < K) { out_ids[x * K + r] = ap_key_id(key); out_sc[x * K + r] = ap_key_score(key); }
    if (t < K && t >= total) { out_ids[x * K + t] = -1; out_sc[x * K + t] = -INFINITY; }
}

namespace {
struct InsertBufs {
    void *all[32];
    int n = 0;
    template <typename T> int get(T **p, size_t count) {
        const int rc = ap_dev_alloc(p, count);
        if (rc == AP_OK) all[n++] = *p;
        return rc;
    }
    void keep(void *p) { for (int i = 0; i < n; i++) if (all[i] == p) all[i] = nullptr; }
    ~InsertBufs() { for (int i = 0; i < n; i++) if (all[i]) (void)hipFree(all[i]); }
};

unsigned grid_for(size_t n) { return (unsigned)std::min<size_t>((n + 255) / 256, 8192); }

#define AP_COPY(dst, src, count, T) AP_CHECK_HIP(hipMemcpyAsync((dst), (src), (size_t)(count) * sizeof(T), hipMemcpyDeviceToDevice, st))
}  // namespace

static int insert_impl(const ap_index *old, ap_index *nx, int32_t beam, const ap_insert_trace *tr, hipStream_t st) {
    const ap_build_params &p = nx->params;
    const int64_t n0 = old->corpus.n, n1 = nx->corpus.n, m = n1 - n0;
    const int32_t K = p.knn_k, R = p.degree, P = p.sp_len, KR = R / 2;
    const size_t esize = nx->dtype == AP_F32 ? 4 : 2;
    ApStageEvents marks;
    AP_CHECK_HIP(marks.create());
    hipEvent_t *ev = marks.ev;
    auto mark = [&](int i) { return hipEventRecord(ev[i], st); };
    InsertBufs B;
    AP_CHECK_HIP(mark(0));
    // step 0: S0 over the enlarged corpus
    AP_TRY(ap_ingest_impl(nx, st));
    AP_TRY(ap_alloc_graph(nx));
    AP_CHECK_HIP(mark(1));

    // step 1: candidate set one -- each new document is searched in the old graph (edge-less rows stand in for the
    // new documents, which nothing points at), from the old entry points, under the construction weights
    AP_COPY(nx->graph, old->graph, (size_t)n0 * R, int32_t);
    AP_TRY(ap_fill_u32(nx->graph + (size_t)n0 * R, (size_t)m * R, 0xffffffffu, st));
    AP_COPY(nx->entry, old->entry, p.n_entry, int32_t);
    nx->has_graph = true;
    int32_t *c1_ids = nullptr, *c2_ids = nullptr, *spi2[2] = {nullptr, nullptr}, *new_ids = nullptr;
    float *c1_sc = nullptr, *c2_sc = nullptr, *sps2[2] = {nullptr, nullptr}, *w_dev = nullptr, *qdense = nullptr;
    AP_TRY(B.get(&c1_ids, (size_t)m * K));
    AP_TRY(B.get(&c1_sc, (size_t)m * K));
    AP_TRY(B.get(&w_dev, 4));
    AP_CHECK_HIP(hipMemcpyAsync(w_dev, p.build_w, 3 * sizeof(float), hipMemcpyHostToDevice, st));
    const void *qd = static_cast<const char *>(nx->docs.dense) + (size_t)n0 * nx->docs.dim * esize;
    if (nx->dtype != AP_F32) {   // the search reads its queries' dense rows as f32
        AP_TRY(B.get(&qdense, (size_t)m * nx->docs.dim));
        hipLaunchKernelGGL(k_bf16_to_f32, dim3(grid_for((size_t)m * nx->docs.dim)), dim3(256), 0, st, static_cast<const uint16_t *>(qd),
                           qdense, (size_t)m * nx->docs.dim);
        AP_CHECK_HIP(hipGetLastError());
        qd = qdense;
    }
    {
        const int32_t L = std::min<int32_t>(AP_MAX_BEAM, std::max<int32_t>(beam > 0 ? beam : 2 * K, K));
        const ApVecs Q{m, nx->docs.dim, qd, nx->docs.sp_indptr + n0, nx->docs.sp_idx, nx->docs.sp_val,
                       nx->docs.tx_indptr + n0, nx->docs.tx_idx, nx->docs.tx_val};
        AP_TRY(ap_search_core(nx, Q, w_dev, 0, K, L, 0, 1, true, c1_ids, c1_sc, st));   // runs in slabs of queries by itself
    }
    nx->has_graph = false;

    // step 2: candidate set two -- seed lists and refinement rounds among the new documents alone, on a view of the
    // index that starts at document n0 (list offsets are absolute, so only the row-indexed arrays shift)
    AP_TRY(B.get(&c2_ids, (size_t)m * K));
    AP_TRY(B.get(&c2_sc, (size_t)m * K));
    for (int i = 0; i < 2; i++) {
        AP_TRY(B.get(&spi2[i], (size_t)3 * m * P));
        AP_TRY(B.get(&sps2[i], (size_t)3 * m * P));
    }
    AP_TRY(ap_fill_u32(spi2[0], (size_t)3 * m * P, 0xffffffffu, st));
    AP_TRY(ap_fill_u32(sps2[0], (size_t)3 * m * P, 0xff800000u, st));
    int cur = 0;
    int32_t *r_ids[2] = {c2_ids, nullptr};
    float *r_sc[2] = {c2_sc, nullptr};
    if (m >= 2) {
        ap_index vx = *nx;
        vx.corpus.n = m;
        vx.docs.n = m;
        vx.docs.dense = static_cast<const char *>(nx->docs.dense) + (size_t)n0 * nx->docs.dim * esize;
        vx.docs.sp_indptr += n0; vx.docs.tx_indptr += n0;
        vx.self_sim += n0; vx.dense_norm += n0; vx.meta += n0;
        AP_TRY(B.get(&r_ids[1], (size_t)m * K));
        AP_TRY(B.get(&r_sc[1], (size_t)m * K));
        AP_TRY(ap_seed_knn_impl(&vx, nullptr, m, K, r_ids[0], r_sc[0], st));
        for (int32_t t = 0; t < p.nd_rounds; t++) {
            AP_TRY(ap_stage_refine(&vx, K, p.nd_sample, P, r_ids[cur], spi2[cur], sps2[cur], nullptr, m, r_ids[1 - cur], r_sc[1 - cur],
                                   spi2[1 - cur], sps2[1 - cur], st));
            cur = 1 - cur;
        }
        if (p.nd_rounds == 0) AP_TRY(ap_rescore_lists(&vx, m, K, r_ids[cur], r_sc[cur], st));
        hipLaunchKernelGGL(k_shift_ids, dim3(grid_for((size_t)m * K)), dim3(256), 0, st, r_ids[cur], (size_t)m * K, (int32_t)n0);
        hipLaunchKernelGGL(k_shift_ids, dim3(grid_for((size_t)3 * m * P)), dim3(256), 0, st, spi2[cur], (size_t)3 * m * P, (int32_t)n0);
        AP_CHECK_HIP(hipGetLastError());
    } else {
        AP_TRY(ap_fill_u32(r_ids[0], (size_t)m * K, 0xffffffffu, st));
        AP_TRY(ap_fill_u32(r_sc[0], (size_t)m * K, 0xff800000u, st));
    }
    AP_CHECK_HIP(mark(2));

    // step 3: the K-list of a new document = the best K of both sets; scored once more without 2-hop exploration so
    // that its per-path lists take in the list's members
    int32_t *knn = nullptr, *spi = nullptr, *se = nullptr, *sorted = nullptr, *f_ids = nullptr, *f_spi = nullptr;
    float *knn_sc = nullptr, *sps = nullptr, *f_sc = nullptr, *f_sps = nullptr;
    AP_TRY(B.get(&knn, (size_t)n1 * K));
    AP_TRY(B.get(&knn_sc, (size_t)n1 * K));
    AP_TRY(B.get(&spi, (size_t)3 * n1 * P));
    AP_TRY(B.get(&sps, (size_t)3 * n1 * P));
    AP_TRY(B.get(&se, (size_t)n1 * R));
    AP_TRY(B.get(&sorted, (size_t)n1 * K));
    AP_TRY(B.get(&f_ids, (size_t)m * K));
    AP_TRY(B.get(&f_sc, (size_t)m * K));
    AP_TRY(B.get(&f_spi, (size_t)3 * m * P));
    AP_TRY(B.get(&f_sps, (size_t)3 * m * P));
    AP_TRY(B.get(&new_ids, (size_t)m));
    AP_TRY(ap_fill_u32(knn, (size_t)n0 * K, 0xffffffffu, st));          // rows of old documents are never read
    AP_TRY(ap_fill_u32(knn_sc, (size_t)n0 * K, 0xff800000u, st));
    const int64_t slice = AP_MAX_LAUNCH_THREADS / 512;
    for (int64_t x0 = 0; x0 < m; x0 += slice) {
        hipLaunchKernelGGL(k_merge_ranked, dim3((unsigned)std::min<int64_t>(slice, m - x0)), dim3(512), 0, st, K,
                           c1_ids, c1_sc, r_ids[cur], r_sc[cur], x0, knn + (size_t)n0 * K, knn_sc + (size_t)n0 * K);
        AP_CHECK_HIP(hipGetLastError());
    }
    hipLaunchKernelGGL(k_iota, dim3(grid_for((size_t)m)), dim3(256), 0, st, new_ids, m, (int32_t)n0);
    AP_CHECK_HIP(hipGetLastError());
    if (tr) {
        if (tr->cand1_ids) AP_COPY(tr->cand1_ids, c1_ids, (size_t)m * K, int32_t);
        if (tr->cand1_sc) AP_COPY(tr->cand1_sc, c1_sc, (size_t)m * K, float);
        if (tr->cand2_ids) AP_COPY(tr->cand2_ids, r_ids[cur], (size_t)m * K, int32_t);
        if (tr->cand2_sc) AP_COPY(tr->cand2_sc, r_sc[cur], (size_t)m * K, float);
        if (tr->cand2_sp_ids) AP_COPY(tr->cand2_sp_ids, spi2[cur], (size_t)3 * m * P, int32_t);
        if (tr->cand2_sp_sc) AP_COPY(tr->cand2_sp_sc, sps2[cur], (size_t)3 * m * P, float);
        if (tr->merged_ids) AP_COPY(tr->merged_ids, knn + (size_t)n0 * K, (size_t)m * K, int32_t);
        if (tr->merged_sc) AP_COPY(tr->merged_sc, knn_sc + (size_t)n0 * K, (size_t)m * K, float);
    }
    for (int path = 0; path < 3; path++) {   // per-path lists: old rows as they were, new rows from step 2
        AP_COPY(spi + ((size_t)path * n1) * P, old->st_spi + ((size_t)path * n0) * P, (size_t)n0 * P, int32_t);
        AP_COPY(sps + ((size_t)path * n1) * P, old->st_sps + ((size_t)path * n0) * P, (size_t)n0 * P, float);
        AP_COPY(spi + ((size_t)path * n1 + n0) * P, spi2[cur] + ((size_t)path * m) * P, (size_t)m * P, int32_t);
        AP_COPY(sps + ((size_t)path * n1 + n0) * P, sps2[cur] + ((size_t)path * m) * P, (size_t)m * P, float);
    }
    AP_TRY(ap_stage_refine(nx, K, 0, P, knn, spi, sps, new_ids, m, f_ids, f_sc, f_spi, f_sps, st));
    AP_COPY(knn + (size_t)n0 * K, f_ids, (size_t)m * K, int32_t);
    AP_COPY(knn_sc + (size_t)n0 * K, f_sc, (size_t)m * K, float);
    for (int path = 0; path < 3; path++) {
        AP_COPY(spi + ((size_t)path * n1 + n0) * P, f_spi + ((size_t)path * m) * P, (size_t)m * P, int32_t);
        AP_COPY(sps + ((size_t)path * n1 + n0) * P, f_sps + ((size_t)path * m) * P, (size_t)m * P, float);
    }
    if (tr) {
        if (tr->knn_ids) AP_COPY(tr->knn_ids, f_ids, (size_t)m * K, int32_t);
        if (tr->knn_sc) AP_COPY(tr->knn_sc, f_sc, (size_t)m * K, float);
    }
    AP_CHECK_HIP(mark(3));

    // step 4: S4/S5 for the new documents; the old documents keep their pruned lists and keyword edges
    AP_COPY(se, old->st_se, (size_t)n0 * R, int32_t);
    AP_COPY(sorted, old->st_sorted, (size_t)n0 * K, int32_t);
    AP_COPY(nx->kw, old->kw, (size_t)n0 * KR, int32_t);
    AP_COPY(nx->kw_count, old->kw_count, (size_t)n0, int32_t);
    AP_TRY(ap_prune_impl(nx, K, R, knn, knn_sc, new_ids, m, nullptr, nullptr, sorted + (size_t)n0 * K, se + (size_t)n0 * R,
                         nx->kw + (size_t)n0 * KR, nx->kw_count + n0, nullptr, st));
    AP_CHECK_HIP(mark(4));
    // S6 over all documents: old documents gain reverse neighbours among the new ones
    AP_TRY(ap_assemble_impl(nx, R, K, P, se, sorted, spi, nx->graph, st));
    AP_TRY(ap_stage_entry_points(nx, p.n_entry, nx->entry, st));
    AP_CHECK_HIP(mark(5));
    if (old->deleted) {   // marks of deletion carry over (bits past n0 in the old last word were never set)
        const size_t w0 = ((size_t)n0 + 31) / 32, w1 = ((size_t)n1 + 31) / 32;
        AP_TRY(ap_dev_alloc(&nx->deleted, w1));
        AP_TRY(ap_dev_alloc(&nx->deleted_bad, 1));
        AP_TRY(ap_fill_u32(nx->deleted, w1, 0u, st));
        AP_COPY(nx->deleted, old->deleted, w0, uint32_t);
    }
    AP_CHECK_HIP(hipStreamSynchronize(st));
    float total = 0.f;
    for (int i = 0; i < 5; i++) {
        float ms = 0.f;
        AP_CHECK_HIP(hipEventElapsedTime(&ms, ev[i], ev[i + 1]));
        nx->timings[i] = ms * 1e-3f;
        total += ms * 1e-3f;
    }
    nx->timings[5] = total;
    nx->has_graph = true;
    nx->st_se = se; nx->st_sorted = sorted; nx->st_spi = spi; nx->st_sps = sps;
    B.keep(se); B.keep(sorted); B.keep(spi); B.keep(sps);
    return AP_OK;
}

extern "C" int ap_insert_documents(const ap_index *old, const ap_corpus *enlarged, int32_t beam, const ap_insert_trace *trace,
                                   void *stream, ap_index **out) {
    AP_REQUIRE(out != nullptr, "out is NULL");
    *out = nullptr;
    AP_REQUIRE(old && enlarged, "NULL argument");
    if (!old->has_graph || !old->st_se) {
        ap_set_error("insertion needs an index built here (ap_build_index or ap_insert_documents): an imported graph carries no construction state");
        return AP_ESTATE;
    }
    AP_TRY(ap_validate_corpus(enlarged));
    AP_REQUIRE(enlarged->n > old->corpus.n, "the enlarged corpus holds %lld documents, the index %lld: nothing to insert",
               (long long)enlarged->n, (long long)old->corpus.n);
    AP_REQUIRE(enlarged->dim == old->corpus.dim && enlarged->dense_dtype == old->corpus.dense_dtype &&
               enlarged->sp_vocab == old->corpus.sp_vocab && enlarged->tx_vocab == old->corpus.tx_vocab,
               "the enlarged corpus must keep dimension, dense type and vocabularies");
    AP_REQUIRE(beam >= 0 && beam <= AP_MAX_BEAM, "beam = %d must be in [0, %d] (0 = twice the list length)", beam, AP_MAX_BEAM);
    ap_index *nx = new (std::nothrow) ap_index();
    if (!nx) { ap_set_error("out of host memory"); return AP_ENOMEM; }
    nx->corpus = *enlarged;
    nx->params = old->params;
    nx->dtype = enlarged->dense_dtype;
    memcpy(nx->w_default, old->w_default, sizeof(nx->w_default));
    const int rc = insert_impl(old, nx, beam, trace, (hipStream_t)stream);
    (void)hipStreamSynchronize((hipStream_t)stream);
    if (rc != AP_OK) { nx->has_graph = false; ap_free_index(nx); return rc; }
    *out = nx;
    return AP_OK;
}

extern "C" int ap_export_build_state(const ap_index *ix, int32_t *se, int32_t *sorted_ids, int32_t *sp_ids, float *sp_sc, void *stream) {
    AP_REQUIRE(ix, "index is NULL");
    if (!ix->st_se) { ap_set_error("this index carries no construction state"); return AP_ESTATE; }
    hipStream_t st = (hipStream_t)stream;
    const size_t n = (size_t)ix->corpus.n, R = (size_t)ix->params.degree, K = (size_t)ix->params.knn_k, P = (size_t)ix->params.sp_len;
    if (se) AP_COPY(se, ix->st_se, n * R, int32_t);
    if (sorted_ids) AP_COPY(sorted_ids, ix->st_sorted, n * K, int32_t);
    if (sp_ids) AP_COPY(sp_ids, ix->st_spi, 3 * n * P, int32_t);
    if (sp_sc) AP_COPY(sp_sc, ix->st_sps, 3 * n * P, float);
    return AP_OK;
}
