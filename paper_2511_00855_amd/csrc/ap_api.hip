// Index lifetime, argument validation, S0 (lexical encoding) and the graph
// import/export calls of the C ABI.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <new>
#include <algorithm>
#include "ap_common.hpp"

static thread_local char g_err[512] = "";

void ap_set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

extern "C" const char *ap_last_error(void) { return g_err; }

ApDebug g_ap_debug;

extern "C" int ap_debug_set(const char *name, int64_t value) {
    AP_REQUIRE(name != nullptr, "name is NULL");
    AP_REQUIRE(value >= 0, "value must be >= 0 (0 = the library's own choice)");
    struct { const char *name; int64_t *field; } table[] = {
        {"seed_sample_cols", &g_ap_debug.seed_sample_cols},       {"seed_buffer_cap", &g_ap_debug.seed_buffer_cap},
        {"seed_tau_ulps", &g_ap_debug.seed_tau_ulps},             {"max_launch_threads", &g_ap_debug.max_launch_threads},
        {"search_workspace_bytes", &g_ap_debug.search_workspace_bytes}, {"search_visited_global", &g_ap_debug.search_visited_global},
        {"search_query_lists", &g_ap_debug.search_query_lists},         {"seed_one_sided", &g_ap_debug.seed_one_sided},
    };
    for (auto &t : table)
        if (strcmp(name, t.name) == 0) { *t.field = value; return AP_OK; }
    ap_set_error("unknown debug setting '%s'", name);
    return AP_EINVAL;
}

// Long steps of a construction report where they are on stderr when ALLANPOE_PROGRESS is set in the environment
// (a corpus of millions of documents spends minutes in the seed stage).
void ap_progress(const char *fmt, ...) {
    static const bool on = getenv("ALLANPOE_PROGRESS") != nullptr;
    if (!on) return;
    va_list ap;
    va_start(ap, fmt);
    fputs("[allanpoe] ", stderr);
    vfprintf(stderr, fmt, ap);
    fputc('\n', stderr);
    fflush(stderr);
    va_end(ap);
}

int ap_validate_corpus(const ap_corpus *c) {
    AP_REQUIRE(c != nullptr, "corpus is NULL");
    AP_REQUIRE(c->n >= 1 && c->n < (1ll << 30), "corpus.n = %lld must be in [1, 2^30)", (long long)c->n);
    AP_REQUIRE(c->dense_dtype == AP_F32 || c->dense_dtype == AP_BF16, "corpus.dense_dtype = %d is not AP_F32/AP_BF16",
               c->dense_dtype);
    const int epc = c->dense_dtype == AP_BF16 ? 8 : 4;
    AP_REQUIRE(c->dim >= epc && c->dim % epc == 0 && c->dim <= 256 * epc,
               "corpus.dim = %d must be a multiple of %d and at most %d", c->dim, epc, 256 * epc);
    AP_REQUIRE(c->dense && c->sp_indptr && c->sp_idx && c->sp_val && c->tx_indptr && c->tx_idx && c->tx_tf,
               "corpus has a NULL array");
    AP_REQUIRE(((uintptr_t)c->dense & 15) == 0, "corpus.dense must be 16-byte aligned");
    AP_REQUIRE(c->sp_vocab >= 1 && c->tx_vocab >= 1, "vocabulary sizes must be positive");
    return AP_OK;
}

int ap_validate_params(const ap_build_params *p) {
    AP_REQUIRE(p != nullptr, "params is NULL");
    AP_REQUIRE(p->degree >= 4 && p->degree % 4 == 0 && p->degree <= 128, "degree = %d must be a multiple of 4 in [4, 128]",
               p->degree);
    AP_REQUIRE(p->knn_k >= p->degree && p->knn_k <= 256, "knn_k = %d must be in [degree, 256]", p->knn_k);
    AP_REQUIRE(p->nd_rounds >= 0, "nd_rounds = %d must be >= 0", p->nd_rounds);
    AP_REQUIRE(p->prune_mode >= AP_PRUNE_JOINT && p->prune_mode <= AP_PRUNE_IP_ONLY, "prune_mode = %d must be 0, 1 or 2", p->prune_mode);
    AP_REQUIRE(p->nd_sample >= 1 && p->nd_sample <= 32, "nd_sample = %d must be in [1, 32]", p->nd_sample);
    AP_REQUIRE(p->n_entry >= 1 && p->n_entry <= 256, "n_entry = %d must be in [1, 256]", p->n_entry);
    AP_REQUIRE(p->sp_len >= 0 && p->sp_len <= 32, "sp_len = %d must be in [0, 32]", p->sp_len);
    AP_REQUIRE(p->bm25_k1 >= 0.f && p->bm25_b >= 0.f && p->bm25_b <= 1.f, "bm25_k1 >= 0 and 0 <= bm25_b <= 1 required");
    return AP_OK;
}

// ------------------------------------------------------------------ S0 kernels
// Lexical encoding (Section 3.2): the text of a document becomes a lexical
// sparse vector of BM25 term importances.  The paper prints no formula; this
// is the Robertson form with the non-negative IDF, computed in f64 once at
// ingest and stored as f32:
//   w(d,t) = IDF(t) * tf (k1+1) / (tf + k1 (1 - b + b |d|/avgdl)),
//   IDF(t) = ln(1 + (N - df + 0.5)/(df + 0.5)).
__global__ void k_df_and_tokens(const int32_t *__restrict__ idx, const float *__restrict__ tf, int64_t nnz,
                                int32_t *__restrict__ df, unsigned long long *__restrict__ total) {
    unsigned long long local = 0;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * blockDim.x) {
        atomicAdd(&df[idx[e]], 1);
        local += (unsigned long long)llrintf(tf[e]);
    }
    for (int o = 32; o > 0; o >>= 1) local += __shfl_xor(local, o, 64);
    if ((threadIdx.x & 63) == 0 && local) atomicAdd(total, local);
}

__global__ void k_bm25_weights(const int64_t *__restrict__ indptr, const int32_t *__restrict__ idx,
                               const float *__restrict__ tf, int64_t n, const int32_t *__restrict__ df,
                               const unsigned long long *__restrict__ total, double k1, double b,
                               float *__restrict__ w, float *__restrict__ stats) {
    const double avgdl = (double)(*total) / (double)n;
    if (blockIdx.x == 0 && threadIdx.x == 0) stats[0] = (float)avgdl;
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t beg = indptr[i], end = indptr[i + 1];
        double len = 0.0;
        for (int64_t e = beg; e < end; e++) len += (double)tf[e];
        const double norm = k1 * (1.0 - b + b * len / avgdl);
        for (int64_t e = beg; e < end; e++) {
            const double d = (double)df[idx[e]];
            const double idf = log(1.0 + ((double)n - d + 0.5) / (d + 0.5));
            const double f = (double)tf[e];
            w[e] = (float)(idf * f * (k1 + 1.0) / (f + norm));
        }
    }
}

// Fused self-similarity M_w(v,v) = w_d |v_d|^2 + w_s |v_s|^2 + w_f |v_f|^2, one wave per document.
template <int DT>
__global__ void k_self_sim(ApVecs D, float wd, float ws, float wf, float *__restrict__ out, float *__restrict__ dnorm) {
    constexpr int EPC = ApDense<DT>::EPC;
    const int lane = threadIdx.x & 63;
    const int64_t wave = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t v = wave; v < D.n; v += nwaves) {
        float pd = 0.f, ps = 0.f, pf = 0.f;
        for (int col = lane * EPC; col < D.dim; col += 64 * EPC) {
            float d[EPC];
            ApDense<DT>::load(D.dense, v, D.dim, col, d);
#pragma unroll
            for (int e = 0; e < EPC; e++) pd = fmaf(d[e], d[e], pd);
        }
        for (int64_t e = D.sp_indptr[v] + lane; e < D.sp_indptr[v + 1]; e += 64) ps = fmaf(D.sp_val[e], D.sp_val[e], ps);
        for (int64_t e = D.tx_indptr[v] + lane; e < D.tx_indptr[v + 1]; e += 64) pf = fmaf(D.tx_val[e], D.tx_val[e], pf);
        pd = ap_wave_sum(pd); ps = ap_wave_sum(ps); pf = ap_wave_sum(pf);
        if (lane == 0) { out[v] = ap_fuse(wd, ws, wf, pd, ps, pf); dnorm[v] = sqrtf(pd); }
    }
}

// Search-side records: per document, its sparse entries then its lexical entries (term, weight bits),
// plus a 16-byte descriptor.  One wave per document.
__global__ void k_pack_records(ApVecs D, const float *__restrict__ dnorm, uint2 *__restrict__ rec, uint4 *__restrict__ meta) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t v = wave; v < D.n; v += nwaves) {
        const int64_t sb = D.sp_indptr[v], tb = D.tx_indptr[v];
        const int32_t sn = (int32_t)(D.sp_indptr[v + 1] - sb), tn = (int32_t)(D.tx_indptr[v + 1] - tb);
        const int64_t off = sb + tb;
        for (int32_t e = lane; e < sn; e += 64) rec[off + e] = make_uint2((uint32_t)D.sp_idx[sb + e], __float_as_uint(D.sp_val[sb + e]));
        for (int32_t e = lane; e < tn; e += 64) rec[off + sn + e] = make_uint2((uint32_t)D.tx_idx[tb + e], __float_as_uint(D.tx_val[tb + e]));
        if (lane == 0) meta[v] = make_uint4((uint32_t)off, (uint32_t)sn | ((uint32_t)tn << 16), __float_as_uint(dnorm[v]), 0u);
    }
}

// largest list length of either part (documents whose lists do not fit the 16-bit counts of a descriptor are refused)
__global__ void k_max_list_len(const int64_t *__restrict__ sp_indptr, const int64_t *__restrict__ tx_indptr, int64_t n, int32_t *out) {
    int32_t m = 0;
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t a = sp_indptr[i + 1] - sp_indptr[i], b = tx_indptr[i + 1] - tx_indptr[i];
        const int64_t x = a > b ? a : b;
        m = x > m ? (x > 0x7fffffff ? 0x7fffffff : (int32_t)x) : m;
    }
    atomicMax(out, m);
}

// One CSR part of the corpus as the kernels rely on it: offsets ascending from 0 to the total, term ids strictly
// ascending within a row and inside the vocabulary, values finite (and, for term counts, not negative).
__global__ void k_check_csr(const int64_t *__restrict__ ip, const int32_t *__restrict__ idx, const float *__restrict__ val, int64_t n,
                            int64_t total, int32_t vocab, int counts, int32_t *__restrict__ bad) {
    for (int64_t x = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; x < n; x += (int64_t)gridDim.x * blockDim.x) {
        if (!ap_row_ok(ip, x, total)) { atomicAdd(bad, 1); continue; }
        int32_t wrong = 0;
        const int64_t b = ip[x], e = ip[x + 1];
        for (int64_t p = b; p < e; p++) {
            const int32_t t = idx[p];
            const float v = val[p];
            wrong += (t < 0 || t >= vocab || (p > b && idx[p - 1] >= t) || !(v - v == 0.f) || (counts && v < 0.f)) ? 1 : 0;
        }
        if (wrong) atomicAdd(bad, wrong);
    }
}

__global__ void k_fill_u32(uint32_t *p, size_t n, uint32_t v) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

int ap_fill_u32(void *p, size_t n, uint32_t v, hipStream_t st) {
    if (n == 0) return AP_OK;
    size_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)blocks), dim3(256), 0, st, (uint32_t *)p, n, v);
    AP_CHECK_HIP(hipGetLastError());
    return AP_OK;
}

int ap_ingest_impl(ap_index *ix, hipStream_t st) {
    const ap_corpus &c = ix->corpus;
    int64_t last = 0;
    AP_CHECK_HIP(hipMemcpyAsync(&last, c.tx_indptr + c.n, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    AP_CHECK_HIP(hipStreamSynchronize(st));
    int64_t sp_last = 0;
    AP_CHECK_HIP(hipMemcpyAsync(&sp_last, c.sp_indptr + c.n, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    AP_CHECK_HIP(hipStreamSynchronize(st));
    AP_REQUIRE(last >= 0 && sp_last >= 0, "indptr[n] is negative");
    AP_REQUIRE(last + sp_last < (1ll << 32), "the two CSR parts together must hold fewer than 2^32 entries");
    ix->tx_nnz = last;
    AP_TRY(ap_dev_alloc(&ix->stats, 4));
    {
        int32_t *bad = reinterpret_cast<int32_t *>(ix->stats);
        AP_TRY(ap_fill_u32(bad, 1, 0, st));
        const int blocks = (int)std::min<int64_t>((c.n + 255) / 256, 8192);
        hipLaunchKernelGGL(k_check_csr, dim3(blocks), dim3(256), 0, st, c.sp_indptr, c.sp_idx, c.sp_val, c.n, sp_last, c.sp_vocab, 0, bad);
        hipLaunchKernelGGL(k_check_csr, dim3(blocks), dim3(256), 0, st, c.tx_indptr, c.tx_idx, c.tx_tf, c.n, last, c.tx_vocab, 1, bad);
        AP_CHECK_HIP(hipGetLastError());
        int32_t h = 0;
        AP_CHECK_HIP(hipMemcpyAsync(&h, bad, sizeof(h), hipMemcpyDeviceToHost, st));
        AP_CHECK_HIP(hipStreamSynchronize(st));
        AP_REQUIRE(h == 0, "the corpus CSR is malformed in %d places (row offsets must ascend from 0 to the total; term ids strictly "
                   "ascending within a row and inside the vocabulary; values finite, term counts not negative)", h);
    }
    AP_TRY(ap_dev_alloc(&ix->tx_w, (size_t)last));
    AP_TRY(ap_dev_alloc(&ix->df, (size_t)c.tx_vocab));
    AP_TRY(ap_dev_alloc(&ix->self_sim, (size_t)c.n));
    AP_TRY(ap_dev_alloc(&ix->dense_norm, (size_t)c.n));
    AP_TRY(ap_dev_alloc(&ix->w_dev, 4));
    AP_TRY(ap_dev_alloc(&ix->counters, 2));
    AP_TRY(ap_fill_u32(ix->counters, 4, 0u, st));
    AP_TRY(ap_fill_u32(ix->df, (size_t)c.tx_vocab, 0, st));
    AP_TRY(ap_fill_u32(ix->stats, 4, 0, st));
    unsigned long long *total = reinterpret_cast<unsigned long long *>(ix->stats + 2);
    if (last > 0) {
        int blocks = (int)((last + 255) / 256 < 8192 ? (last + 255) / 256 : 8192);
        hipLaunchKernelGGL(k_df_and_tokens, dim3(blocks), dim3(256), 0, st, c.tx_idx, c.tx_tf, last, ix->df, total);
        AP_CHECK_HIP(hipGetLastError());
    }
    {
        int blocks = (int)((c.n + 255) / 256 < 8192 ? (c.n + 255) / 256 : 8192);
        hipLaunchKernelGGL(k_bm25_weights, dim3(blocks), dim3(256), 0, st, c.tx_indptr, c.tx_idx, c.tx_tf, c.n, ix->df,
                           total, (double)ix->params.bm25_k1, (double)ix->params.bm25_b, ix->tx_w, ix->stats);
        AP_CHECK_HIP(hipGetLastError());
    }
    ix->docs = ApVecs{c.n, c.dim, c.dense, c.sp_indptr, c.sp_idx, c.sp_val, c.tx_indptr, c.tx_idx, ix->tx_w};
    {
        int64_t waves = c.n < 16384 ? c.n : 16384;
        int blocks = (int)((waves + 3) / 4);
        const float *w = ix->params.build_w;
        if (ix->dtype == AP_F32)
            hipLaunchKernelGGL(k_self_sim<AP_F32>, dim3(blocks), dim3(256), 0, st, ix->docs, w[0], w[1], w[2], ix->self_sim, ix->dense_norm);
        else
            hipLaunchKernelGGL(k_self_sim<AP_BF16>, dim3(blocks), dim3(256), 0, st, ix->docs, w[0], w[1], w[2], ix->self_sim, ix->dense_norm);
        AP_CHECK_HIP(hipGetLastError());
    }
    {
        AP_TRY(ap_dev_alloc(&ix->rec, (size_t)(last + sp_last) + 1));   // one spare entry: the scorers read a record's first entry unconditionally
        AP_TRY(ap_dev_alloc(&ix->meta, (size_t)c.n));
        int32_t *mx = reinterpret_cast<int32_t *>(ix->stats + 1);
        int blocks = (int)((c.n + 255) / 256 < 4096 ? (c.n + 255) / 256 : 4096);
        hipLaunchKernelGGL(k_max_list_len, dim3(blocks), dim3(256), 0, st, c.sp_indptr, c.tx_indptr, c.n, mx);
        AP_CHECK_HIP(hipGetLastError());
        int32_t longest = 0;
        AP_CHECK_HIP(hipMemcpyAsync(&longest, mx, sizeof(int32_t), hipMemcpyDeviceToHost, st));
        AP_CHECK_HIP(hipStreamSynchronize(st));
        AP_REQUIRE(longest < 65536, "a document list has %d entries; at most 65535 per part are supported", longest);
        int64_t waves = c.n < 16384 ? c.n : 16384;
        hipLaunchKernelGGL(k_pack_records, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, ix->docs, ix->dense_norm, ix->rec, ix->meta);
        AP_CHECK_HIP(hipGetLastError());
    }
    AP_CHECK_HIP(hipMemcpyAsync(ix->w_dev, ix->w_default, 3 * sizeof(float), hipMemcpyHostToDevice, st));
    AP_CHECK_HIP(hipStreamSynchronize(st));
    // set-up of this device for searches that must not allocate: the address of their static workspace
    void *ws = nullptr;
    AP_TRY(ap_static_scratch(&ws));
    return AP_OK;
}

static int new_index(const ap_corpus *corpus, const ap_build_params *params, ap_index **out) {
    AP_REQUIRE(out != nullptr, "out is NULL");
    *out = nullptr;
    AP_TRY(ap_validate_corpus(corpus));
    AP_TRY(ap_validate_params(params));
    ap_index *ix = new (std::nothrow) ap_index();
    if (!ix) { ap_set_error("out of host memory"); return AP_ENOMEM; }
    ix->corpus = *corpus;
    ix->params = *params;
    if (ix->params.sp_len == 0) ix->params.sp_len = (ix->params.degree + 5) / 6;
    ix->dtype = corpus->dense_dtype;
    *out = ix;
    return AP_OK;
}

extern "C" int ap_ingest(const ap_corpus *corpus, const ap_build_params *params, void *stream, ap_index **out) {
    AP_TRY(new_index(corpus, params, out));
    int rc = ap_ingest_impl(*out, (hipStream_t)stream);
    if (rc != AP_OK) { ap_free_index(*out); *out = nullptr; }
    return rc;
}

extern "C" void ap_free_index(ap_index *ix) {
    if (!ix) return;
    void *ptrs[] = {ix->kg_en_ip, ix->kg_en, ix->kg_le, ix->kg_le_count, ix->st_se, ix->st_sorted, ix->st_spi, ix->st_sps, ix->deleted, ix->deleted_bad, ix->counters, ix->tx_w, ix->df, ix->stats, ix->self_sim, ix->graph, ix->kw, ix->kw_count, ix->entry, ix->visited, ix->w_dev,
                    ix->search_counts, ix->dense_norm, ix->rec, ix->meta};
    for (void *p : ptrs) if (p) (void)hipFree(p);
    for (hipEvent_t e : ix->ev_search) if (e) (void)hipEventDestroy(e);
    delete ix;
}

extern "C" int ap_set_weights(ap_index *ix, const float w[3]) {
    AP_REQUIRE(ix && w, "NULL argument");
    for (int i = 0; i < 3; i++) AP_REQUIRE(w[i] == w[i] && w[i] - w[i] == 0.f, "weights must be finite");
    memcpy(ix->w_default, w, 3 * sizeof(float));
    // a 12-byte blocking copy: the new default applies to every search enqueued after this call returns
    AP_CHECK_HIP(hipMemcpy(ix->w_dev, ix->w_default, 3 * sizeof(float), hipMemcpyHostToDevice));
    return AP_OK;
}

extern "C" int ap_export_ingest(const ap_index *ix, float *tx_w, int32_t *df, float *avgdl, float *self_sim, void *stream) {
    AP_REQUIRE(ix, "index is NULL");
    hipStream_t st = (hipStream_t)stream;
    if (tx_w) AP_CHECK_HIP(hipMemcpyAsync(tx_w, ix->tx_w, (size_t)ix->tx_nnz * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (df) AP_CHECK_HIP(hipMemcpyAsync(df, ix->df, (size_t)ix->corpus.tx_vocab * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    if (avgdl) AP_CHECK_HIP(hipMemcpyAsync(avgdl, ix->stats, sizeof(float), hipMemcpyDeviceToDevice, st));
    if (self_sim) AP_CHECK_HIP(hipMemcpyAsync(self_sim, ix->self_sim, (size_t)ix->corpus.n * sizeof(float), hipMemcpyDeviceToDevice, st));
    return AP_OK;
}

int ap_alloc_graph(ap_index *ix) {
    const size_t n = (size_t)ix->corpus.n, R = (size_t)ix->params.degree;
    if (!ix->graph) AP_TRY(ap_dev_alloc(&ix->graph, n * R));
    if (!ix->kw) AP_TRY(ap_dev_alloc(&ix->kw, n * (R / 2)));
    if (!ix->kw_count) AP_TRY(ap_dev_alloc(&ix->kw_count, n));
    if (!ix->entry) AP_TRY(ap_dev_alloc(&ix->entry, (size_t)ix->params.n_entry));
    return AP_OK;
}

// An imported graph comes from outside: every id must be -1 (padding) or a document, every keyword count within
// its row.  The searches rely on it.
__global__ void k_count_bad_ids(const int32_t *__restrict__ ids, size_t count, int64_t n, int32_t lo, int32_t *__restrict__ bad) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        if (ids[i] < lo || ids[i] >= n) atomicAdd(bad, 1);
}

static int ap_check_imported(ap_index *ix, hipStream_t st) {
    const size_t n = (size_t)ix->corpus.n, R = (size_t)ix->params.degree;
    int32_t *bad = nullptr;
    AP_TRY(ap_dev_alloc(&bad, 1));
    int rc = ap_fill_u32(bad, 1, 0u, st);
    auto count = [&](const int32_t *p, size_t cnt, int64_t hi, int32_t lo) {
        const unsigned blocks = (unsigned)std::min<size_t>((cnt + 255) / 256, 8192);
        hipLaunchKernelGGL(k_count_bad_ids, dim3(blocks ? blocks : 1), dim3(256), 0, st, p, cnt, hi, lo, bad);
    };
    if (rc == AP_OK) {
        count(ix->graph, n * R, (int64_t)n, -1);
        count(ix->kw, n * (R / 2), (int64_t)n, -1);
        count(ix->kw_count, n, (int64_t)(R / 2) + 1, 0);
        count(ix->entry, (size_t)ix->params.n_entry, (int64_t)n, -1);
    }
    int32_t h = 0;
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(&h, bad, sizeof(h), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(bad);
    if (rc != AP_OK) return rc;
    AP_CHECK_HIP(e);
    AP_REQUIRE(h == 0, "the imported graph holds %d ids or counts out of range", h);
    return AP_OK;
}

extern "C" int ap_import_graph(const ap_corpus *corpus, const ap_build_params *params, const int32_t *semantic,
                               const int32_t *keyword, const int32_t *kw_count, const int32_t *entry, void *stream,
                               ap_index **out) {
    AP_REQUIRE(semantic && entry, "semantic and entry are required");
    AP_REQUIRE((keyword == nullptr) == (kw_count == nullptr), "keyword and kw_count come together or not at all");
    AP_TRY(new_index(corpus, params, out));
    ap_index *ix = *out;
    hipStream_t st = (hipStream_t)stream;
    int rc = ap_ingest_impl(ix, st);
    if (rc == AP_OK) rc = ap_alloc_graph(ix);
    if (rc != AP_OK) { ap_free_index(ix); *out = nullptr; return rc; }
    const size_t n = (size_t)corpus->n, R = (size_t)params->degree;
    hipError_t e = hipMemcpyAsync(ix->graph, semantic, n * R * sizeof(int32_t), hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess && keyword) e = hipMemcpyAsync(ix->kw, keyword, n * (R / 2) * sizeof(int32_t), hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess && kw_count) e = hipMemcpyAsync(ix->kw_count, kw_count, n * sizeof(int32_t), hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess && !kw_count) {
        rc = ap_fill_u32(ix->kw_count, n, 0, st);
        if (rc == AP_OK) rc = ap_fill_u32(ix->kw, n * (R / 2), 0xffffffffu, st);
    }
    if (e == hipSuccess) e = hipMemcpyAsync(ix->entry, entry, (size_t)params->n_entry * sizeof(int32_t), hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e == hipSuccess && rc == AP_OK) rc = ap_check_imported(ix, st);
    if (e != hipSuccess || rc != AP_OK) {
        if (e != hipSuccess) { ap_set_error("graph import copy failed: %s", hipGetErrorString(e)); rc = AP_EHIP; }
        ap_free_index(ix); *out = nullptr; return rc;
    }
    ix->has_graph = true;
    return AP_OK;
}

extern "C" int ap_export_graph(const ap_index *ix, int32_t *semantic, int32_t *keyword, int32_t *kw_count, int32_t *entry,
                               void *stream) {
    AP_REQUIRE(ix, "index is NULL");
    if (!ix->has_graph) { ap_set_error("index has no graph"); return AP_ESTATE; }
    hipStream_t st = (hipStream_t)stream;
    const size_t n = (size_t)ix->corpus.n, R = (size_t)ix->params.degree;
    if (semantic) AP_CHECK_HIP(hipMemcpyAsync(semantic, ix->graph, n * R * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    if (keyword) AP_CHECK_HIP(hipMemcpyAsync(keyword, ix->kw, n * (R / 2) * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    if (kw_count) AP_CHECK_HIP(hipMemcpyAsync(kw_count, ix->kw_count, n * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    if (entry) AP_CHECK_HIP(hipMemcpyAsync(entry, ix->entry, (size_t)ix->params.n_entry * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    return AP_OK;
}

// Mark-deletion (Section 4.1, updates of the hybrid index): deleted documents stay in the graph and are searched
// through; the searches leave them out of their answers.
__global__ void k_mark_deleted(uint32_t *__restrict__ bits, int64_t n, const int32_t *__restrict__ ids, int64_t count, int restore,
                               int32_t *__restrict__ bad) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t v = ids[i];
        if (v < 0 || v >= n) { atomicAdd(bad, 1); continue; }
        if (restore) atomicAnd(&bits[v >> 5], ~(1u << (v & 31)));
        else atomicOr(&bits[v >> 5], 1u << (v & 31));
    }
}

extern "C" int ap_mark_deleted(ap_index *ix, const int32_t *ids, int64_t count, int restore, void *stream) {
    AP_REQUIRE(ix, "index is NULL");
    AP_REQUIRE(count >= 0 && (ids || count == 0), "ids is NULL");
    if (count == 0) return AP_OK;
    hipStream_t st = (hipStream_t)stream;
    const size_t words = ((size_t)ix->corpus.n + 31) / 32;
    if (!ix->deleted) {
        if (restore) return AP_OK;   // nothing was ever deleted
        AP_TRY(ap_dev_alloc(&ix->deleted, words));
        AP_TRY(ap_dev_alloc(&ix->deleted_bad, 1));
        AP_TRY(ap_fill_u32(ix->deleted, words, 0u, st));
    }
    AP_TRY(ap_fill_u32(ix->deleted_bad, 1, 0u, st));
    const unsigned blocks = (unsigned)std::min<int64_t>((count + 255) / 256, 4096);
    hipLaunchKernelGGL(k_mark_deleted, dim3(blocks), dim3(256), 0, st, ix->deleted, ix->corpus.n, ids, count, restore, ix->deleted_bad);
    AP_CHECK_HIP(hipGetLastError());
    int32_t bad = 0;
    AP_CHECK_HIP(hipMemcpyAsync(&bad, ix->deleted_bad, sizeof(bad), hipMemcpyDeviceToHost, st));
    AP_CHECK_HIP(hipStreamSynchronize(st));
    AP_REQUIRE(bad == 0, "%d of the %lld ids are outside [0, n); the others were applied", bad, (long long)count);
    return AP_OK;
}

// A plain streaming copy of known size: the yardstick the HBM byte counters are scaled by.
__global__ void k_copy_u128(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

extern "C" int ap_calibration_copy(void *dst, const void *src, size_t bytes, void *stream) {
    AP_REQUIRE(dst && src && bytes % 16 == 0 && (((uintptr_t)dst | (uintptr_t)src) & 15) == 0, "need 16-byte aligned buffers and size");
    if (bytes == 0) return AP_OK;
    hipLaunchKernelGGL(k_copy_u128, dim3(8192), dim3(256), 0, (hipStream_t)stream, (const uint4 *)src, (uint4 *)dst, bytes / 16);
    AP_CHECK_HIP(hipGetLastError());
    return AP_OK;
}

extern "C" int ap_build_counters(const ap_index *ix, uint64_t out2[2], void *stream) {
    AP_REQUIRE(ix && out2, "NULL argument");
    unsigned long long h[2] = {0, 0};
    AP_CHECK_HIP(hipMemcpyAsync(h, ix->counters, sizeof(h), hipMemcpyDeviceToHost, (hipStream_t)stream));
    AP_CHECK_HIP(hipStreamSynchronize((hipStream_t)stream));
    out2[0] = h[0]; out2[1] = ix->seed_flops;
    return AP_OK;
}

extern "C" int ap_build_timings(const ap_index *ix, float out6[6]) {
    AP_REQUIRE(ix && out6, "NULL argument");
    memcpy(out6, ix->timings, sizeof(ix->timings));
    return AP_OK;
}
