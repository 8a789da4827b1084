// Shared declarations of the gfx950 hybrid-index library: the host-side index
// object, error plumbing, and the wave-cooperative hybrid similarity that every
// kernel (pair scoring, construction, search) calls, so that a pair of vectors
// gets bit-identical component sums wherever it is evaluated.
#pragma once
#include <stdlib.h>
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include "../../include/allanpoe.h"

#define AP_WAVE 64

// ---------------------------------------------------------------- errors
void ap_set_error(const char *fmt, ...);
void ap_progress(const char *fmt, ...) __attribute__((format(printf, 1, 2)));   // to stderr, only when ALLANPOE_PROGRESS is set

#define AP_CHECK_HIP(expr)                                                                   \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess) {                                                              \
            ap_set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return AP_EHIP;                                                                  \
        }                                                                                    \
    } while (0)

#define AP_REQUIRE(cond, ...)                                                                \
    do {                                                                                     \
        if (!(cond)) {                                                                       \
            ap_set_error(__VA_ARGS__);                                                       \
            return AP_EINVAL;                                                                \
        }                                                                                    \
    } while (0)

#define AP_TRY(expr)                                                                         \
    do {                                                                                     \
        int rc_ = (expr);                                                                    \
        if (rc_ != AP_OK) return rc_;                                                        \
    } while (0)

// ---------------------------------------------------------------- device views
// One side of the similarity as the kernels see it: dense rows plus two CSR
// parts whose values are already the final weights (BM25 for documents, term
// counts for queries).
struct ApVecs {
    int64_t n;
    int32_t dim;
    const void *dense;
    const int64_t *sp_indptr;
    const int32_t *sp_idx;
    const float *sp_val;
    const int64_t *tx_indptr;
    const int32_t *tx_idx;
    const float *tx_val;
};

struct ap_index {
    ap_corpus corpus;          // borrowed arrays
    ap_build_params params;
    ApVecs docs;               // device view with tx_val = owned BM25 weights
    int32_t dtype;
    int64_t tx_nnz;
    float *tx_w = nullptr;     // owned: BM25 weight per lexical entry
    int32_t *df = nullptr;     // owned: document frequency per term
    unsigned long long *counters = nullptr;   // owned: [0] hybrid similarities evaluated by refinement rounds on this index
    mutable unsigned long long seed_flops = 0;   // FLOPs (2 per multiply-add, padded tiles included) of the seed stage's dense products so far
    float *stats = nullptr;    // owned: [0] avgdl
    float *self_sim = nullptr; // owned: fused self-similarity under build_w
    float *dense_norm = nullptr; // owned: |d_dense| per document (upper bound of the dense part in the search)
    // owned: the search-side copy of the two sparse parts, one contiguous record per document:
    // rec[meta.x .. +sp_n) = (term, weight bits) of the learned-sparse list, then tx_n lexical entries;
    // meta[v] = {first entry, sp_n | tx_n << 16, bits of |d_dense|, 0}
    uint2 *rec = nullptr;
    uint4 *meta = nullptr;
    int32_t *graph = nullptr;  // owned: n x degree
    int32_t *kw = nullptr;     // owned: n x degree/2
    int32_t *kw_count = nullptr;
    int32_t *entry = nullptr;  // owned: n_entry
    bool has_graph = false;
    uint32_t *deleted = nullptr;   // owned: one bit per document, set = mark-deleted (allocated on first use)
    int32_t *deleted_bad = nullptr; // owned: 1 counter, ids out of range in the last ap_mark_deleted
    float w_default[3] = {1.f, 1.f, 1.f};
    // search workspace (grow only)
    uint32_t *visited = nullptr;
    size_t visited_words = 0;
    float *w_dev = nullptr;    // 3 floats: device copy of w_default
    int32_t *search_counts = nullptr;  // nq x 2 of the last search: similarities evaluated, iterations
    size_t search_counts_cap = 0;
    int32_t last_nq = 0;
    hipEvent_t ev_search[2] = {nullptr, nullptr};
    float timings[6] = {0, 0, 0, 0, 0, 0};
    // owned: what the construction leaves behind for later insertions (NULL for imported graphs):
    // pruned lists n x degree, detour-sorted lists n x knn_k, per-path lists 3 x n x sp_len with their scores
    int32_t *st_se = nullptr, *st_sorted = nullptr, *st_spi = nullptr;
    float *st_sps = nullptr;
    // knowledge-graph augmentation (ap_set_knowledge_graph): the caller's entity lists and relations (borrowed),
    // the entity-to-document mapping and the logical edges (owned)
    const int64_t *kg_de_ip = nullptr, *kg_ip = nullptr;
    const int32_t *kg_de = nullptr, *kg_idx = nullptr;
    int64_t *kg_en_ip = nullptr;
    int32_t *kg_en = nullptr, *kg_le = nullptr, *kg_le_count = nullptr;
    int32_t kg_n_ent = 0, kg_le_cap = 0;
    int64_t kg_total = 0;
};

template <typename T>
static inline int ap_dev_alloc(T **p, size_t count) {
    *p = nullptr;
    if (count == 0) count = 1;
    hipError_t e = hipMalloc((void **)p, count * sizeof(T));
    if (e != hipSuccess) {
        ap_set_error("hipMalloc of %zu bytes failed: %s", count * sizeof(T), hipGetErrorString(e));
        return AP_ENOMEM;
    }
    return AP_OK;
}

// Debug settings (ap_debug_set): 0 = the library's own choice.  They exist so that tests can drive small inputs
// through the code paths of large ones; nothing here changes a result.
struct ApDebug {
    int64_t seed_sample_cols = 0;        // columns sampled for the seed threshold (forces the thresholded sweep on small corpora)
    int64_t seed_buffer_cap = 0;         // capacity of a row's candidate buffer in that sweep (forces the overflow fallback)
    int64_t seed_tau_ulps = 0;           // raises every row's threshold by this many ulps (forces the short-row fallback)
    int64_t seed_one_sided = 0;          // 1: whole-corpus seed lists by the one-sided sweep, not the symmetric one
    int64_t max_launch_threads = 0;      // a multiple of 1024: launches that grow with the corpus are cut into slices of this many threads
    int64_t search_visited_global = 0;   // 1: the searches' visited sets stay in global memory even where they would fit LDS
    int64_t search_query_lists = 0;      // 1: the searches look the query's terms up in its lists (the path of queries too long for the LDS tables)
    int64_t search_workspace_bytes = 0;  // cap of the search's visited-set workspace (forces searches in several slabs of queries)
};
extern ApDebug g_ap_debug;

// A kernel launch holds fewer than 2^32 threads: launches whose grid grows with the corpus are cut into slices of at
// most this many threads (grids beyond the limit were seen to wrap around silently).
static inline int64_t ap_max_launch_threads() {
    const int64_t v = g_ap_debug.max_launch_threads;
    return v >= 1024 && v % 1024 == 0 ? v : (int64_t)1 << 31;
}
#define AP_MAX_LAUNCH_THREADS ap_max_launch_threads()

// CSR row offsets must start at 0, never decrease and end at `total`; a row that fails is not read.
__device__ __forceinline__ bool ap_row_ok(const int64_t *ip, int64_t x, int64_t total) {
    const int64_t b = ip[x], e = ip[x + 1];
    return b >= 0 && e >= b && e <= total && (x > 0 || b == 0);
}

// The six stage marks of a construction or an insertion; destroyed on every way out.
struct ApStageEvents {
    hipEvent_t ev[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    hipError_t create() {
        for (auto &e : ev) { const hipError_t r = hipEventCreate(&e); if (r != hipSuccess) return r; }
        return hipSuccess;
    }
    ~ApStageEvents() { for (auto &e : ev) if (e) (void)hipEventDestroy(e); }
};

int ap_validate_corpus(const ap_corpus *c);
int ap_validate_params(const ap_build_params *p);
int ap_ingest_impl(ap_index *ix, hipStream_t st);
int ap_alloc_graph(ap_index *ix);
int ap_fill_u32(void *p, size_t n, uint32_t v, hipStream_t st);
// stage bodies shared by the whole build and by insertion (ap_build.hip)
int ap_seed_knn_impl(const ap_index *ix, const int32_t *node_ids, int64_t nn, int32_t K, int32_t *out_ids, float *out_sc,
                     hipStream_t st);
int ap_prune_impl(const ap_index *ix, int32_t K, int32_t R, const int32_t *knn_ids, const float *knn_sc, const int32_t *node_ids,
                  int64_t nn, float *pm_out, int32_t *count, int32_t *sorted_ids, int32_t *se, int32_t *ke, int32_t *ke_count,
                  int32_t *flag, hipStream_t st);
int ap_assemble_impl(const ap_index *ix, int32_t R, int32_t K, int32_t P, const int32_t *se, const int32_t *sorted_ids,
                     const int32_t *sp_ids, int32_t *out_graph, hipStream_t st);
int ap_rescore_lists(const ap_index *ix, int64_t nn, int32_t K, const int32_t *knn, float *sc, hipStream_t st);
// The visited-set workspace of a search call: `slab` queries are in flight at a time, each with a bitset of one bit
// per document.  `counts` (nq x 3) and the two events belong to the index's measurement surface and may be absent.
struct ApSearchWs {
    uint32_t *visited = nullptr;
    int32_t slab = 0;
    int32_t *counts = nullptr;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
};
// sizes the workspace an index owns (grow only, capped) for a call of nq queries (ap_search.hip)
int ap_search_reserve(ap_index *ix, int32_t nq, hipStream_t st, ApSearchWs *ws);
// address, on the current device, of the static workspace of ap_search_batch_noalloc (looked up once per device)
int ap_static_scratch(void **out);
// the plain search with an arbitrary query view and device weights (ap_search.hip); big_tables: the queries are as long
// as documents, give them larger look-up tables
int ap_search_core(ap_index *ix, const ApVecs &Q, const float *w_dev, int32_t w_stride, int32_t k, int32_t beam, int32_t max_iters,
                   int32_t width, bool big_tables, int32_t *out_ids, float *out_scores, hipStream_t st);

// ---------------------------------------------------------------- device code
#ifdef __HIPCC__

// total order: larger key = ranks first (score descending, id ascending).
// key = [order-preserving score bits : 32][(2^30-1 - id) : 30 .. 1][flag : 0]
__device__ __forceinline__ uint32_t ap_f2ord(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ap_ord2f(uint32_t u) {
    return __uint_as_float((u & 0x80000000u) ? (u & 0x7fffffffu) : ~u);
}
__device__ __forceinline__ uint64_t ap_make_key(float s, int32_t id, uint32_t flag) {
    return ((uint64_t)ap_f2ord(s) << 32) | (uint64_t)(((0x3fffffffu - (uint32_t)id) << 1) | flag);
}
__device__ __forceinline__ int32_t ap_key_id(uint64_t k) {
    return (int32_t)(0x3fffffffu - (((uint32_t)k) >> 1));
}
__device__ __forceinline__ float ap_key_score(uint64_t k) { return ap_ord2f((uint32_t)(k >> 32)); }

template <int DT> struct ApDense;
template <> struct ApDense<AP_F32> {
    static constexpr int EPC = 4;  // elements per 16-byte chunk
    __device__ static __forceinline__ void load(const void *base, int64_t row, int32_t dim, int32_t col, float *o) {
        const float4 v = *reinterpret_cast<const float4 *>(static_cast<const float *>(base) + row * dim + col);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
};
template <> struct ApDense<AP_BF16> {
    static constexpr int EPC = 8;
    __device__ static __forceinline__ void load(const void *base, int64_t row, int32_t dim, int32_t col, float *o) {
        const uint4 v = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(base) + row * dim + col);
        o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
        o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
        o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
        o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
    }
};

// The "a" side of a similarity (the query, or the node whose neighbourhood is
// being built): its two sparse lists, resident in LDS (or global when too
// long), plus its dense slice, which each lane keeps in registers:
// chunk i of lane l covers columns (i*64 + l)*EPC .. +EPC.
struct ApLists {
    const int32_t *sp_idx; const float *sp_val; int32_t sp_n;
    const int32_t *tx_idx; const float *tx_val; int32_t tx_n;
};

// Loads the a side's dense slice into registers with the column mapping of a
// b side stored as DT.  SRC is the storage type of the a side itself (queries
// are always f32; documents are DT).
template <int DT, int NV, int SRC>
__device__ __forceinline__ void ap_load_aside(const void *base, int64_t row, int32_t dim, float *qa) {
    constexpr int EPC = ApDense<DT>::EPC;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < NV; i++) {
        const int col = (i * 64 + lane) * EPC;
        if (col < dim) {
            if (SRC == DT) ApDense<DT>::load(base, row, dim, col, qa + i * EPC);
            else {  // f32 source, bf16 column mapping: 8 consecutive floats
                ApDense<AP_F32>::load(base, row, dim, col, qa + i * EPC);
                ApDense<AP_F32>::load(base, row, dim, col + 4, qa + i * EPC + 4);
            }
        } else {
#pragma unroll
            for (int e = 0; e < EPC; e++) qa[i * EPC + e] = 0.f;
        }
    }
}

// Sum over the 64 lanes of a wave, the same value returned in every lane.
// Inside each row of 16 lanes the exchange is done with DPP (quad permutes,
// then half-row and row mirrors), which costs a VALU cycle or two per step;
// only the last two steps (lanes 16 and 32 apart) go through the LDS crossbar.
template <int CTRL>
__device__ __forceinline__ float ap_dpp(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float ap_wave_sum(float v) {
    v += ap_dpp<0xB1>(v);    // quad_perm [1,0,3,2]: lane ^ 1
    v += ap_dpp<0x4E>(v);    // quad_perm [2,3,0,1]: lane ^ 2
    v += ap_dpp<0x141>(v);   // row_half_mirror: quads 0<->1, 2<->3 of a row
    v += ap_dpp<0x140>(v);   // row_mirror: half rows 0<->1
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}

// Two sums at once: the wave sums of a and of b, each with the additions of ap_wave_sum (the same tree, so the same
// bits), for the price of little more than one.  In the first exchange every lane keeps one of its two values and
// hands the other to its neighbour; from then on half of the lanes reduce a and the other half b.  Which half a lane
// is in, (lane ^ lane >> 2) & 1, is flipped by the first exchange and kept by all the later ones.
__device__ __forceinline__ void ap_wave_sum2(float a, float b, float &sa, float &sb) {
    const int lane = threadIdx.x & 63;
    const bool second = ((lane ^ (lane >> 2)) & 1) != 0;
    float v = second ? b : a;
    v += ap_dpp<0xB1>(second ? a : b);   // the neighbour (lane ^ 1) keeps the other kind and sends this lane's kind
    v += ap_dpp<0x4E>(v);
    v += ap_dpp<0x141>(v);
    v += ap_dpp<0x140>(v);
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    sa = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    sb = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 1));
}

#define AP_LDS __attribute__((address_space(3)))

// Orders one wave's LDS traffic: what any lane wrote before this point is what every lane of the wave reads after it.
// The barrier alone only pins the instruction schedule; the fence is what keeps the compiler from moving or caching
// the accesses across it (the hardware runs a wave's LDS instructions in order).
__device__ __forceinline__ void ap_wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Largest power of two <= n (0 for n <= 0): first stride of the halving search below.
__device__ __forceinline__ int32_t ap_pow2_floor(int32_t n) { return n > 0 ? (1 << (31 - __clz(n))) : 0; }

// If term t occurs in the ascending list a (a_n entries), adds a_val * v to p.
// The lower bound is found with a fixed, wave-uniform number of halving steps
// (no divergence); t = -1 never matches.  IP / VP are pointer types so that a
// list in LDS is read with ds_read and one in global memory with global loads.
template <typename IP, typename VP>
__device__ __forceinline__ float ap_match_fma(IP a_idx, VP a_val, int32_t a_n, int32_t step0, int32_t t, float v, float p) {
    if (a_n <= 0) return p;            // wave-uniform
    // straight-line code: every step reads a valid entry (index clamped) and selects
    int32_t pos = 0;
    for (int32_t st = step0; st > 0; st >>= 1) {
        const int32_t p2 = pos + st;
        const int32_t at = (p2 < a_n ? p2 : a_n) - 1;
        const bool take = (p2 <= a_n) & (a_idx[at] < t);
        pos = take ? p2 : pos;
    }
    const int32_t at = pos < a_n ? pos : a_n - 1;
    const bool hit = (pos < a_n) & (a_idx[at] == t);
    return fmaf(hit ? a_val[at] : 0.f, v, p);   // adds exactly 0 when the term is absent
}

// ---- small open-addressing tables (term -> weight) in LDS ----------------
// A slot is one 64-bit word: term id in the low half (-1 = empty), weight
// bits in the high half.  Linear probing; a table is never more than half
// full, so every probe sequence ends at an empty slot.
__device__ __forceinline__ uint32_t ap_term_hash(int32_t t, int bits) {
    return (__umul24((uint32_t)t & 0xffffffu, 0x9E3779u) ^ ((uint32_t)t >> 24)) >> (32 - bits) ;
}

// ---- bucketed tables: one read per look-up ---------------------------------
// A table of 2^bits slots seen as 2^(bits-1) buckets of two slots (16 bytes, read at once).  A term belongs to the
// bucket its hash names, and the hash's multiplier is chosen per table so that no bucket has to hold three terms: a
// query's few dozen terms nearly always allow that under one of the first multipliers tried (seed 0 is
// ap_term_hash's).  A look-up is then one 16-byte read and two compares, with no probe sequence.
__device__ __forceinline__ uint32_t ap_seed_mult(int32_t seed) { return ((0x9E3779u + 0x3C6EF4u * (uint32_t)seed) | 1u) & 0xffffffu; }
__device__ __forceinline__ uint32_t ap_term_hash_m(int32_t t, uint32_t mult, int bits) {
    return (__umul24((uint32_t)t & 0xffffffu, mult) ^ ((uint32_t)t >> 24)) >> (32 - bits);
}
// Weight of term t, 0 if absent.  An empty slot holds term -1 and weight bits 0, so t = -1 (a lane past the end of
// a list) reads 0 as well.  tab: 16-byte aligned.
template <typename TP>
__device__ __forceinline__ float ap_bucket_get(TP tab, uint32_t mult, int bits, int32_t t) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const uint32_t h = ap_term_hash_m(t, mult, bits - 1);
    const u32x4 b = *reinterpret_cast<const AP_LDS u32x4 *>(tab + 2 * h);
    return __uint_as_float(b.x == (uint32_t)t ? b.y : (b.z == (uint32_t)t ? b.w : 0u));
}
#define AP_SEED_TRIES 32
// One wave builds the table of the n <= 64 CH entries (idx, val), lane l holding entries l, l + 64, ...: it tries
// multipliers until no bucket gets a third term, clears the table and stores the entries.  Every lane returns the
// seed, -1 if none of the first AP_SEED_TRIES does it (the table then holds nothing usable).
template <int CH = 1>
__device__ __forceinline__ int32_t ap_bucket_build(const int32_t *idx, const float *val, int32_t n, uint64_t *tab, int bits) {
    const int lane = threadIdx.x & 63;
    const int32_t nb = 1 << (bits - 1);
    int32_t term[CH];
#pragma unroll
    for (int c = 0; c < CH; c++) term[c] = c * 64 + lane < n ? idx[c * 64 + lane] : -1;
    int32_t *cnt = reinterpret_cast<int32_t *>(tab);   // bucket counters while searching (the table has 2^(bits+1) words)
    for (int32_t s = 0; s < AP_SEED_TRIES; s++) {
        for (int32_t i = lane; i < nb; i += 64) cnt[i] = 0;
        ap_wave_sync();
        uint32_t h[CH];
        int32_t place[CH];
        bool bad = false;
#pragma unroll
        for (int c = 0; c < CH; c++) {
            h[c] = ap_term_hash_m(term[c], ap_seed_mult(s), bits - 1);
            place[c] = c * 64 + lane < n ? atomicAdd(&cnt[h[c]], 1) : 0;
            bad = bad || place[c] >= 2;
        }
        ap_wave_sync();
        if (__ballot(bad) == 0ull) {
            for (int32_t i = lane; i < 2 * nb; i += 64) tab[i] = 0xffffffffull;
            ap_wave_sync();
#pragma unroll
            for (int c = 0; c < CH; c++)
                if (c * 64 + lane < n) tab[2 * h[c] + place[c]] = ((uint64_t)__float_as_uint(val[c * 64 + lane]) << 32) | (uint32_t)term[c];
            return s;
        }
    }
    return -1;
}

// Weight of term t in the table, 0 if absent (t = -1 is never present).
template <typename TP>
__device__ __forceinline__ float ap_table_get(TP tab, int slots, int bits, int32_t t) {
    uint32_t h = ap_term_hash(t, bits);
    for (;;) {
        const uint64_t e = tab[h];
        const int32_t et = (int32_t)(uint32_t)e;
        if (et == t) return __uint_as_float((uint32_t)(e >> 32));
        if (et == -1) return 0.f;
        h = (h + 1) & (slots - 1);
    }
}

// NL look-ups at once: every round issues the LDS reads of all look-ups that
// are still probing, so their latencies overlap; the number of rounds is the
// longest probe sequence among them.  Straight-line code: a finished look-up
// re-reads harmlessly.  Look-ups k < NSP use the first table (2^SPB slots),
// the others the second (2^TXB slots).  val[k] = weight of term[k], 0 if absent.
template <int NL, int NSP, int SPB, int TXB>
__device__ __forceinline__ void ap_table_get_many(const AP_LDS uint64_t *tsp, const AP_LDS uint64_t *ttx, const int32_t *term,
                                                  float *val) {
    uint32_t h[NL];
    bool pend[NL];
    bool any = false;
#pragma unroll
    for (int k = 0; k < NL; k++) {
        h[k] = ap_term_hash(term[k], k < NSP ? SPB : TXB);
        val[k] = 0.f;
        pend[k] = term[k] >= 0;
        any = any || pend[k];
    }
    while (__any(any)) {
        uint64_t e[NL];
#pragma unroll
        for (int k = 0; k < NL; k++) e[k] = k < NSP ? tsp[h[k]] : ttx[h[k]];
        any = false;
#pragma unroll
        for (int k = 0; k < NL; k++) {
            const int32_t et = (int32_t)(uint32_t)e[k];
            const bool hit = pend[k] & (et == term[k]);
            val[k] = hit ? __uint_as_float((uint32_t)(e[k] >> 32)) : val[k];
            pend[k] = pend[k] & (et != term[k]) & (et != -1);
            h[k] = (h[k] + 1) & ((1u << (k < NSP ? SPB : TXB)) - 1u);
            any = any | pend[k];
        }
    }
}

// Inserts (term, weight bits) into a table that holds no such term yet.
__device__ __forceinline__ void ap_table_put(uint64_t *tab, int slots, int bits, int32_t t, int32_t vb) {
    int32_t *w32 = reinterpret_cast<int32_t *>(tab);
    uint32_t h = ap_term_hash(t, bits);
    for (;;) {
        const int32_t old = atomicCAS(&w32[2 * h], -1, t);
        if (old == -1) { w32[2 * h + 1] = vb; return; }
        h = (h + 1) & (slots - 1);
    }
}

// Partial inner product of an ascending list held by the a side with the
// b side's list [beg, end) in global memory: lane l takes entries
// beg+l, beg+l+64, ... of b and searches a (Section 4.1, Step 1; on the search
// side the document's entries are looked up in the short query list,
// Section 4.2.1).
template <typename IP, typename VP>
__device__ __forceinline__ float ap_sparse_partial(IP a_idx, VP a_val, int32_t a_n, const int32_t *b_idx,
                                                   const float *b_val, int64_t beg, int64_t end, int lane) {
    float p = 0.f;
    const int32_t step0 = ap_pow2_floor(a_n);
    for (int64_t e0 = beg; e0 < end; e0 += 64) {
        const int64_t e = e0 + lane;
        const int32_t t = e < end ? b_idx[e] : -1;
        const float v = e < end ? b_val[e] : 0.f;
        p = ap_match_fma(a_idx, a_val, a_n, step0, t, v, p);
    }
    return p;
}

// Dense part of Definition 1: <a_d, B_d[row]>, lane l holding columns (64i+l)*EPC.. of the a side in qa.
// All lanes return the same sum.
template <int DT, int NV>
__device__ __forceinline__ float ap_dense_dot(const ApVecs &B, const float *qa, int64_t row) {
    constexpr int EPC = ApDense<DT>::EPC;
    const int lane = threadIdx.x & 63;
    float d[NV * EPC];
#pragma unroll
    for (int i = 0; i < NV; i++) {
        const int col = (i * 64 + lane) * EPC;
        if (col < B.dim) ApDense<DT>::load(B.dense, row, B.dim, col, d + i * EPC);
    }
    float pd = 0.f;
#pragma unroll
    for (int i = 0; i < NV; i++) {
        const int col = (i * 64 + lane) * EPC;
        if (col < B.dim) {
#pragma unroll
            for (int e = 0; e < EPC; e++) pd = fmaf(qa[i * EPC + e], d[i * EPC + e], pd);
        }
    }
    return ap_wave_sum(pd);
}

// The same product in two steps, so that the rows of several candidates can be on their way before the first is
// used: the raw 16-byte groups first, the multiply-adds (same order, same bits as ap_dense_dot) later.
template <int DT, int NV>
__device__ __forceinline__ void ap_dense_load_raw(const ApVecs &B, int64_t row, uint4 *raw) {
    constexpr int EPC = ApDense<DT>::EPC;
    const int lane = threadIdx.x & 63;
    const char *base = static_cast<const char *>(B.dense) + row * (int64_t)B.dim * (16 / EPC);
#pragma unroll
    for (int i = 0; i < NV; i++) {   // a lane past the end of the row re-reads the row's first group (never used: see ap_dense_dot_raw)
        const int col = (i * 64 + lane) * EPC;
        raw[i] = *reinterpret_cast<const uint4 *>(base + (int64_t)(col < B.dim ? col : 0) * (16 / EPC));
    }
}
template <int DT, int NV>
__device__ __forceinline__ float ap_dense_dot_raw(const ApVecs &B, const float *qa, const uint4 *raw) {
    constexpr int EPC = ApDense<DT>::EPC;
    const int lane = threadIdx.x & 63;
    float pd = 0.f;
#pragma unroll
    for (int i = 0; i < NV; i++) {
        const int col = (i * 64 + lane) * EPC;
        if (col < B.dim) {
            float d[EPC];
            const uint4 v = raw[i];
            if constexpr (DT == AP_F32) {
                d[0] = __uint_as_float(v.x); d[1] = __uint_as_float(v.y); d[2] = __uint_as_float(v.z); d[3] = __uint_as_float(v.w);
            } else {
                d[0] = __uint_as_float(v.x << 16); d[1] = __uint_as_float(v.x & 0xffff0000u);
                d[2] = __uint_as_float(v.y << 16); d[3] = __uint_as_float(v.y & 0xffff0000u);
                d[4] = __uint_as_float(v.z << 16); d[5] = __uint_as_float(v.z & 0xffff0000u);
                d[6] = __uint_as_float(v.w << 16); d[7] = __uint_as_float(v.w & 0xffff0000u);
            }
#pragma unroll
            for (int e = 0; e < EPC; e++) pd = fmaf(qa[i * EPC + e], d[e], pd);
        }
    }
    return ap_wave_sum(pd);
}

// Sparse and lexical parts of Definition 1 for one row of B whose lists are at
// [spb, spb+spn) and [txb, txb+txn).  The first SS / TS 64-entry slots of the
// two lists are loaded before any look-up starts (all loads in flight
// together); longer lists continue with a plain loop.  Lane l always
// accumulates entries l, l+64, ... in that order, so the sums do not depend
// on SS, TS or on where the a side's lists live.
template <int SS, int TS>
__device__ __forceinline__ void ap_lists_load(const ApVecs &B, int64_t spb, int32_t spn, int64_t txb, int32_t txn,
                                              int32_t *si, float *sv, int32_t *ti, float *tv) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 0; k < SS; k++) {
        const int32_t e = k * 64 + lane;
        si[k] = e < spn ? B.sp_idx[spb + e] : -1;
        sv[k] = e < spn ? B.sp_val[spb + e] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < TS; k++) {
        const int32_t e = k * 64 + lane;
        ti[k] = e < txn ? B.tx_idx[txb + e] : -1;
        tv[k] = e < txn ? B.tx_val[txb + e] : 0.f;
    }
}

// A wave-uniform 32-bit value moved to scalar registers.  The builtin returns a signed int: an offset of 2^31 or more
// must come back as unsigned before it is added to a pointer.
__device__ __forceinline__ uint32_t ap_uniform_u32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ int32_t ap_uniform_i32(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint64_t ap_uniform_u64(uint64_t v) {
    return ((uint64_t)ap_uniform_u32((uint32_t)(v >> 32)) << 32) | (uint64_t)ap_uniform_u32((uint32_t)v);
}
// The wave's number inside its workgroup, as a scalar: loops that stride over it then run on scalar branches.
__device__ __forceinline__ int ap_wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// ---- packed document records (search side) -------------------------------
// One document's sparse entries followed by its lexical entries, 8 bytes each
// (term id, weight bits), so that a candidate costs one contiguous segment
// and one 16-byte descriptor instead of four segments and five scattered words.
// `r` points at the document's first entry (wave-uniform).
// Straight-line code: a lane past the end of a list reads the record's first entry instead (a line the wave fetches
// anyway) and discards it, so the loads issue back to back with no branch around any of them.  The record array
// ends with one spare entry, so that the first entry of an empty record is readable too.
template <int SS, int TS>
__device__ __forceinline__ void ap_rec_load_raw(const uint2 *r, int32_t spn, int32_t txn, uint2 *xs, uint2 *xt) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 0; k < SS; k++) { const int32_t e = k * 64 + lane; xs[k] = r[e < spn ? e : 0]; }
#pragma unroll
    for (int k = 0; k < TS; k++) { const int32_t e = k * 64 + lane; xt[k] = r[e < txn ? spn + e : 0]; }
}
// What the loads brought, as (term, weight) per slot.  A lane past the end of a list gets term -1, which no look-up
// finds, so that its weight (the first entry's, a finite number) is multiplied by exactly 0.
template <int SS, int TS>
__device__ __forceinline__ void ap_rec_decode(const uint2 *xs, const uint2 *xt, int32_t spn, int32_t txn, int32_t *si, float *sv,
                                              int32_t *ti, float *tv) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 0; k < SS; k++) {
        const bool ok = k * 64 + lane < spn;
        si[k] = ok ? (int32_t)xs[k].x : -1; sv[k] = __uint_as_float(xs[k].y);
    }
#pragma unroll
    for (int k = 0; k < TS; k++) {
        const bool ok = k * 64 + lane < txn;
        ti[k] = ok ? (int32_t)xt[k].x : -1; tv[k] = __uint_as_float(xt[k].y);
    }
}
template <int SS, int TS>
__device__ __forceinline__ void ap_rec_load(const uint2 *r, int32_t spn, int32_t txn, int32_t *si, float *sv, int32_t *ti, float *tv) {
    uint2 xs[SS], xt[TS];
    ap_rec_load_raw<SS, TS>(r, spn, txn, xs, xt);
    ap_rec_decode<SS, TS>(xs, xt, spn, txn, si, sv, ti, tv);
}

// Sparse and lexical sums of a packed record against the a side's look-up
// tables; same per-lane accumulation order as ap_lists_reduce.
template <int SS, int TS, int SPB, int TXB>
__device__ __forceinline__ void ap_rec_reduce_tab(const uint2 *r, const AP_LDS uint64_t *tsp, const AP_LDS uint64_t *ttx, int32_t spn,
                                                  int32_t txn, const int32_t *si, const float *sv, const int32_t *ti,
                                                  const float *tv, float &ss, float &sf) {
    const int lane = threadIdx.x & 63;
    int32_t term[SS + TS];
    float av[SS + TS];
#pragma unroll
    for (int k = 0; k < SS; k++) term[k] = si[k];
#pragma unroll
    for (int k = 0; k < TS; k++) term[SS + k] = ti[k];
    ap_table_get_many<SS + TS, SS, SPB, TXB>(tsp, ttx, term, av);
    float ps = 0.f, pf = 0.f;
#pragma unroll
    for (int k = 0; k < SS; k++) ps = fmaf(av[k], sv[k], ps);
    for (int32_t e0 = SS * 64; e0 < spn; e0 += 64) {
        const int32_t e = e0 + lane;
        uint2 x = make_uint2(0xffffffffu, 0u);
        if (e < spn) x = r[e];
        ps = fmaf((int32_t)x.x >= 0 ? ap_table_get(tsp, 1 << SPB, SPB, (int32_t)x.x) : 0.f, __uint_as_float(x.y), ps);
    }
#pragma unroll
    for (int k = 0; k < TS; k++) pf = fmaf(av[SS + k], tv[k], pf);
    for (int32_t e0 = TS * 64; e0 < txn; e0 += 64) {
        const int32_t e = e0 + lane;
        uint2 x = make_uint2(0xffffffffu, 0u);
        if (e < txn) x = r[spn + e];
        pf = fmaf((int32_t)x.x >= 0 ? ap_table_get(ttx, 1 << TXB, TXB, (int32_t)x.x) : 0.f, __uint_as_float(x.y), pf);
    }
    ss = ap_wave_sum(ps);
    sf = ap_wave_sum(pf);
}

// The same sums against bucketed tables (multipliers msp, mtx): one read per look-up, no probing, and the two
// wave sums share their exchanges.  Same per-lane accumulation order, same reduction tree: the same bits.
template <int SS, int TS, int SPB, int TXB>
__device__ __forceinline__ void ap_rec_reduce_bucket(const uint2 *r, const AP_LDS uint64_t *tsp, const AP_LDS uint64_t *ttx, uint32_t msp,
                                                     uint32_t mtx, int32_t spn, int32_t txn, const int32_t *si, const float *sv,
                                                     const int32_t *ti, const float *tv, float &ss, float &sf) {
    const int lane = threadIdx.x & 63;
    float av[SS + TS];
#pragma unroll
    for (int k = 0; k < SS; k++) av[k] = ap_bucket_get(tsp, msp, SPB, si[k]);
#pragma unroll
    for (int k = 0; k < TS; k++) av[SS + k] = ap_bucket_get(ttx, mtx, TXB, ti[k]);
    float ps = 0.f, pf = 0.f;
#pragma unroll
    for (int k = 0; k < SS; k++) ps = fmaf(av[k], sv[k], ps);
    for (int32_t e0 = SS * 64; e0 < spn; e0 += 64) {
        const int32_t e = e0 + lane;
        uint2 x = make_uint2(0xffffffffu, 0u);
        if (e < spn) x = r[e];
        ps = fmaf(ap_bucket_get(tsp, msp, SPB, (int32_t)x.x), __uint_as_float(x.y), ps);
    }
#pragma unroll
    for (int k = 0; k < TS; k++) pf = fmaf(av[SS + k], tv[k], pf);
    for (int32_t e0 = TS * 64; e0 < txn; e0 += 64) {
        const int32_t e = e0 + lane;
        uint2 x = make_uint2(0xffffffffu, 0u);
        if (e < txn) x = r[spn + e];
        pf = fmaf(ap_bucket_get(ttx, mtx, TXB, (int32_t)x.x), __uint_as_float(x.y), pf);
    }
    ap_wave_sum2(ps, pf, ss, sf);
}

// The same sums with the a side's lists searched where they lie (lists too long for the tables).
template <int SS, int TS>
__device__ __forceinline__ void ap_rec_reduce_lists(const uint2 *r, const ApLists &a, int32_t spn, int32_t txn, const int32_t *si,
                                                    const float *sv, const int32_t *ti, const float *tv, float &ss, float &sf) {
    const int lane = threadIdx.x & 63;
    const int32_t sp_step = ap_pow2_floor(a.sp_n), tx_step = ap_pow2_floor(a.tx_n);
    float ps = 0.f, pf = 0.f;
#pragma unroll
    for (int k = 0; k < SS; k++) ps = ap_match_fma(a.sp_idx, a.sp_val, a.sp_n, sp_step, si[k], sv[k], ps);
    for (int32_t e0 = SS * 64; e0 < spn; e0 += 64) {
        const int32_t e = e0 + lane;
        uint2 x = make_uint2(0xffffffffu, 0u);
        if (e < spn) x = r[e];
        ps = ap_match_fma(a.sp_idx, a.sp_val, a.sp_n, sp_step, (int32_t)x.x, __uint_as_float(x.y), ps);
    }
#pragma unroll
    for (int k = 0; k < TS; k++) pf = ap_match_fma(a.tx_idx, a.tx_val, a.tx_n, tx_step, ti[k], tv[k], pf);
    for (int32_t e0 = TS * 64; e0 < txn; e0 += 64) {
        const int32_t e = e0 + lane;
        uint2 x = make_uint2(0xffffffffu, 0u);
        if (e < txn) x = r[spn + e];
        pf = ap_match_fma(a.tx_idx, a.tx_val, a.tx_n, tx_step, (int32_t)x.x, __uint_as_float(x.y), pf);
    }
    ss = ap_wave_sum(ps);
    sf = ap_wave_sum(pf);
}

template <int SS, int TS, typename IP, typename VP>
__device__ __forceinline__ void ap_lists_reduce(const ApVecs &B, IP a_sp_idx, VP a_sp_val, int32_t a_sp_n, IP a_tx_idx,
                                                VP a_tx_val, int32_t a_tx_n, int64_t spb, int32_t spn, int64_t txb,
                                                int32_t txn, const int32_t *si, const float *sv, const int32_t *ti,
                                                const float *tv, float &ss, float &sf) {
    const int lane = threadIdx.x & 63;
    const int32_t sp_step = ap_pow2_floor(a_sp_n), tx_step = ap_pow2_floor(a_tx_n);
    float ps = 0.f, pf = 0.f;
#pragma unroll
    for (int k = 0; k < SS; k++)
        if (k * 64 < spn) ps = ap_match_fma(a_sp_idx, a_sp_val, a_sp_n, sp_step, si[k], sv[k], ps);
    for (int32_t e0 = SS * 64; e0 < spn; e0 += 64) {
        const int32_t e = e0 + lane;
        const int32_t t = e < spn ? B.sp_idx[spb + e] : -1;
        const float x = e < spn ? B.sp_val[spb + e] : 0.f;
        ps = ap_match_fma(a_sp_idx, a_sp_val, a_sp_n, sp_step, t, x, ps);
    }
#pragma unroll
    for (int k = 0; k < TS; k++)
        if (k * 64 < txn) pf = ap_match_fma(a_tx_idx, a_tx_val, a_tx_n, tx_step, ti[k], tv[k], pf);
    for (int32_t e0 = TS * 64; e0 < txn; e0 += 64) {
        const int32_t e = e0 + lane;
        const int32_t t = e < txn ? B.tx_idx[txb + e] : -1;
        const float x = e < txn ? B.tx_val[txb + e] : 0.f;
        pf = ap_match_fma(a_tx_idx, a_tx_val, a_tx_n, tx_step, t, x, pf);
    }
    ss = ap_wave_sum(ps);
    sf = ap_wave_sum(pf);
}

template <int SS, int TS, typename IP, typename VP>
__device__ __forceinline__ void ap_lists_dot(const ApVecs &B, IP a_sp_idx, VP a_sp_val, int32_t a_sp_n, IP a_tx_idx,
                                             VP a_tx_val, int32_t a_tx_n, int64_t spb, int32_t spn, int64_t txb, int32_t txn,
                                             float &ss, float &sf) {
    int32_t si[SS], ti[TS];
    float sv[SS], tv[TS];
    ap_lists_load<SS, TS>(B, spb, spn, txb, txn, si, sv, ti, tv);
    ap_lists_reduce<SS, TS>(B, a_sp_idx, a_sp_val, a_sp_n, a_tx_idx, a_tx_val, a_tx_n, spb, spn, txb, txn, si, sv, ti, tv, ss, sf);
}

// Hybrid similarity (Definition 1) of the a side with row j of B.  All 64
// lanes take part and all return the same three sums.
template <int DT, int NV>
__device__ __forceinline__ void ap_hybrid_wave(const ApVecs &B, const float *qa, const ApLists &a, int64_t j,
                                               float &sd, float &ss, float &sf) {
    const int64_t spb = B.sp_indptr[j], txb = B.tx_indptr[j];
    const int32_t spn = (int32_t)(B.sp_indptr[j + 1] - spb), txn = (int32_t)(B.tx_indptr[j + 1] - txb);
    sd = ap_dense_dot<DT, NV>(B, qa, j);
    ap_lists_dot<2, 1>(B, a.sp_idx, a.sp_val, a.sp_n, a.tx_idx, a.tx_val, a.tx_n, spb, spn, txb, txn, ss, sf);
}

__device__ __forceinline__ float ap_fuse(float wd, float ws, float wf, float sd, float ss, float sf) {
    return fmaf(wf, sf, fmaf(ws, ss, wd * sd));
}

// Copies the two lists of row `row` of A into LDS (cap entries each) and
// returns pointers to them; a list longer than cap stays in global memory.
__device__ __forceinline__ ApLists ap_stage_lists(const ApVecs &A, int64_t row, int32_t *l_sp_idx, float *l_sp_val,
                                                  int32_t *l_tx_idx, float *l_tx_val, int cap) {
    ApLists a;
    const int64_t sb = A.sp_indptr[row], se = A.sp_indptr[row + 1];
    const int64_t tb = A.tx_indptr[row], te = A.tx_indptr[row + 1];
    a.sp_n = (int32_t)(se - sb);
    a.tx_n = (int32_t)(te - tb);
    if (a.sp_n <= cap) {
        for (int i = threadIdx.x; i < a.sp_n; i += blockDim.x) { l_sp_idx[i] = A.sp_idx[sb + i]; l_sp_val[i] = A.sp_val[sb + i]; }
        a.sp_idx = l_sp_idx; a.sp_val = l_sp_val;
    } else { a.sp_idx = A.sp_idx + sb; a.sp_val = A.sp_val + sb; }
    if (a.tx_n <= cap) {
        for (int i = threadIdx.x; i < a.tx_n; i += blockDim.x) { l_tx_idx[i] = A.tx_idx[tb + i]; l_tx_val[i] = A.tx_val[tb + i]; }
        a.tx_idx = l_tx_idx; a.tx_val = l_tx_val;
    } else { a.tx_idx = A.tx_idx + tb; a.tx_val = A.tx_val + tb; }
    return a;
}

// dispatch on (dense dtype, chunks per lane): F(kernel-args...) is expanded
// with DT and NV as compile-time constants.
#define AP_DISPATCH_DENSE(dtype, dim, BODY)                                                      \
    do {                                                                                         \
        const int epc_ = (dtype) == AP_BF16 ? 8 : 4;                                             \
        const int nv_ = ((dim) + 64 * epc_ - 1) / (64 * epc_);                                   \
        if ((dtype) == AP_F32) {                                                                 \
            if (nv_ <= 1) { constexpr int DT = AP_F32, NV = 1; BODY; }                           \
            else if (nv_ == 2) { constexpr int DT = AP_F32, NV = 2; BODY; }                      \
            else if (nv_ == 3) { constexpr int DT = AP_F32, NV = 3; BODY; }                      \
            else { constexpr int DT = AP_F32, NV = 4; BODY; }                                    \
        } else {                                                                                 \
            if (nv_ <= 1) { constexpr int DT = AP_BF16, NV = 1; BODY; }                          \
            else if (nv_ == 2) { constexpr int DT = AP_BF16, NV = 2; BODY; }                     \
            else if (nv_ == 3) { constexpr int DT = AP_BF16, NV = 3; BODY; }                     \
            else { constexpr int DT = AP_BF16, NV = 4; BODY; }                                   \
        }                                                                                        \
    } while (0)

#endif  // __HIPCC__
