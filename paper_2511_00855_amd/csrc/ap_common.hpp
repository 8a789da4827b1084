// Shared declarations of the gfx950 hybrid-index library: the host-side index
// object, error plumbing, and the wave-cooperative hybrid similarity that every
// kernel (pair scoring, construction, search) calls, so that a pair of vectors
// gets bit-identical component sums wherever it is evaluated.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include "../../include/allanpoe.h"

#define AP_WAVE 64

// ---------------------------------------------------------------- errors
void ap_set_error(const char *fmt, ...);

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
    float *stats = nullptr;    // owned: [0] avgdl
    float *self_sim = nullptr; // owned: fused self-similarity under build_w
    int32_t *graph = nullptr;  // owned: n x degree
    int32_t *kw = nullptr;     // owned: n x degree/2
    int32_t *kw_count = nullptr;
    int32_t *entry = nullptr;  // owned: n_entry
    bool has_graph = false;
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

int ap_validate_corpus(const ap_corpus *c);
int ap_validate_params(const ap_build_params *p);
int ap_ingest_impl(ap_index *ix, hipStream_t st);

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

__device__ __forceinline__ float ap_wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

#define AP_LDS __attribute__((address_space(3)))

// Largest power of two <= n (0 for n <= 0): first stride of the halving search below.
__device__ __forceinline__ int32_t ap_pow2_floor(int32_t n) { return n > 0 ? (1 << (31 - __clz(n))) : 0; }

// If term t occurs in the ascending list a (a_n entries), adds a_val * v to p.
// The lower bound is found with a fixed, wave-uniform number of halving steps
// (no divergence); t = -1 never matches.  IP / VP are pointer types so that a
// list in LDS is read with ds_read and one in global memory with global loads.
template <typename IP, typename VP>
__device__ __forceinline__ float ap_match_fma(IP a_idx, VP a_val, int32_t a_n, int32_t step0, int32_t t, float v, float p) {
    int32_t pos = 0;
    for (int32_t st = step0; st > 0; st >>= 1) {
        const int32_t p2 = pos + st;
        if (p2 <= a_n && a_idx[p2 - 1] < t) pos = p2;
    }
    if (pos < a_n && a_idx[pos] == t) p = fmaf(a_val[pos], v, p);
    return p;
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

// Hybrid similarity (Definition 1) of the a side with up to G rows of B at
// once.  All 64 lanes of the wave take part; the loads of all G rows are
// issued before any of them is consumed, so that G rows are in flight per
// wave.  Row g has its sparse list at [spb[g], spb[g]+spn[g]) and its lexical
// list at [txb[g], txb[g]+txn[g]).  SS / TS are the numbers of 64-entry slots
// of the sparse / lexical list that are prefetched into registers; longer
// lists continue with a plain loop.  Every lane returns the same three sums
// per row, and the sums are bit-identical for any G, SS, TS and pointer kind:
// lane l always accumulates entries l, l+64, ... in that order.
template <int DT, int NV, int G, int SS, int TS, typename IP, typename VP>
__device__ __forceinline__ void ap_hybrid_batch(const ApVecs &B, const float *qa, IP a_sp_idx, VP a_sp_val, int32_t a_sp_n,
                                                IP a_tx_idx, VP a_tx_val, int32_t a_tx_n, int32_t ng, const int32_t *v,
                                                const int64_t *spb, const int32_t *spn, const int64_t *txb,
                                                const int32_t *txn, float *sd, float *ss, float *sf) {
    constexpr int EPC = ApDense<DT>::EPC;
    const int lane = threadIdx.x & 63;
    float d[G][NV * EPC];
    int32_t si[G][SS], ti[G][TS];
    float sv[G][SS], tv[G][TS];
#pragma unroll
    for (int g = 0; g < G; g++) {
        if (g < ng) {
#pragma unroll
            for (int i = 0; i < NV; i++) {
                const int col = (i * 64 + lane) * EPC;
                if (col < B.dim) ApDense<DT>::load(B.dense, v[g], B.dim, col, d[g] + i * EPC);
            }
#pragma unroll
            for (int k = 0; k < SS; k++) {
                const int32_t e = k * 64 + lane;
                si[g][k] = e < spn[g] ? B.sp_idx[spb[g] + e] : -1;
                sv[g][k] = e < spn[g] ? B.sp_val[spb[g] + e] : 0.f;
            }
#pragma unroll
            for (int k = 0; k < TS; k++) {
                const int32_t e = k * 64 + lane;
                ti[g][k] = e < txn[g] ? B.tx_idx[txb[g] + e] : -1;
                tv[g][k] = e < txn[g] ? B.tx_val[txb[g] + e] : 0.f;
            }
        }
    }
    const int32_t sp_step = ap_pow2_floor(a_sp_n), tx_step = ap_pow2_floor(a_tx_n);
#pragma unroll
    for (int g = 0; g < G; g++) {
        if (g < ng) {
            float pd = 0.f, ps = 0.f, pf = 0.f;
#pragma unroll
            for (int i = 0; i < NV; i++) {
                const int col = (i * 64 + lane) * EPC;
                if (col < B.dim) {
#pragma unroll
                    for (int e = 0; e < EPC; e++) pd = fmaf(qa[i * EPC + e], d[g][i * EPC + e], pd);
                }
            }
#pragma unroll
            for (int k = 0; k < SS; k++)
                if (k * 64 < spn[g]) ps = ap_match_fma(a_sp_idx, a_sp_val, a_sp_n, sp_step, si[g][k], sv[g][k], ps);
            for (int32_t e0 = SS * 64; e0 < spn[g]; e0 += 64) {
                const int32_t e = e0 + lane;
                const int32_t t = e < spn[g] ? B.sp_idx[spb[g] + e] : -1;
                const float x = e < spn[g] ? B.sp_val[spb[g] + e] : 0.f;
                ps = ap_match_fma(a_sp_idx, a_sp_val, a_sp_n, sp_step, t, x, ps);
            }
#pragma unroll
            for (int k = 0; k < TS; k++)
                if (k * 64 < txn[g]) pf = ap_match_fma(a_tx_idx, a_tx_val, a_tx_n, tx_step, ti[g][k], tv[g][k], pf);
            for (int32_t e0 = TS * 64; e0 < txn[g]; e0 += 64) {
                const int32_t e = e0 + lane;
                const int32_t t = e < txn[g] ? B.tx_idx[txb[g] + e] : -1;
                const float x = e < txn[g] ? B.tx_val[txb[g] + e] : 0.f;
                pf = ap_match_fma(a_tx_idx, a_tx_val, a_tx_n, tx_step, t, x, pf);
            }
            sd[g] = ap_wave_sum(pd);
            ss[g] = ap_wave_sum(ps);
            sf[g] = ap_wave_sum(pf);
        }
    }
}

// One row: the same arithmetic as the batch form.
template <int DT, int NV>
__device__ __forceinline__ void ap_hybrid_wave(const ApVecs &B, const float *qa, const ApLists &a, int64_t j,
                                               float &sd, float &ss, float &sf) {
    const int32_t v = (int32_t)j;
    const int64_t spb = B.sp_indptr[j], txb = B.tx_indptr[j];
    const int32_t spn = (int32_t)(B.sp_indptr[j + 1] - spb), txn = (int32_t)(B.tx_indptr[j + 1] - txb);
    ap_hybrid_batch<DT, NV, 1, 2, 1>(B, qa, a.sp_idx, a.sp_val, a.sp_n, a.tx_idx, a.tx_val, a.tx_n, 1, &v, &spb, &spn, &txb,
                                     &txn, &sd, &ss, &sf);
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
