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

// Partial inner product of an ascending list held by the a side with the
// b side's list [beg, end) in global memory: lane l takes entries
// beg+l, beg+l+64, ... of b and binary-searches a (Section 4.1, Step 1).
__device__ __forceinline__ float ap_sparse_partial(const int32_t *a_idx, const float *a_val, int32_t a_n,
                                                   const int32_t *b_idx, const float *b_val, int64_t beg,
                                                   int64_t end, int lane) {
    float p = 0.f;
    for (int64_t e = beg + lane; e < end; e += 64) {
        const int32_t t = b_idx[e];
        const float v = b_val[e];
        int32_t lo = 0, hi = a_n;
        while (lo < hi) {
            const int32_t mid = (lo + hi) >> 1;
            if (a_idx[mid] < t) lo = mid + 1; else hi = mid;
        }
        if (lo < a_n && a_idx[lo] == t) p = fmaf(a_val[lo], v, p);
    }
    return p;
}

// Hybrid similarity of the a side with row j of B (Definition 1).  All 64
// lanes of the wave take part and all return the same three sums.
template <int DT, int NV>
__device__ __forceinline__ void ap_hybrid_wave(const ApVecs &B, const float *qa, const ApLists &a, int64_t j,
                                               float &sd, float &ss, float &sf) {
    constexpr int EPC = ApDense<DT>::EPC;
    const int lane = threadIdx.x & 63;
    float pd = 0.f;
#pragma unroll
    for (int i = 0; i < NV; i++) {
        const int col = (i * 64 + lane) * EPC;
        if (col < B.dim) {
            float d[EPC];
            ApDense<DT>::load(B.dense, j, B.dim, col, d);
#pragma unroll
            for (int e = 0; e < EPC; e++) pd = fmaf(qa[i * EPC + e], d[e], pd);
        }
    }
    const float ps = ap_sparse_partial(a.sp_idx, a.sp_val, a.sp_n, B.sp_idx, B.sp_val, B.sp_indptr[j],
                                       B.sp_indptr[j + 1], lane);
    const float pf = ap_sparse_partial(a.tx_idx, a.tx_val, a.tx_n, B.tx_idx, B.tx_val, B.tx_indptr[j],
                                       B.tx_indptr[j + 1], lane);
    sd = ap_wave_sum(pd);
    ss = ap_wave_sum(ps);
    sf = ap_wave_sum(pf);
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
