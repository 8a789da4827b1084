// S1 as stand-alone calls: hybrid similarities of explicit (a, candidate)
// pairs, and the exhaustive scorer + exact top-k used as ground truth.
#include "ap_common.hpp"

#define AP_LIST_CAP 512  // a-side list entries staged in LDS; longer lists are read from global memory

// One block (4 waves) per a row and chunk of candidates; wave w takes
// candidates chunk_begin + w, + 4, ...
template <int DT, int NV, int SRC>
__global__ __launch_bounds__(256) void k_hybrid_pairs(ApVecs A, ApVecs B, const int32_t *__restrict__ a_ids,
                                                      const int32_t *__restrict__ cand, int32_t c, int32_t chunk,
                                                      const float *__restrict__ w, int32_t w_stride,
                                                      float *__restrict__ out4) {
    __shared__ int32_t l_sp_idx[AP_LIST_CAP];
    __shared__ float l_sp_val[AP_LIST_CAP];
    __shared__ int32_t l_tx_idx[AP_LIST_CAP];
    __shared__ float l_tx_val[AP_LIST_CAP];
    const int64_t x = blockIdx.x;
    const int64_t row = a_ids ? (int64_t)a_ids[x] : x;
    const int32_t y0 = blockIdx.y * chunk;
    const int32_t y1 = y0 + chunk < c ? y0 + chunk : c;
    if (row < 0 || row >= A.n) {   // not a row of A: the whole line of results is holes (uniform over the workgroup)
        for (int32_t y = y0 + (int32_t)threadIdx.x; y < y1; y += blockDim.x)
            *reinterpret_cast<float4 *>(out4 + (x * c + y) * 4) = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        return;
    }
    const ApLists a = ap_stage_lists(A, row, l_sp_idx, l_sp_val, l_tx_idx, l_tx_val, AP_LIST_CAP);
    float qa[NV * ApDense<DT>::EPC];
    ap_load_aside<DT, NV, SRC>(A.dense, row, A.dim, qa);
    __syncthreads();
    const float wd = w[x * w_stride + 0], ws = w[x * w_stride + 1], wf = w[x * w_stride + 2];
    const int lane = threadIdx.x & 63, wave = ap_wave_id();
    for (int32_t y = y0 + wave; y < y1; y += 4) {
        const int32_t j = cand[x * c + y];
        float sd, ss, sf, fu;
        if (j >= 0 && j < B.n) {
            ap_hybrid_wave<DT, NV>(B, qa, a, j, sd, ss, sf);
            fu = ap_fuse(wd, ws, wf, sd, ss, sf);
        } else {
            sd = ss = sf = fu = -INFINITY;
        }
        if (lane == 0) *reinterpret_cast<float4 *>(out4 + (x * c + y) * 4) = make_float4(sd, ss, sf, fu);
    }
}

static ApVecs query_view(const ap_queries *q, int32_t dim) {
    return ApVecs{q->nq, dim, q->dense, q->sp_indptr, q->sp_idx, q->sp_val, q->tx_indptr, q->tx_idx, q->tx_cnt};
}

int ap_validate_queries(const ap_queries *q) {
    AP_REQUIRE(q != nullptr, "queries is NULL");
    AP_REQUIRE(q->nq >= 0, "queries.nq is negative");
    if (q->nq == 0) return AP_OK;
    AP_REQUIRE(q->dense && q->sp_indptr && q->sp_idx && q->sp_val && q->tx_indptr && q->tx_idx && q->tx_cnt,
               "queries has a NULL array");
    AP_REQUIRE(((uintptr_t)q->dense & 15) == 0, "queries.dense must be 16-byte aligned");
    return AP_OK;
}

extern "C" int ap_hybrid_scores(const ap_index *ix, const ap_queries *q, const int32_t *cand_ids, int32_t c,
                                const float *per_query_w, float *out4, void *stream) {
    AP_REQUIRE(ix && cand_ids && out4, "NULL argument");
    AP_TRY(ap_validate_queries(q));
    AP_REQUIRE(c >= 0, "c is negative");
    if (q->nq == 0 || c == 0) return AP_OK;
    AP_REQUIRE(((uintptr_t)out4 & 15) == 0, "out4 must be 16-byte aligned");
    const ApVecs A = query_view(q, ix->docs.dim);
    const float *w = per_query_w ? per_query_w : ix->w_dev;
    const int32_t ws = per_query_w ? 3 : 0;
    int32_t chunk = 256;
    // enough blocks to fill the chip even for few queries
    while (chunk > 16 && (int64_t)q->nq * ((c + chunk - 1) / chunk) < 2048) chunk >>= 1;
    dim3 grid((unsigned)q->nq, (unsigned)((c + chunk - 1) / chunk));
    AP_REQUIRE(grid.y <= 65535, "too many candidates per query");
    AP_DISPATCH_DENSE(ix->dtype, ix->docs.dim,
                      hipLaunchKernelGGL((k_hybrid_pairs<DT, NV, AP_F32>), grid, dim3(256), 0, (hipStream_t)stream, A,
                                         ix->docs, (const int32_t *)nullptr, cand_ids, c, chunk, w, ws, out4));
    AP_CHECK_HIP(hipGetLastError());
    return AP_OK;
}

extern "C" int ap_hybrid_scores_docs(const ap_index *ix, const int32_t *a_ids, int32_t na, const int32_t *cand_ids,
                                     int32_t c, const float w3[3], float *out4, void *stream) {
    AP_REQUIRE(ix && a_ids && cand_ids && out4 && w3, "NULL argument");
    AP_REQUIRE(na >= 0 && c >= 0, "negative count");
    if (na == 0 || c == 0) return AP_OK;
    AP_REQUIRE(((uintptr_t)out4 & 15) == 0, "out4 must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    // weights travel through a small device buffer owned by this call
    float *wdev = nullptr;
    AP_TRY(ap_dev_alloc(&wdev, 4));
    hipError_t e = hipMemcpyAsync(wdev, w3, 3 * sizeof(float), hipMemcpyHostToDevice, st);
    if (e != hipSuccess) { (void)hipFree(wdev); ap_set_error("weight copy failed: %s", hipGetErrorString(e)); return AP_EHIP; }
    int32_t chunk = 256;
    while (chunk > 16 && (int64_t)na * ((c + chunk - 1) / chunk) < 2048) chunk >>= 1;
    dim3 grid((unsigned)na, (unsigned)((c + chunk - 1) / chunk));
    if (grid.y > 65535) { (void)hipFree(wdev); ap_set_error("too many candidates per row"); return AP_EINVAL; }
    AP_DISPATCH_DENSE(ix->dtype, ix->docs.dim,
                      hipLaunchKernelGGL((k_hybrid_pairs<DT, NV, DT>), grid, dim3(256), 0, st, ix->docs, ix->docs, a_ids,
                                         cand_ids, c, chunk, (const float *)wdev, 0, out4));
    e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(wdev);
    if (e != hipSuccess) { ap_set_error("ap_hybrid_scores_docs failed: %s", hipGetErrorString(e)); return AP_EHIP; }
    return AP_OK;
}

// ------------------------------------------------------------------ exhaustive scorer
// Ground truth for recall: fused scores of a block of queries against every
// document, then exact top-k by repeated arg-max under the total order.
// The document row sits in registers and is reused for QB queries staged in
// LDS, so the corpus is streamed nq/QB times instead of nq times.
#define AP_BF_QB 8
#define AP_BF_QCAP 64

template <int DT, int NV>
__global__ __launch_bounds__(256) void k_bf_scores(ApVecs Q, ApVecs D, int32_t q0, int32_t nqb,
                                                   const float *__restrict__ w, int32_t w_stride,
                                                   float *__restrict__ scores /* nqb x n */) {
    constexpr int EPC = ApDense<DT>::EPC;
    extern __shared__ float smem[];
    float *qd = smem;                                                // QB x dim
    int32_t *qsi = reinterpret_cast<int32_t *>(qd + AP_BF_QB * Q.dim);  // QB x QCAP
    float *qsv = reinterpret_cast<float *>(qsi + AP_BF_QB * AP_BF_QCAP);
    int32_t *qti = reinterpret_cast<int32_t *>(qsv + AP_BF_QB * AP_BF_QCAP);
    float *qtv = reinterpret_cast<float *>(qti + AP_BF_QB * AP_BF_QCAP);
    __shared__ ApLists lists[AP_BF_QB];
    __shared__ float wq[AP_BF_QB][3];
    const int32_t qb = q0 + blockIdx.y * AP_BF_QB;
    const int32_t nq_here = (q0 + nqb - qb) < AP_BF_QB ? (q0 + nqb - qb) : AP_BF_QB;
    for (int i = threadIdx.x; i < nq_here * Q.dim; i += blockDim.x)
        qd[i] = static_cast<const float *>(Q.dense)[(int64_t)qb * Q.dim + i];
    for (int x = 0; x < nq_here; x++) {
        const ApLists a = ap_stage_lists(Q, qb + x, qsi + x * AP_BF_QCAP, qsv + x * AP_BF_QCAP, qti + x * AP_BF_QCAP,
                                         qtv + x * AP_BF_QCAP, AP_BF_QCAP);
        if (threadIdx.x == 0) {
            lists[x] = a;
            wq[x][0] = w[(int64_t)(qb + x) * w_stride + 0];
            wq[x][1] = w[(int64_t)(qb + x) * w_stride + 1];
            wq[x][2] = w[(int64_t)(qb + x) * w_stride + 2];
        }
    }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int64_t wave = blockIdx.x * 4 + ap_wave_id();
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t j = wave; j < D.n; j += nwaves) {
        float dr[NV * EPC];
        ap_load_aside<DT, NV, DT>(D.dense, j, D.dim, dr);
        const int64_t sb = D.sp_indptr[j], se = D.sp_indptr[j + 1], tb = D.tx_indptr[j], te = D.tx_indptr[j + 1];
        for (int x = 0; x < nq_here; x++) {
            float pd = 0.f;
#pragma unroll
            for (int i = 0; i < NV; i++) {
                const int col = (i * 64 + lane) * EPC;
                if (col < D.dim) {
#pragma unroll
                    for (int e = 0; e < EPC; e++) pd = fmaf(qd[x * Q.dim + col + e], dr[i * EPC + e], pd);
                }
            }
            const ApLists a = lists[x];
            const float ps = ap_sparse_partial(a.sp_idx, a.sp_val, a.sp_n, D.sp_idx, D.sp_val, sb, se, lane);
            const float pf = ap_sparse_partial(a.tx_idx, a.tx_val, a.tx_n, D.tx_idx, D.tx_val, tb, te, lane);
            const float sd = ap_wave_sum(pd), ss = ap_wave_sum(ps), sf = ap_wave_sum(pf);
            if (lane == 0) scores[(int64_t)(qb - q0 + x) * D.n + j] = ap_fuse(wq[x][0], wq[x][1], wq[x][2], sd, ss, sf);
        }
    }
}

// k rounds of block-wide arg-max: round r finds the best key that ranks after
// the winner of round r-1.
__global__ __launch_bounds__(256) void k_bf_topk(const float *__restrict__ scores, int64_t n, int32_t k,
                                                 int32_t *__restrict__ out_ids, float *__restrict__ out_scores) {
    __shared__ uint64_t red[4];
    __shared__ uint64_t prev_s;
    const float *row = scores + (int64_t)blockIdx.x * n;
    uint64_t prev = ~0ull;
    for (int32_t r = 0; r < k; r++) {
        uint64_t best = 0;
        for (int64_t j = threadIdx.x; j < n; j += blockDim.x) {
            const uint64_t key = ap_make_key(row[j], (int32_t)j, 1);
            if (key < prev && key > best) best = key;
        }
        for (int o = 32; o > 0; o >>= 1) {
            const uint64_t other = __shfl_xor(best, o, 64);
            best = other > best ? other : best;
        }
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = best;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint64_t b = red[0];
            for (int i = 1; i < 4; i++) b = red[i] > b ? red[i] : b;
            prev_s = b;
            out_ids[(int64_t)blockIdx.x * k + r] = b ? ap_key_id(b) : -1;
            out_scores[(int64_t)blockIdx.x * k + r] = b ? ap_key_score(b) : -INFINITY;
        }
        __syncthreads();
        prev = prev_s;  // 0 when nothing is left: later rounds find nothing either
    }
}

extern "C" int ap_bruteforce_topk(const ap_index *ix, const ap_queries *q, const float *per_query_w, int32_t k,
                                  int32_t *out_ids, float *out_scores, void *stream) {
    AP_REQUIRE(ix && out_ids && out_scores, "NULL argument");
    AP_TRY(ap_validate_queries(q));
    AP_REQUIRE(k >= 1, "k must be positive");
    if (q->nq == 0) return AP_OK;
    hipStream_t st = (hipStream_t)stream;
    const ApVecs Q = query_view(q, ix->docs.dim);
    const int64_t n = ix->docs.n;
    const float *w = per_query_w ? per_query_w : ix->w_dev;
    const int32_t ws = per_query_w ? 3 : 0;
    // queries are processed in slabs so that the score scratch stays <= 2 GiB
    int64_t slab = (int64_t)(1ull << 29) / n;
    slab = slab / AP_BF_QB * AP_BF_QB;
    if (slab < AP_BF_QB) slab = AP_BF_QB;
    if (slab > q->nq) slab = (q->nq + AP_BF_QB - 1) / AP_BF_QB * AP_BF_QB;
    float *scratch = nullptr;
    AP_TRY(ap_dev_alloc(&scratch, (size_t)slab * (size_t)n));
    const size_t smem = (size_t)AP_BF_QB * ((size_t)ix->docs.dim + 4 * AP_BF_QCAP) * 4;
    int rc = AP_OK;
    hipError_t e = hipSuccess;
    for (int32_t q0 = 0; q0 < q->nq && e == hipSuccess; q0 += (int32_t)slab) {
        const int32_t nqb = (q->nq - q0) < slab ? (q->nq - q0) : (int32_t)slab;
        int64_t xb = (n + 3) / 4;
        if (xb > 256) xb = 256;
        dim3 grid((unsigned)xb, (unsigned)((nqb + AP_BF_QB - 1) / AP_BF_QB));
        AP_DISPATCH_DENSE(ix->dtype, ix->docs.dim, {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_bf_scores<DT, NV>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e == hipSuccess)
                hipLaunchKernelGGL((k_bf_scores<DT, NV>), grid, dim3(256), smem, st, Q, ix->docs, q0, nqb, w, ws, scratch);
        });
        if (e == hipSuccess) e = hipGetLastError();
        if (e != hipSuccess) break;
        hipLaunchKernelGGL(k_bf_topk, dim3((unsigned)nqb), dim3(256), 0, st, scratch, n, k, out_ids + (int64_t)q0 * k,
                           out_scores + (int64_t)q0 * k);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(scratch);
    if (e != hipSuccess) { ap_set_error("ap_bruteforce_topk failed: %s", hipGetErrorString(e)); rc = AP_EHIP; }
    return rc;
}
