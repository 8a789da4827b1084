// S7-S9: batched best-first search (Algorithm 2 without its entity branches),
// one workgroup per query.  The KW instantiation adds the keyword branches of
// Section 4.2.2: keyword edges of parents that satisfy the query's keyword
// constraint, a secondary pool of satisfying documents the pool did not keep,
// and the final filter.
//
// Per query, in LDS: the candidate pool (one sorted array of 64-bit keys that
// plays both `cand` and `topk` of Algorithm 2; bit 0 of a key = "not yet
// expanded"), the descriptors and keys of the neighbours scored in this
// iteration, and the query's two sparse lists as look-up tables.  The query's
// dense slice stays in registers.  The visited set is an exact bitset (one bit
// per document): in LDS for small pools on small corpora, else in a global
// workspace of bounded size (large batches run in slabs of queries).
#include <stdlib.h>
#include <algorithm>
#include <mutex>
#include "ap_common.hpp"


int ap_validate_queries(const ap_queries *q);

// The visited set of a query: one bit per document, in LDS when the corpus is small enough for that not to cost a
// workgroup its place on the CU (ap_search_launch decides), else in a per-call global workspace.  Marks document v and
// tells whether it had been marked before.  Only the workgroup that searches the query ever touches its set, so the
// global atomic needs workgroup scope only.
#ifndef AP_VIS_SCOPE
#define AP_VIS_SCOPE __HIP_MEMORY_SCOPE_WORKGROUP
#endif
struct ApVisited {
    uint32_t *g;             // global bitset of this query
    AP_LDS uint32_t *l;      // LDS bitset, or null
    __device__ __forceinline__ bool test_and_set(int32_t v) const {
        const uint32_t bit = 1u << (v & 31);
        uint32_t old;
        if (l) old = __hip_atomic_fetch_or(l + (v >> 5), bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);   // uniform branch
        else old = __hip_atomic_fetch_or(g + (v >> 5), bit, __ATOMIC_RELAXED, AP_VIS_SCOPE);
        return (old & bit) != 0u;
    }
};

struct ApSearchArgs {
    ApVecs D, Q;
    const int32_t *graph;
    const int32_t *entry;
    const float *w;     // per query (stride 3) or the index default (stride 0)
    int32_t w_stride;
    int32_t R, E, k, L, max_iters, width, cmax;
    int32_t vis_lds;    // the visited sets live in LDS (words words after the kernel's other arrays), not in `visited`
    int32_t nxtw;       // words of the scratch that parks positions when more keys enter at once than the workgroup has threads (else 0)
    int32_t q0;         // the launch covers queries q0 .. q0 + gridDim.x (a slab of the batch)
    int32_t no_tables;  // debug: search the query's lists where they lie even when they fit the LDS tables
    uint32_t *visited;  // one bitset per query of the slab
    size_t words;       // visited words per query
    int32_t *out_ids;
    float *out_scores;
    int32_t *counts;    // nq x 3: candidates scored, iterations, candidates whose dense row was skipped (NULL: not wanted)
    const uint2 *rec;   // packed (term, weight) records of the documents' two sparse parts
    const uint4 *meta;  // per document: first entry, counts, |d_dense|
    const uint32_t *deleted;   // one bit per document, NULL = nothing is mark-deleted: left out of the answers only
    // keyword-constrained search only
    const int32_t *kw_edges;   // n x KR keyword edges, kw_count[u] of them valid
    const int32_t *kw_count;
    const int32_t *kw_terms;   // nq x kw_stride required terms, -1 = unused slot
    int32_t KR, kw_stride, kw_all, kw_use_edges;
};

// Pool keys.  Plain search: ap_make_key (30-bit id, bit 0 = "not yet expanded").
// Keyword search: 29-bit id, bit 0 as before, bit 1 = "satisfies the keyword
// constraint".  Ids are unique within a pool, so the flag bits never decide an order.
#define AP_KW_MAX_TERMS 16
template <bool KW> __device__ __forceinline__ uint64_t ap_pool_key(float s, int32_t id, uint32_t flags) {
    if (KW) return ((uint64_t)ap_f2ord(s) << 32) | (uint64_t)(((0x1fffffffu - (uint32_t)id) << 2) | flags);
    return ap_make_key(s, id, flags);
}
template <bool KW> __device__ __forceinline__ int32_t ap_pool_id(uint64_t k) {
    if (KW) return (int32_t)(0x1fffffffu - (((uint32_t)k) >> 2));
    return ap_key_id(k);
}

// Number of entries of the descending array keys[0..n) that rank before `key`.
__device__ __forceinline__ int32_t ap_rank_in(const uint64_t *keys, int32_t n, uint64_t key) {
    int32_t lo = 0, hi = n;
    while (lo < hi) {
        const int32_t mid = (lo + hi) >> 1;
        if (keys[mid] > key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Scores the c candidates of this iteration; wave w of the workgroup's NW takes candidates w, w+NW, ...
// The sparse and lexical parts (the short segments) are evaluated first.  When
// the pool is full and even the largest dense part the norms allow,
// |w_d| |q_d| |d_d|, could not lift the candidate past the pool's last entry,
// the dense row is not read at all: the candidate could not have entered the
// pool, so the result of the search is unchanged (it still counts as visited).
// TAB: the query's lists are look-up tables in LDS (the usual case); otherwise
// they are searched where they lie in global memory.
// Returns the number of candidates whose dense row was skipped (wave-uniform).
// Sizes of the query's two look-up tables (at most a quarter full).  Ordinary queries: 256 + 128 slots (lists up to
// 64 / 32 entries).  Queries that are documents (insertion): 1024 + 512 slots (lists up to 256 / 128 entries).  Both are
// bucketed: two slots a bucket, a hash multiplier per table under which no bucket needs a third.
template <bool BIG> struct ApQTab {
    static constexpr int SPB = BIG ? 10 : 8;
    static constexpr int TXB = BIG ? 9 : 7;
    static constexpr int SLOTS = (1 << SPB) + (1 << TXB);
};

// KW: each candidate's lexical terms are also compared with the query's required
// terms (s_kw[0..n_kw)); the key of a candidate that satisfies the constraint
// carries the "satisfies" flag, and its dense row may only be skipped when the
// bound also rules out the secondary pool (full, and its last score above the bound).
// G: candidates a wave keeps on their way at once.  Their records are loaded together, then reduced one by one;
// then the dense rows of those that still need one are loaded together and multiplied one by one.  G = 1 is the
// plain order (record, sums, dense row); larger G trades registers for memory requests in flight, which pays where
// a large pool leaves a CU with few waves.  The order of the additions inside a candidate does not depend on G.
template <int DT, int NV, bool TAB, bool KW, bool BIG, int NW, int G>
__device__ __forceinline__ int32_t ap_score_candidates(const ApVecs &D, const uint2 *rec, const float *qa, const uint64_t *qtab,
                                                       const ApLists &a, float wd, float ws, float wf, float qnorm, bool pool_full,
                                                       float worst_score, const uint4 *s_meta, int32_t c,
                                                       uint64_t *newk, const int32_t *s_kw, int32_t n_kw, bool kw_all,
                                                       bool second_full, float second_worst, uint32_t msp, uint32_t mtx) {
    const int lane = threadIdx.x & 63, wave = ap_wave_id();
    int32_t skipped = 0;
    for (int32_t i0 = wave; i0 < c; i0 += NW * G) {
        uint2 xs[G][2], xt[G][1];
        const uint2 *r[G];
        int32_t spn[G], txn[G], v[G];
        float dn[G];
#pragma unroll
        for (int gi = 0; gi < G; gi++) {
            const int32_t i = i0 + NW * gi;
            if (i < c) {
                const uint4 m = s_meta[i];
                // the descriptor is the same in every lane: keep the record's address in scalar registers
                r[gi] = rec + ap_uniform_u32(m.x);
                spn[gi] = __builtin_amdgcn_readfirstlane((int32_t)(m.y & 0xffffu));
                txn[gi] = __builtin_amdgcn_readfirstlane((int32_t)(m.y >> 16));
                dn[gi] = __uint_as_float(ap_uniform_u32(m.z));
                v[gi] = (int32_t)ap_uniform_u32(m.w);
                ap_rec_load_raw<2, 1>(r[gi], spn[gi], txn[gi], xs[gi], xt[gi]);
            }
        }
        float ss[G], sf[G];
        uint32_t flags[G];
        bool need[G];      // uniform: the candidate's dense row has to be read
#pragma unroll
        for (int gi = 0; gi < G; gi++) {
            const int32_t i = i0 + NW * gi;
            need[gi] = false;
            if (i >= c) continue;
            int32_t si[2], ti[1];
            float sv[2], tv[1];
            ap_rec_decode<2, 1>(xs[gi], xt[gi], spn[gi], txn[gi], si, sv, ti, tv);
            if (TAB)   // bucketed tables, one read per look-up
                ap_rec_reduce_bucket<2, 1, ApQTab<BIG>::SPB, ApQTab<BIG>::TXB>(r[gi], (const AP_LDS uint64_t *)qtab,
                                                                               (const AP_LDS uint64_t *)(qtab + (1 << ApQTab<BIG>::SPB)),
                                                                               msp, mtx, spn[gi], txn[gi], si, sv, ti, tv, ss[gi], sf[gi]);
            else
                ap_rec_reduce_lists<2, 1>(r[gi], a, spn[gi], txn[gi], si, sv, ti, tv, ss[gi], sf[gi]);
            // upper bound of the fused score, with slack far above fp32 rounding
            const float dmax = fabsf(wd) * qnorm * dn[gi] * 1.0001f;
            const float part = fmaf(wf, sf[gi], ws * ss[gi]);
            const float ub = part + dmax + 1e-5f * (fabsf(ws * ss[gi]) + fabsf(wf * sf[gi]) + dmax);
            flags[gi] = 1u;
            if (KW && n_kw > 0) {
                uint32_t hit = 0;   // bit j: required term j occurs in the candidate's text
                for (int32_t e0 = 0; e0 < txn[gi]; e0 += 64) {
                    int32_t term = ti[0];
                    if (e0 > 0) term = e0 + lane < txn[gi] ? (int32_t)r[gi][spn[gi] + e0 + lane].x : -1;
                    for (int32_t j = 0; j < n_kw; j++) hit |= __ballot(term == s_kw[j]) != 0ull ? 1u << j : 0u;
                }
                const bool sat = kw_all ? hit == (1u << n_kw) - 1u : hit != 0u;
                flags[gi] |= sat ? 2u : 0u;
            }
            if (pool_full && ub < worst_score && (!(flags[gi] & 2u) || (second_full && ub < second_worst))) {
                if (lane == 0) newk[i] = (uint64_t)(uint32_t)(i + 1);   // ranks after every real key (score bits 0), distinct per candidate
                skipped++;
            } else {
                need[gi] = true;
            }
        }
        uint4 raw[G][NV];
#pragma unroll
        for (int gi = 0; gi < G; gi++)
            if (need[gi]) ap_dense_load_raw<DT, NV>(D, v[gi], raw[gi]);
#pragma unroll
        for (int gi = 0; gi < G; gi++) {
            if (need[gi]) {
                const float sd = ap_dense_dot_raw<DT, NV>(D, qa, raw[gi]);
                if (lane == 0) newk[i0 + NW * gi] = ap_pool_key<KW>(ap_fuse(wd, ws, wf, sd, ss[gi], sf[gi]), v[gi], flags[gi]);
            }
        }
    }
    return skipped;
}

// Candidates a wave keeps in flight (ap_score_candidates' G), by workgroup size, as measured on a million-document
// shape: a second candidate costs some 35 registers, which the four- and eight-wave workgroups that share a CU cannot
// spare (one is fastest there: other waves hide the latency); sixteen waves alone on a CU gain 6 % from a second one
// and nothing from a third.
#ifndef AP_SEARCH_G_256
#define AP_SEARCH_G_256 1
#endif
#ifndef AP_SEARCH_G_512
#define AP_SEARCH_G_512 1
#endif
#ifndef AP_SEARCH_G_1024
#define AP_SEARCH_G_1024 2
#endif
#ifndef AP_RANK_LANES
#define AP_RANK_LANES 16        // lanes that rank one entering key of a large pool (16, 32 or 64)
#endif
#ifndef AP_SEARCH_WAVES_512
#define AP_SEARCH_WAVES_512 6
#endif
template <int NT> struct ApSearchG { static constexpr int G = NT == 1024 ? AP_SEARCH_G_1024 : NT == 512 ? AP_SEARCH_G_512 : AP_SEARCH_G_256; };

// Profiling aid of debug builds (-DAP_SEARCH_PROFILE): thread 0 of every workgroup adds the time it spent in each
// phase of the loop (100 MHz ticks) to a device array that ap_debug_search_profile reads and clears.
#ifdef AP_SEARCH_PROFILE
__device__ unsigned long long g_search_prof[8];
#define AP_PROF_DECL unsigned long long prof_t = wall_clock64(), prof_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}
#define AP_PROF(i) do { const unsigned long long now_ = wall_clock64(); prof_acc[i] += now_ - prof_t; prof_t = now_; } while (0)
#define AP_PROF_FLUSH do { if (threadIdx.x == 0) for (int i_ = 0; i_ < 8; i_++) atomicAdd(&g_search_prof[i_], prof_acc[i_]); } while (0)
extern "C" int ap_debug_search_profile(unsigned long long out8[8]) {
    AP_CHECK_HIP(hipMemcpyFromSymbol(out8, HIP_SYMBOL(g_search_prof), sizeof(g_search_prof)));
    unsigned long long z[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    AP_CHECK_HIP(hipMemcpyToSymbol(HIP_SYMBOL(g_search_prof), z, sizeof(z)));
    return AP_OK;
}
#else
#define AP_PROF_DECL
#define AP_PROF(i)
#define AP_PROF_FLUSH
#endif

// NT threads per workgroup.  256 (four waves) is the usual size: seven workgroups share a CU while the pool is small
// enough, and the register budget is the 72 VGPRs of seven waves per SIMD.  When the pool is so large that the LDS
// holds four workgroups or fewer, 512 or 1024 threads keep the CU's SIMDs occupied with one query's candidates.
#ifndef AP_SEARCH_WAVES_PER_SIMD
#define AP_SEARCH_WAVES_PER_SIMD 7
#endif
#ifndef AP_SEARCH_NT512_AT
#define AP_SEARCH_NT512_AT 4    // workgroups of 256 threads a CU's LDS holds at or below which 512 threads are used
#endif
#ifndef AP_SEARCH_NT1024_AT
#define AP_SEARCH_NT1024_AT 1   // ... and 1024 threads
#endif
// Wide bf16 rows (more than 1024 columns: 24 or 32 query values per lane) do not fit seven waves' registers without
// spilling; they run at five waves per SIMD.
template <int DT, int NV, int NT> struct ApSearchWaves {
    static constexpr int MIN = (DT == AP_BF16 && NV >= 3) ? (NT == 1024 ? 4 : 5) : NT == 256 ? AP_SEARCH_WAVES_PER_SIMD : NT == 512 ? AP_SEARCH_WAVES_512 : 4;
};
template <int DT, int NV, bool KW, bool BIG, int NT>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(ApSearchWaves<DT, NV, NT>::MIN, 8)))
void k_search(ApSearchArgs g) {
    extern __shared__ __attribute__((aligned(16))) uint64_t smem64[];   // 16-byte aligned: the descriptors are read as uint4
    // Large pools (workgroups of 512 or 1024 threads): the keys that cannot enter are dropped before sorting, and
    // parents are picked from a bitmap of the unexpanded entries.
    constexpr bool PIPE = !KW && !BIG && NT >= 512;
    constexpr int SPB = ApQTab<BIG>::SPB, TXB = ApQTab<BIG>::TXB;
    // The query's two look-up tables are a static array: at an address the compiler knows, so that a look-up's address
    // is the hash alone.  The dynamic part starts with this iteration's candidates: 16 bytes each, the document's
    // descriptor with its id in the fourth word.
    // PIPE: once the candidates are scored their space is free until the next gather, and holds the entering keys,
    // unordered (xk) and sorted (newS): what lets the largest pool (16384 entries) take sixteen parents' neighbours.
    __shared__ __attribute__((aligned(16))) uint64_t qtab[ApQTab<BIG>::SLOTS];
    uint4 *s_meta = reinterpret_cast<uint4 *>(smem64);
    uint64_t *cur = reinterpret_cast<uint64_t *>(s_meta + g.cmax);   // the pool: L keys, best first
    uint64_t *newk = cur + g.L;              // keys of this iteration's candidates, unordered
    uint64_t *newS = PIPE ? reinterpret_cast<uint64_t *>(s_meta) + g.cmax : newk + g.cmax;   // the same, sorted
    uint64_t *nxt = newk + (PIPE ? 1 : 2) * g.cmax;   // scratch of nxtw words (only wide searches of small pools need it)
    uint64_t *xk = PIPE ? reinterpret_cast<uint64_t *>(s_meta) : nxt + g.nxtw;   // cmax words.  KW: satisfying keys the pool did not keep in this iteration; PIPE: entering keys, unordered
    uint64_t *kwc = nxt + g.nxtw + (KW ? g.cmax : 0);   // KW: the secondary pool, k keys, best first
    uint64_t *umask = kwc + (KW ? g.k : 0);   // PIPE: one bit per pool entry; after it the visited set when it lives in LDS
    __shared__ int32_t s_cnt, s_np, s_skip, s_xn, s_kc, s_nin, s_rmin;
    __shared__ int32_t s_par[16], s_psat[16];
    __shared__ int32_t s_kw[AP_KW_MAX_TERMS];
    __shared__ int32_t s_seed[2];

    const int64_t q = (int64_t)g.q0 + blockIdx.x;
    const int lane = threadIdx.x & 63, wave = ap_wave_id();
    // the query's lists: look-up tables in LDS when they are short (the usual case), else left in global memory
    ApLists a;
    {
        const int64_t sb = g.Q.sp_indptr[q], tb = g.Q.tx_indptr[q];
        a.sp_n = (int32_t)(g.Q.sp_indptr[q + 1] - sb); a.tx_n = (int32_t)(g.Q.tx_indptr[q + 1] - tb);
        a.sp_idx = g.Q.sp_idx + sb; a.sp_val = g.Q.sp_val + sb; a.tx_idx = g.Q.tx_idx + tb; a.tx_val = g.Q.tx_val + tb;
    }
    // Wave 0 builds the two bucketed tables (lists of at most 64 / 32 entries; 256 / 128 for queries that are documents);
    // if no multiplier fits a list, or a list is longer, the lists are searched where they lie.
    bool use_tab = !g.no_tables && a.sp_n <= (1 << SPB) / 4 && a.tx_n <= (1 << TXB) / 4;   // uniform
    uint32_t msp = 0, mtx = 0;
    if (use_tab && wave == 0) {
        const int32_t s0 = ap_bucket_build<BIG ? 4 : 1>(a.sp_idx, a.sp_val, a.sp_n, qtab, SPB);
        const int32_t s1 = ap_bucket_build<BIG ? 2 : 1>(a.tx_idx, a.tx_val, a.tx_n, qtab + (1 << SPB), TXB);
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
    float qnorm;
    {
        float p = 0.f;
#pragma unroll
        for (int i = 0; i < NV * ApDense<DT>::EPC; i++) p = fmaf(qa[i], qa[i], p);
        qnorm = sqrtf(ap_wave_sum(p));
    }
    const float wd = g.w[q * g.w_stride + 0], ws = g.w[q * g.w_stride + 1], wf = g.w[q * g.w_stride + 2];
    ApVisited vis{g.visited + (size_t)blockIdx.x * g.words, nullptr};
    if (g.vis_lds) {   // uniform
        vis.l = (AP_LDS uint32_t *)reinterpret_cast<uint32_t *>(umask + (PIPE ? (g.L + 63) / 64 : 0));
        for (size_t i = threadIdx.x; i < g.words; i += blockDim.x) vis.l[i] = 0u;
    }
    if (threadIdx.x == 0) { s_cnt = 0; s_skip = 0; s_xn = 0; s_kc = 0; s_nin = 0; }
    // the query's required terms, unused slots squeezed out (uniform)
    int32_t n_kw = 0;
    if (KW) {
        for (int32_t j = 0; j < g.kw_stride; j++) {
            const int32_t t = g.kw_terms[q * g.kw_stride + j];
            if (t >= 0) { if (threadIdx.x == 0) s_kw[n_kw] = t; n_kw++; }
        }
    }
    const bool kw_on = KW && n_kw > 0;
    int32_t kc = 0;   // entries in the secondary pool (maintained by wave 0)
    __syncthreads();

    // S7: entry points
    for (int32_t i = threadIdx.x; i < g.E; i += blockDim.x) {
        const int32_t v = g.entry[i];
        if (v >= 0) {
            const bool seen = vis.test_and_set(v);
            const uint4 m = g.meta[v];
            if (!seen) s_meta[atomicAdd(&s_cnt, 1)] = make_uint4(m.x, m.y, m.z, (uint32_t)v);
        }
    }
    __syncthreads();
    int32_t len = 0, it = 0, nscored = 0, nskipped = 0;
    int32_t fu = 0;   // every pool entry before this position has been expanded
    AP_PROF_DECL;
    for (;;) {
        AP_PROF(0);
        const int32_t c = ap_uniform_i32(s_cnt);   // counts and keys that every thread reads alike are kept in scalar registers
        nscored += c;
        const bool pool_full = len == g.L;
        const uint64_t worst = pool_full ? ap_uniform_u64(cur[g.L - 1]) : 0ull;
        const float worst_score = ap_key_score(worst);
        const bool second_full = kw_on && s_kc == g.k;   // s_kc and kwc were last written before the previous barriers
        const float second_worst = second_full ? ap_key_score(kwc[g.k - 1]) : 0.f;
        constexpr int G = ApSearchG<NT>::G;
        if (use_tab)
            nskipped += ap_score_candidates<DT, NV, true, KW, BIG, NT / 64, G>(g.D, g.rec, qa, qtab, a, wd, ws, wf, qnorm, pool_full, worst_score,
                                                                 s_meta, c, newk, s_kw, n_kw, g.kw_all != 0, second_full, second_worst, msp, mtx);
        else
            nskipped += ap_score_candidates<DT, NV, false, KW, BIG, NT / 64, G>(g.D, g.rec, qa, qtab, a, wd, ws, wf, qnorm, pool_full, worst_score,
                                                                  s_meta, c, newk, s_kw, n_kw, g.kw_all != 0, second_full, second_worst, 0u, 0u);
        AP_PROF(1);
        __syncthreads();
        AP_PROF(2);
        if (threadIdx.x == 0) s_cnt = 0;   // every thread has read this iteration's count; the gather counts anew after further barriers
        int32_t cin;
        if (PIPE) {
            // Only keys that rank before the pool's last entry can enter (any key while the pool has room): late in a
            // search they are a small part of the iteration's candidates, so they are picked out first (unordered, in
            // xk) and ranked among themselves afterwards.
            for (int32_t t = threadIdx.x; t < c; t += blockDim.x) {
                const uint64_t key = newk[t];
                if ((key >> 32) != 0ull && key > worst) xk[atomicAdd(&s_nin, 1)] = key;
            }
            __syncthreads();
            cin = ap_uniform_i32(s_nin);
            // A group of AP_RANK_LANES lanes per entering key finds both of its ranks: among the entering keys (a compare
            // per lane and step) and among the pool (as many probes a step as the group has lanes: four steps of 16
            // for 16384 entries instead of fourteen halvings).  The first gives the key its place in newS, the second
            // goes to rr (in newk's space, which is free now).  Late in a search few keys enter, and what costs is the
            // chain of dependent LDS reads per key: four keys share a wave's steps.
            constexpr int GL = AP_RANK_LANES, GSH = GL == 64 ? 6 : GL == 32 ? 5 : 4, GPW = 64 / GL;
            static_assert(GL == 16 || GL == 32 || GL == 64, "lanes per key");
            const int grp = lane >> GSH, gl = lane & (GL - 1);
            auto group_count = [&](bool p) -> int32_t {   // lanes of this lane's group for which p holds
                const uint64_t m = __ballot(p);
                if (GL == 64) return (int32_t)__popcll(m);
                return (int32_t)__popc((uint32_t)(m >> (grp * GL)) & (GL == 32 ? 0xffffffffu : 0xffffu));
            };
            int32_t *rr = reinterpret_cast<int32_t *>(newk);
            for (int32_t j0 = wave * GPW; j0 < cin; j0 += NT / 64 * GPW) {
                const int32_t j = j0 + grp;
                const bool on = j < cin;
                const uint64_t key = on ? xk[j] : 0ull;
                int32_t e = 0;
                for (int32_t i0 = 0; i0 < cin; i0 += GL) e += group_count(on && i0 + gl < cin && xk[i0 + gl] > key);
                int32_t lo = 0, hi = on ? len : 0;   // the rank (number of pool entries that rank before the key) lies in [lo, hi]
                while (__any(hi > lo)) {
                    const int32_t step = (hi - lo + GL - 1) >> GSH;
                    const int32_t at = lo + (gl + 1) * step - 1;
                    const int32_t n_before = group_count(hi > lo && at < hi && cur[at] > key);
                    const int32_t nlo = lo + n_before * step, nhi = lo + (n_before + 1) * step - 1;
                    if (hi > lo) { lo = nlo; hi = nhi < hi ? nhi : hi; }
                }
                if (on && gl == 0) { newS[e] = key; rr[e] = lo; }
            }
            __syncthreads();
            if (threadIdx.x == 0) s_nin = 0;   // next touched after the barriers of the merge or the pick
        } else {
            // sort the new keys by ranking them among themselves; only those that
            // rank before the pool's last entry (when the pool is full) can enter
            for (int32_t t = threadIdx.x; t < c; t += blockDim.x) {
                const uint64_t key = newk[t];
                int32_t r = 0;
                for (int32_t j = 0; j < c; j++) r += newk[j] > key;
                newS[r] = key;
            }
            __syncthreads();
            cin = ap_uniform_i32(ap_rank_in(newS, c, worst));   // new keys that rank before `worst` (all of them while the pool has room)
        }
        AP_PROF(3);
        if (kw_on) {
            // scored, satisfying, but ranked after the full pool's last entry: to the secondary pool
            for (int32_t t = cin + (int32_t)threadIdx.x; t < c; t += blockDim.x) {
                const uint64_t key = newS[t];
                if ((key >> 32) != 0ull && (key & 2ull)) xk[atomicAdd(&s_xn, 1)] = key;
            }
        }
        if (PIPE && cin > 0) {
            // In-place rank merge of a large pool.  The entering keys are few against the pool, so what costs is
            // latency and barriers: the number of entering keys that land before each 64-entry block of the pool is
            // tabulated, after which a pool entry finds how far it moves with two reads; entries from the first
            // insertion point on are read in chunks of 4 NT from the back of the pool to the front and written one
            // barrier later (a chunk's writes never reach below its own start).
            const int32_t *rr = reinterpret_cast<const int32_t *>(newk);   // rank of every entering key among the pool, ascending
            int32_t *bshift = reinterpret_cast<int32_t *>(umask);          // entering keys that land before block b
            const int32_t rmin = ap_uniform_i32(rr[0]);
            fu = fu < rmin ? fu : rmin;   // the best entering key lands at rmin, unexpanded; entries before it stay put
            const int32_t nb = (len + 63) >> 6;
            for (int32_t b = threadIdx.x; b <= nb; b += NT) {   // number of ranks below 64 b
                int32_t lo = 0, hi = cin;
                while (lo < hi) {
                    const int32_t mid = (lo + hi) >> 1;
                    if (rr[mid] < 64 * b) lo = mid + 1; else hi = mid;
                }
                bshift[b] = lo;
            }
            __syncthreads();
            constexpr int CH = 4;
            for (int32_t hi = len; hi > rmin; hi -= CH * NT) {
                const int32_t lo = hi - CH * NT > rmin ? hi - CH * NT : rmin;
                uint64_t held[CH]; int32_t dest[CH];
#pragma unroll
                for (int m = 0; m < CH; m++) {
                    const int32_t t = lo + (int32_t)threadIdx.x + NT * m;
                    dest[m] = g.L;
                    if (t < hi) {
                        held[m] = cur[t];
                        int32_t k = bshift[t >> 6];
                        while (k < cin && rr[k] <= t) k++;   // insertion points inside the entry's own block: rarely any
                        dest[m] = t + k;
                    }
                }
                __syncthreads();
#pragma unroll
                for (int m = 0; m < CH; m++)
                    if (dest[m] < g.L) cur[dest[m]] = held[m];
                // no barrier here: these writes land at or after `lo`, the next chunk's reads come before it
            }
            for (int32_t t = threadIdx.x; t < cin; t += NT) {
                const int32_t r = rr[t] + t;
                if (r < g.L) cur[r] = newS[t];
            }
            len = len + cin < g.L ? len + cin : g.L;
            __syncthreads();
        } else if (cin > 0) {
            // In-place rank merge.  A pool entry at position t moves up by the number of entering keys that rank
            // before it, so only entries from the first insertion point on move, and they only move towards the
            // end: chunks of 2 NT entries are read, then (one barrier later) written, from the back of the pool to the
            // front.  A chunk's writes never reach below its own start, so they need not be fenced from the reads of
            // the chunk before it; the barrier of that chunk orders them before its writes.
            uint64_t nkey = 0; int32_t npos = g.L;
            if ((int32_t)threadIdx.x < cin) { nkey = newS[threadIdx.x]; npos = (int32_t)threadIdx.x + ap_rank_in(cur, len, nkey); }
            if (threadIdx.x == 0) s_rmin = npos;   // where the best entering key lands
            for (int32_t t = (int32_t)threadIdx.x + NT; t < cin; t += NT) {   // more entering keys than threads (wide searches)
                const uint64_t key = newS[t];
                nxt[t] = (uint64_t)(uint32_t)(t + ap_rank_in(cur, len, key));   // park the positions in the scratch array
            }
            __syncthreads();
            const int32_t rmin = ap_uniform_i32(s_rmin);
            fu = fu < rmin ? fu : rmin;   // the best entering key lands at rmin, unexpanded; entries before it stay put
            for (int32_t hi = len; hi > rmin; hi -= 2 * NT) {
                const int32_t lo = hi - 2 * NT > rmin ? hi - 2 * NT : rmin;
                uint64_t held[2]; int32_t dest[2];
#pragma unroll
                for (int m = 0; m < 2; m++) {
                    const int32_t t = lo + (int32_t)threadIdx.x + NT * m;
                    dest[m] = g.L;
                    if (t < hi) { held[m] = cur[t]; dest[m] = t + ap_rank_in(newS, cin, held[m]); }
                }
                __syncthreads();
#pragma unroll
                for (int m = 0; m < 2; m++) {
                    if (dest[m] < g.L) cur[dest[m]] = held[m];
                    else if (kw_on && lo + (int32_t)threadIdx.x + NT * m < hi && (held[m] & 2ull)) xk[atomicAdd(&s_xn, 1)] = held[m];   // evicted
                }
                // no barrier here: these writes land at or after `lo`, the next chunk's reads come before it
            }
            if (npos < g.L) cur[npos] = nkey;
            else if (kw_on && (int32_t)threadIdx.x < cin && (nkey & 2ull)) xk[atomicAdd(&s_xn, 1)] = nkey;
            for (int32_t t = (int32_t)threadIdx.x + NT; t < cin; t += NT) {
                const int32_t r = (int32_t)(uint32_t)nxt[t];
                if (r < g.L) cur[r] = newS[t];
                else if (kw_on && (newS[t] & 2ull)) xk[atomicAdd(&s_xn, 1)] = newS[t];
            }
            len = len + cin < g.L ? len + cin : g.L;
            __syncthreads();
        }
        if (kw_on) {
            // the secondary pool keeps the k best of everything handed over so far (any order of arrival gives the same k)
            __syncthreads();
            if (wave == 0) {
                const int32_t m = s_xn;
                if (g.deleted) {   // a mark-deleted document cannot be an answer: it does not take a place here
                    for (int32_t j = lane; j < m; j += 64) {
                        const int32_t v = ap_pool_id<KW>(xk[j]);
                        if ((g.deleted[v >> 5] >> (v & 31)) & 1u) xk[j] = 0ull;
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                }
                for (int32_t j = 0; j < m; j++) {
                    const uint64_t key = xk[j] & ~1ull;
                    if (key == 0ull || (kc == g.k && key < kwc[kc - 1])) continue;
                    int32_t pos = 0;
                    for (int32_t base = 0; base < kc; base += 64) {
                        const int32_t i = base + lane;
                        pos += __popcll(__ballot(i < kc && kwc[i] > key));
                    }
                    const int32_t last = kc < g.k ? kc : g.k - 1;   // entries [pos, last) move one place towards the end
                    for (int32_t hi = last; hi > pos; hi -= 64) {
                        const int32_t lo = hi - 64 > pos ? hi - 64 : pos;
                        const int32_t i = lo + lane;
                        uint64_t h = 0;
                        if (i < hi) h = kwc[i];
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        if (i < hi) kwc[i + 1] = h;
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                    }
                    if (lane == 0) kwc[pos] = key;
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    kc = kc < g.k ? kc + 1 : g.k;
                }
                if (lane == 0) { s_xn = 0; s_kc = kc; }
            }
        }
        AP_PROF(4);
        if (g.max_iters > 0 && it >= g.max_iters) break;
        // S8: pick the best `width` unexpanded entries (wave 0), mark them expanded
        int32_t pipe_np = 0;
        if (PIPE) {
            // Late in a search the unexpanded entries are few and far apart, and a scan by one wave would walk most of
            // the pool: every wave reduces its share of the pool from the cursor on to one bit per entry, and wave 0
            // picks from the bits.
            const int32_t b0 = fu >> 6, nb = (len + 63) >> 6;
            for (int32_t b = b0 + wave; b < nb; b += NT / 64) {
                const int32_t i = b * 64 + lane;
                const uint64_t m = __ballot(i < len && (cur[i] & 1ull));
                if (lane == 0) umask[b] = m;
            }
            __syncthreads();
            // Every wave picks for itself (the same scalar steps over the same bits, so the same parents): the first
            // `width` set bits are found with uniform steps and lane j takes the j-th.  No barrier is needed between
            // the pick and the gather of the parents' neighbours; wave 0 marks the parents expanded.
            int32_t found = 0, last = -1, mine = -1;
            for (int32_t base = b0; base < nb && found < g.width; base += 64) {
                const int32_t b = base + lane;
                const uint64_t m = b < nb ? umask[b] : 0ull;
                uint64_t nz = __ballot(m != 0ull);
                while (nz != 0ull && found < g.width) {
                    const int32_t src = (int32_t)__builtin_ctzll(nz);
                    nz &= nz - 1ull;
                    uint64_t word = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int32_t)(m >> 32), src) << 32) |
                                    (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int32_t)(uint32_t)m, src);
                    while (word != 0ull && found < g.width) {
                        last = (base + src) * 64 + (int32_t)__builtin_ctzll(word);
                        word &= word - 1ull;
                        if (lane == found) mine = last;
                        found++;
                    }
                }
            }
            if (mine >= 0) {
                const uint64_t key = cur[mine];
                s_par[lane] = ap_pool_id<KW>(key);     // every wave stores the same ids
                if (wave == 0) cur[mine] = key & ~1ull;   // only the flag changes: a wave that reads the entry meanwhile gets the same id
            }
            ap_wave_sync();
            pipe_np = found;
            fu = last >= 0 ? last + 1 : len;   // everything up to the last entry taken is expanded now
        } else if (wave == 0) {
            int32_t found = 0, last = -1;
            for (int32_t base = fu & ~63; base < len && found < g.width; base += 64) {   // the scan starts where it can first succeed
                const int32_t i = base + lane;
                const bool un = i < len && (cur[i] & 1ull);
                const uint64_t mask = __ballot(un);
                const int32_t rank = __popcll(mask & ((1ull << lane) - 1ull));
                const bool take = un && found + rank < g.width;
                if (take) {
                    s_par[found + rank] = ap_pool_id<KW>(cur[i]);
                    if (KW) s_psat[found + rank] = (int32_t)((cur[i] >> 1) & 1ull);
                    cur[i] &= ~1ull;
                }
                const uint64_t tmask = __ballot(take);
                if (tmask) last = base + 63 - (int32_t)__builtin_clzll(tmask);
                found += __popcll(mask);
            }
            fu = last >= 0 ? last + 1 : len;   // everything up to the last entry taken is expanded now
            if (lane == 0) s_np = found < g.width ? found : g.width;
        }
        if (!PIPE) __syncthreads();
        AP_PROF(5);
        const int32_t np = PIPE ? pipe_np : ap_uniform_i32(s_np);
        if (np == 0) break;
        // neighbours of the parents that were never seen before; a parent that satisfies the keyword
        // constraint also brings its keyword edges
        const int32_t per = g.R + (KW ? g.KR : 0);
        for (int32_t i = threadIdx.x; i < np * per; i += blockDim.x) {
            int32_t v;
            if (KW) {
                const int32_t pi = i / per, sl = i % per, u = s_par[pi];
                v = -1;
                if (sl < g.R) v = g.graph[(int64_t)u * g.R + sl];
                else if (g.kw_use_edges && s_psat[pi] && sl - g.R < g.kw_count[u]) v = g.kw_edges[(int64_t)u * g.KR + (sl - g.R)];
            } else {
                v = g.graph[(int64_t)s_par[i / g.R] * g.R + (i % g.R)];
            }
            if (v >= 0) {
                // the descriptor (where the record is, how long, the dense norm) is fetched along with the visited
                // test, not after it: one memory round trip less per iteration for 16 bytes per neighbour already seen
                const bool seen = vis.test_and_set(v);
                const uint4 m = g.meta[v];
                if (!seen) s_meta[atomicAdd(&s_cnt, 1)] = make_uint4(m.x, m.y, m.z, (uint32_t)v);
            }
        }
        __syncthreads();
        AP_PROF(6);
        it++;
    }
    AP_PROF_FLUSH;
    if (lane == 0) atomicAdd(&s_skip, nskipped);
    __syncthreads();
    if (threadIdx.x == 0 && g.counts) { g.counts[q * 3] = nscored; g.counts[q * 3 + 1] = it; g.counts[q * 3 + 2] = s_skip; }
    // S9
    if (kw_on) {
        // Everything in the secondary pool ranked after the pool's last entry when it was handed over, and that
        // entry only ever improves: the satisfying pool entries in order, then the secondary pool, is the merged order.
        if (wave == 0) {
            int32_t o = 0;
            for (int32_t base = 0; base < len && o < g.k; base += 64) {
                const int32_t i = base + lane;
                bool sat = i < len && (cur[i] & 2ull);
                if (sat && g.deleted) { const int32_t v = ap_pool_id<KW>(cur[i]); sat = !((g.deleted[v >> 5] >> (v & 31)) & 1u); }
                const uint64_t mask = __ballot(sat);
                const int32_t at = o + __popcll(mask & ((1ull << lane) - 1ull));
                if (sat && at < g.k) {
                    g.out_ids[q * g.k + at] = ap_pool_id<KW>(cur[i]);
                    g.out_scores[q * g.k + at] = ap_key_score(cur[i]);
                }
                o += __popcll(mask);
            }
            o = o < g.k ? o : g.k;
            for (int32_t i = o + lane; i < g.k; i += 64) {
                const bool have = i - o < kc;
                g.out_ids[q * g.k + i] = have ? ap_pool_id<KW>(kwc[i - o]) : -1;
                g.out_scores[q * g.k + i] = have ? ap_key_score(kwc[i - o]) : -INFINITY;
            }
        }
        return;
    }
    if (KW && g.deleted) {
        // mark-deletion (searches on an index with deletions always run this instantiation): the best k live pool entries
        if (wave == 0) {
            int32_t o = 0;
            for (int32_t base = 0; base < len && o < g.k; base += 64) {
                const int32_t i = base + lane;
                bool live = i < len;
                if (live) { const int32_t v = ap_pool_id<KW>(cur[i]); live = !((g.deleted[v >> 5] >> (v & 31)) & 1u); }
                const uint64_t mask = __ballot(live);
                const int32_t at = o + __popcll(mask & ((1ull << lane) - 1ull));
                if (live && at < g.k) {
                    g.out_ids[q * g.k + at] = ap_pool_id<KW>(cur[i]);
                    g.out_scores[q * g.k + at] = ap_key_score(cur[i]);
                }
                o += __popcll(mask);
            }
            for (int32_t i = (o < g.k ? o : g.k) + lane; i < g.k; i += 64) { g.out_ids[q * g.k + i] = -1; g.out_scores[q * g.k + i] = -INFINITY; }
        }
        return;
    }
    for (int32_t i = threadIdx.x; i < g.k; i += blockDim.x) {
        g.out_ids[q * g.k + i] = i < len ? ap_pool_id<KW>(cur[i]) : -1;
        g.out_scores[q * g.k + i] = i < len ? ap_key_score(cur[i]) : -INFINITY;
    }
}

// Default cap of the index-owned workspace: 2 GiB of visited bits (16,384 queries of a million documents at a time).
#define AP_SEARCH_WS_BYTES ((size_t)2 << 30)

// Queries per slab when `cap_words` words are available: as many as fit, then evened out over the slabs.
static int32_t ap_slab_size(int32_t nq, size_t words, size_t cap_words) {
    size_t fit = std::max<size_t>(1, cap_words / std::max<size_t>(words, 1));
    fit = std::min<size_t>(fit, (size_t)1 << 21);   // a launch of workgroups of up to 1024 threads holds fewer than 2^32 threads
    if (fit >= (size_t)nq) return nq;
    const size_t slabs = ((size_t)nq + fit - 1) / fit;
    return (int32_t)(((size_t)nq + slabs - 1) / slabs);
}

// Sizes the workspace an index owns (grow only) for a call of nq queries.
int ap_search_reserve(ap_index *ix, int32_t nq, hipStream_t st, ApSearchWs *ws) {
    const size_t words = ((size_t)ix->docs.n + 31) / 32;
    const size_t cap_bytes = g_ap_debug.search_workspace_bytes > 0 ? (size_t)g_ap_debug.search_workspace_bytes : AP_SEARCH_WS_BYTES;
    ws->slab = ap_slab_size(nq, words, cap_bytes / 4);
    const size_t need = words * (size_t)ws->slab;
    if (need > ix->visited_words) {
        if (ix->visited) { AP_CHECK_HIP(hipStreamSynchronize(st)); (void)hipFree(ix->visited); ix->visited = nullptr; ix->visited_words = 0; }
        AP_TRY(ap_dev_alloc(&ix->visited, need));
        ix->visited_words = need;
    }
    if ((size_t)nq * 3 > ix->search_counts_cap) {
        if (ix->search_counts) { AP_CHECK_HIP(hipStreamSynchronize(st)); (void)hipFree(ix->search_counts); ix->search_counts = nullptr; ix->search_counts_cap = 0; }
        AP_TRY(ap_dev_alloc(&ix->search_counts, (size_t)nq * 3));
        ix->search_counts_cap = (size_t)nq * 3;
    }
    if (!ix->ev_search[0]) {
        AP_CHECK_HIP(hipEventCreate(&ix->ev_search[0]));
        AP_CHECK_HIP(hipEventCreate(&ix->ev_search[1]));
    }
    ws->visited = ix->visited;
    ws->counts = ix->search_counts;
    ws->ev0 = ix->ev_search[0]; ws->ev1 = ix->ev_search[1];
    ix->last_nq = nq;
    return AP_OK;
}

// The launch itself.  Q: the queries (any view with f32 dense rows); w_dev / w_stride: device weights, one triple
// per query (stride 3) or one for all (stride 0).  kw_terms == NULL: the plain search; otherwise the
// keyword-constrained one.  The queries run in slabs of ws.slab, one launch each, that share the workspace.
// Nothing here allocates: the workspace comes from the caller.
static int ap_search_launch(const ap_index *ix, const ApSearchWs &ws, const ApVecs &Q, const float *w_dev, int32_t w_stride, int32_t k,
                            int32_t beam, int32_t max_iters, int32_t width, const int32_t *kw_terms, int32_t kw_stride,
                            uint32_t kw_flags, bool big_tables, int32_t *out_ids, float *out_scores, hipStream_t st) {
    // The keyword instantiation also serves plain searches on an index with mark-deleted documents (it carries the
    // answer filter; without required terms it searches exactly like the plain one), so that the plain
    // instantiation stays free of both.
    const bool kw = kw_terms != nullptr || ix->deleted != nullptr;
    const int32_t nq = (int32_t)Q.n;
    if (!kw_terms) kw_stride = 0;
    ApSearchArgs g;
    g.D = ix->docs;
    g.Q = Q;
    g.graph = ix->graph;
    g.entry = ix->entry;
    g.w = w_dev;
    g.w_stride = w_stride;
    g.R = ix->params.degree;
    g.E = ix->params.n_entry;
    g.k = k; g.L = beam; g.max_iters = max_iters; g.width = width;
    g.KR = kw_terms ? ix->params.degree / 2 : 0;
    g.kw_edges = ix->kw; g.kw_count = ix->kw_count; g.kw_terms = kw_terms; g.kw_stride = kw_stride;
    g.kw_all = (kw_flags & AP_KW_ALL) ? 1 : 0;
    g.kw_use_edges = (kw_flags & AP_KW_NO_EDGES) ? 0 : 1;
    g.cmax = g.E > g.width * (g.R + g.KR) ? g.E : g.width * (g.R + g.KR);
    g.words = ((size_t)ix->docs.n + 31) / 32;
    g.visited = ws.visited;
    g.out_ids = out_ids;
    g.out_scores = out_scores;
    g.counts = ws.counts;
    g.rec = ix->rec;
    g.meta = ix->meta;
    g.deleted = ix->deleted;
    auto lds_bytes = [&](int32_t nt) {
        const bool pipe = !kw && !big_tables && nt >= 512;   // the large-pool path: entering keys in the candidates' space, a bitmap of the pool
        const int32_t nxtw = !pipe && g.cmax > nt ? g.cmax : 0;
        return (size_t)(g.L + (pipe ? 1 : 2) * g.cmax + nxtw + (kw ? g.cmax + g.k : 0)) * 8 + (size_t)g.cmax * 16 +
               (size_t)(big_tables ? ApQTab<true>::SLOTS : ApQTab<false>::SLOTS) * 8 + (pipe ? (size_t)((g.L + 63) / 64) * 8 : 0);
    };
    // Workgroup size (plain search): four waves as long as the LDS holds at least five workgroups per CU; a pool
    // that leaves room for two to four gets eight waves, one that fills the CU alone sixteen (measured: each is the
    // fastest in its range).
    int32_t nt = 256;
    if (!kw && !big_tables) {
        const size_t per_cu = (size_t)160 * 1024 / lds_bytes(256);
        nt = per_cu > AP_SEARCH_NT512_AT ? 256 : per_cu > AP_SEARCH_NT1024_AT ? 512 : 1024;
    }
    g.nxtw = nt == 256 && g.cmax > nt ? g.cmax : 0;
    size_t smem = lds_bytes(nt);
    // Visited sets in LDS (four-wave workgroups only): when the bitset fits beside the kernel's other arrays without
    // taking a workgroup's place on the CU (seven of them run on one while the pool is small).  Measured on 100,000
    // documents (12.5 KB a set): 4 to 5 % faster up to beam 512, 29 % slower at beam 2144 where it costs two of the
    // seven workgroups, which is why the rule is about occupancy.  Same results either way.
    g.vis_lds = 0;
    if (nt == 256 && g_ap_debug.search_visited_global == 0) {
        const size_t with = smem + g.words * 4 + 8, lds = (size_t)160 * 1024;
        const size_t now = std::min<size_t>(7, lds / smem), then = with <= lds ? std::min<size_t>(7, lds / with) : 0;
        if (then >= now && then > 0) { g.vis_lds = 1; smem = with; }
    }
    // the kernel's static arrays (counters, parents, required terms) take a few hundred bytes more
    AP_REQUIRE(smem + 512 <= 160 * 1024, "beam and search_width need %zu bytes of LDS (limit 160 KiB)", smem + 512);
    const size_t dyn = smem - (size_t)(big_tables ? ApQTab<true>::SLOTS : ApQTab<false>::SLOTS) * 8;   // the tables are a static array
    hipError_t le = hipSuccess;
#define AP_LAUNCH_SEARCH(KWF, BIGF, NTF)                                                                                         \
    AP_DISPATCH_DENSE(ix->dtype, ix->docs.dim, {                                                                                  \
        if (smem > 48 * 1024)                                                                                                     \
            le = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_search<DT, NV, KWF, BIGF, NTF>),                           \
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);                                       \
        if (le == hipSuccess) hipLaunchKernelGGL((k_search<DT, NV, KWF, BIGF, NTF>), dim3((unsigned)qn), dim3(NTF), dyn, st, g);  \
    })
    for (int32_t q0 = 0; q0 < nq; q0 += ws.slab) {
        const int32_t qn = std::min(ws.slab, nq - q0);
        g.q0 = q0;
        g.no_tables = g_ap_debug.search_query_lists != 0;
        // every slab starts from empty visited sets (a fill kernel, not a memset: callers may capture the stream)
        if (!g.vis_lds) AP_TRY(ap_fill_u32(ws.visited, g.words * (size_t)qn, 0u, st));
        if (q0 == 0 && ws.ev0) AP_CHECK_HIP(hipEventRecord(ws.ev0, st));
        if (kw) AP_LAUNCH_SEARCH(true, false, 256);
        else if (big_tables) AP_LAUNCH_SEARCH(false, true, 256);
        else if (nt == 256) AP_LAUNCH_SEARCH(false, false, 256);
        else if (nt == 512) AP_LAUNCH_SEARCH(false, false, 512);
        else AP_LAUNCH_SEARCH(false, false, 1024);
        AP_CHECK_HIP(le);
        AP_CHECK_HIP(hipGetLastError());
    }
#undef AP_LAUNCH_SEARCH
    if (ws.ev1) AP_CHECK_HIP(hipEventRecord(ws.ev1, st));
    return AP_OK;
}

// Argument checks shared by every entry into the search.
static int ap_search_check(const ap_index *ix, int32_t nq, int32_t k, int32_t beam, int32_t max_iters, int32_t width, bool kw,
                           const int32_t *out_ids, const float *out_scores) {
    if (!ix->has_graph) { ap_set_error("index has no graph: build or import one first"); return AP_ESTATE; }
    AP_REQUIRE(nq == 0 || (out_ids && out_scores), "NULL output");
    AP_REQUIRE(beam >= 1 && beam <= AP_MAX_BEAM, "beam = %d must be in [1, %d]", beam, AP_MAX_BEAM);
    AP_REQUIRE(k >= 1 && k <= beam, "k = %d must be in [1, beam]", k);
    AP_REQUIRE(width >= 1 && width <= 16, "search_width = %d must be in [1, 16]", width);
    AP_REQUIRE(max_iters >= 0, "max_iters must be >= 0");
    AP_REQUIRE(!(kw || ix->deleted) || ix->docs.n < (1ll << 29), "keyword search and searches on an index with deletions need n < 2^29");
    return AP_OK;
}

int ap_search_core(ap_index *ix, const ApVecs &Q, const float *w_dev, int32_t w_stride, int32_t k, int32_t beam, int32_t max_iters,
                   int32_t width, bool big_tables, int32_t *out_ids, float *out_scores, hipStream_t st) {
    AP_TRY(ap_search_check(ix, (int32_t)Q.n, k, beam, max_iters, width, false, out_ids, out_scores));
    if (Q.n == 0) return AP_OK;
    ApSearchWs ws;
    AP_TRY(ap_search_reserve(ix, (int32_t)Q.n, st, &ws));
    return ap_search_launch(ix, ws, Q, w_dev, w_stride, k, beam, max_iters, width, nullptr, 0, 0u, big_tables, out_ids, out_scores, st);
}

static int ap_search_impl(ap_index *ix, const ap_queries *q, const float *per_query_w, const ap_search_params *p,
                          const int32_t *kw_terms, int32_t kw_stride, uint32_t kw_flags, int32_t *out_ids, float *out_scores,
                          void *stream) {
    AP_REQUIRE(ix && p, "NULL argument");
    AP_TRY(ap_validate_queries(q));
    AP_TRY(ap_search_check(ix, q->nq, p->k, p->beam, p->max_iters, p->search_width, kw_terms != nullptr, out_ids, out_scores));
    if (q->nq == 0) return AP_OK;
    const ApVecs Q{q->nq, ix->docs.dim, q->dense, q->sp_indptr, q->sp_idx, q->sp_val, q->tx_indptr, q->tx_idx, q->tx_cnt};
    ApSearchWs ws;
    AP_TRY(ap_search_reserve(ix, q->nq, (hipStream_t)stream, &ws));
    return ap_search_launch(ix, ws, Q, per_query_w ? per_query_w : ix->w_dev, per_query_w ? 3 : 0, p->k, p->beam, p->max_iters,
                            p->search_width, kw_terms, kw_stride, kw_flags, false, out_ids, out_scores, (hipStream_t)stream);
}

extern "C" int ap_search_batch(ap_index *ix, const ap_queries *q, const float *per_query_w,
                               const ap_search_params *p, int32_t *out_ids, float *out_scores, void *stream) {
    return ap_search_impl(ix, q, per_query_w, p, nullptr, 0, 0u, out_ids, out_scores, stream);
}

// ---- the search for callers that cannot allocate ---------------------------------------------------------------
// The visited sets live in a file-scope device array instead of an index-owned allocation.  Each GPU holds its own
// copy of the array at its own address; host code uses the address hipGetSymbolAddress returns for the current
// device, never the array's name (which is only a host-side stand-in).
static __device__ __align__(256) unsigned char scratch[AP_NOALLOC_WORKSPACE_BYTES];

#define AP_MAX_DEVICES 64
static std::mutex g_scratch_lock;
static void *g_scratch_ptr[AP_MAX_DEVICES];   // per device, filled on first use

// The address of `scratch` on the current device (looked up once per device).
int ap_static_scratch(void **out) {
    int dev = -1;
    AP_CHECK_HIP(hipGetDevice(&dev));
    AP_REQUIRE(dev >= 0 && dev < AP_MAX_DEVICES, "device %d is beyond the %d devices this library keeps a workspace for", dev, AP_MAX_DEVICES);
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        AP_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        AP_REQUIRE(p != nullptr, "the static search workspace has no address on device %d", dev);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return AP_OK;
}

extern "C" int ap_search_batch_noalloc(const ap_index *ix, const ap_queries *q, const float *per_query_w,
                                       const ap_search_params *p, int32_t *out_ids, float *out_scores, void *stream) {
    AP_REQUIRE(ix && p, "NULL argument");
    AP_TRY(ap_validate_queries(q));
    AP_TRY(ap_search_check(ix, q->nq, p->k, p->beam, p->max_iters, p->search_width, false, out_ids, out_scores));
    const size_t words = ((size_t)ix->docs.n + 31) / 32;
    // the debug setting that caps the index-owned workspace caps this one too (never beyond the array)
    const size_t cap = g_ap_debug.search_workspace_bytes > 0 ? std::min<size_t>((size_t)g_ap_debug.search_workspace_bytes, AP_NOALLOC_WORKSPACE_BYTES)
                                                             : AP_NOALLOC_WORKSPACE_BYTES;
    AP_REQUIRE(words * 4 <= cap,
               "the corpus has %lld documents: one visited bit per document does not fit the static workspace of %zu bytes "
               "(at most %zu documents); use ap_search_batch",
               (long long)ix->docs.n, cap, cap * 8);
    if (q->nq == 0) return AP_OK;
    void *base = nullptr;
    AP_TRY(ap_static_scratch(&base));
    ApSearchWs ws;                       // no counters, no events: nothing of the index is written
    ws.visited = static_cast<uint32_t *>(base);
    ws.slab = ap_slab_size(q->nq, words, cap / 4);
    const ApVecs Q{q->nq, ix->docs.dim, q->dense, q->sp_indptr, q->sp_idx, q->sp_val, q->tx_indptr, q->tx_idx, q->tx_cnt};
    return ap_search_launch(ix, ws, Q, per_query_w ? per_query_w : ix->w_dev, per_query_w ? 3 : 0, p->k, p->beam, p->max_iters,
                            p->search_width, nullptr, 0, 0u, false, out_ids, out_scores, (hipStream_t)stream);
}

extern "C" int ap_search_batch_keywords(ap_index *ix, const ap_queries *q, const float *per_query_w,
                                        const ap_search_params *p, const int32_t *kw_terms, int32_t kw_stride,
                                        uint32_t kw_flags, int32_t *out_ids, float *out_scores, void *stream) {
    AP_REQUIRE(ix && q, "NULL argument");
    AP_REQUIRE(kw_stride >= 1 && kw_stride <= AP_KW_MAX_TERMS, "kw_stride = %d must be in [1, %d]", kw_stride, AP_KW_MAX_TERMS);
    AP_REQUIRE(kw_terms || q->nq == 0, "kw_terms is NULL");
    AP_REQUIRE((kw_flags & ~(uint32_t)(AP_KW_ALL | AP_KW_NO_EDGES)) == 0, "unknown bits in kw_flags");
    if (!ix->has_graph) { ap_set_error("index has no graph: build or import one first"); return AP_ESTATE; }
    AP_REQUIRE(ix->kw && ix->kw_count, "index has no keyword edges");
    AP_REQUIRE(ix->docs.n < (1ll << 29), "keyword search needs n < 2^29");
    if (q->nq == 0) return ap_search_impl(ix, q, per_query_w, p, nullptr, 0, 0u, out_ids, out_scores, stream);
    return ap_search_impl(ix, q, per_query_w, p, kw_terms, kw_stride, kw_flags, out_ids, out_scores, stream);
}

extern "C" int ap_search_stats(const ap_index *ix, int32_t *out_counts, int32_t nq, float *kernel_ms, void *stream) {
    AP_REQUIRE(ix, "index is NULL");
    if (!ix->ev_search[1] || ix->last_nq == 0) { ap_set_error("no search has run on this index"); return AP_ESTATE; }
    AP_CHECK_HIP(hipEventSynchronize(ix->ev_search[1]));
    if (kernel_ms) AP_CHECK_HIP(hipEventElapsedTime(kernel_ms, ix->ev_search[0], ix->ev_search[1]));
    if (out_counts) {
        AP_REQUIRE(nq == ix->last_nq, "nq = %d does not match the last search (%d)", nq, ix->last_nq);
        AP_CHECK_HIP(hipMemcpyAsync(out_counts, ix->search_counts, (size_t)nq * 3 * sizeof(int32_t), hipMemcpyDeviceToDevice,
                                    (hipStream_t)stream));
    }
    return AP_OK;
}
