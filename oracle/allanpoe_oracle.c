/*
 * CPU oracle for the Allan-Poe hybrid-index hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, single-threaded, fp64-accumulating C that
 * writes out what the paper defines, one step at a time, so that a reader can
 * check each function against the cited passage by eye.  Nothing here is
 * blocked, fused, vectorised or reordered.  It shares no code with the HIP
 * path and the product never calls it: only tests, the smoke check and the
 * benchmark's CPU-baseline leg do.
 *
 * Conventions
 *   - "score" is a similarity (higher is better); the paper's dis is -score.
 *   - Every ranking uses the total order (score descending, id ascending).
 *   - Scores are accumulated in double and rounded to float once, when stored.
 *   - A vector set (documents or queries) = dense rows + learned-sparse CSR +
 *     lexical CSR; ids inside a CSR row are strictly ascending.
 *   - id -1 marks an empty slot in any neighbour list; its score is -INFINITY.
 *
 * Pins (see tests): BM25 hand-worked example, dense expansion of the sparse
 * inner product, Theorem 1 identity, brute-force top-k, independent detour
 * recount, IP-prune invariant, keyword-flag set evaluation, structural
 * invariants of the assembled graph, exhaustive-beam search == brute force.
 * Parity unpinned: the free parameters the paper does not fix (K, T, S, E, the
 * keyword-edge cap, the split of the single-path half of an edge list) are
 * choices, not results; they are only measured (graph recall, search recall).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int64_t n;
    int32_t dim;
    const float *dense;          /* n x dim, row-major */
    const int64_t *sp_indptr;    /* n+1 */
    const int32_t *sp_idx;
    const float *sp_val;
    const int64_t *tx_indptr;    /* n+1 */
    const int32_t *tx_idx;
    const float *tx_val;         /* documents: BM25 weights; queries: term counts */
} orc_vecset;

/* ------------------------------------------------------------------ */
/* total order helpers                                                 */

/* 1 if (sa, ia) ranks strictly before (sb, ib): score desc, id asc. */
static int ranks_before(float sa, int32_t ia, float sb, int32_t ib) {
    if (sa > sb) return 1;
    if (sa < sb) return 0;
    return ia < ib;
}

typedef struct { float s; int32_t id; } scored;

static int cmp_scored(const void *pa, const void *pb) {
    const scored *a = (const scored *)pa, *b = (const scored *)pb;
    if (ranks_before(a->s, a->id, b->s, b->id)) return -1;
    if (ranks_before(b->s, b->id, a->s, a->id)) return 1;
    return 0;
}

static int cmp_i32(const void *pa, const void *pb) {
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

/* ------------------------------------------------------------------ */
/* S0: lexical encoding (Section 3.2: full text becomes a lexical sparse
 * vector whose entries are BM25 term importances).  The paper names BM25 but
 * prints no formula; this is the Robertson/Lucene form with the non-negative
 * IDF, the whole document-side factor stored in the document vector and the
 * raw term count left on the query side:
 *   w(d,t) = IDF(t) * tf * (k1+1) / (tf + k1 * (1 - b + b*|d|/avgdl))
 *   IDF(t) = ln(1 + (N - df_t + 0.5) / (df_t + 0.5))
 * |d| = number of tokens of d, avgdl = mean |d|.                        */
int orc_bm25_encode(int64_t n, int32_t vocab, const int64_t *indptr, const int32_t *idx,
                    const float *tf, double k1, double b, float *out_w, int32_t *out_df,
                    double *out_avgdl) {
    int64_t i, e;
    double total = 0.0, avgdl;
    for (i = 0; i < vocab; i++) out_df[i] = 0;
    for (i = 0; i < n; i++)
        for (e = indptr[i]; e < indptr[i + 1]; e++) {
            if (idx[e] < 0 || idx[e] >= vocab) return -1;
            out_df[idx[e]] += 1;
            total += (double)tf[e];
        }
    avgdl = n > 0 ? total / (double)n : 0.0;
    if (out_avgdl) *out_avgdl = avgdl;
    for (i = 0; i < n; i++) {
        double len = 0.0;
        for (e = indptr[i]; e < indptr[i + 1]; e++) len += (double)tf[e];
        for (e = indptr[i]; e < indptr[i + 1]; e++) {
            double df = (double)out_df[idx[e]];
            double idf = log(1.0 + ((double)n - df + 0.5) / (df + 0.5));
            double f = (double)tf[e];
            double denom = f + k1 * (1.0 - b + b * len / avgdl);
            out_w[e] = (float)(idf * f * (k1 + 1.0) / denom);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* S1: hybrid similarity (Definition 1; Theorem 1): three inner products and
 * their weighted sum.                                                   */

static double dense_ip(const float *a, const float *b, int32_t dim) {
    double s = 0.0;
    int32_t c;
    for (c = 0; c < dim; c++) s += (double)a[c] * (double)b[c];
    return s;
}

/* inner product of two sparse vectors given as ascending (id, value) lists */
static double sparse_ip(const int32_t *ia, const float *va, int64_t na,
                        const int32_t *ib, const float *vb, int64_t nb) {
    double s = 0.0;
    int64_t p = 0, q = 0;
    while (p < na && q < nb) {
        if (ia[p] < ib[q]) p++;
        else if (ia[p] > ib[q]) q++;
        else { s += (double)va[p] * (double)vb[q]; p++; q++; }
    }
    return s;
}

double orc_sparse_ip(const int32_t *ia, const float *va, int64_t na,
                     const int32_t *ib, const float *vb, int64_t nb) {
    return sparse_ip(ia, va, na, ib, vb, nb);
}

/* out3 = (sim_d, sim_s, sim_f) in double */
static void hybrid3(const orc_vecset *A, int64_t i, const orc_vecset *B, int64_t j, double out3[3]) {
    out3[0] = dense_ip(A->dense + i * A->dim, B->dense + j * B->dim, A->dim);
    out3[1] = sparse_ip(A->sp_idx + A->sp_indptr[i], A->sp_val + A->sp_indptr[i],
                        A->sp_indptr[i + 1] - A->sp_indptr[i],
                        B->sp_idx + B->sp_indptr[j], B->sp_val + B->sp_indptr[j],
                        B->sp_indptr[j + 1] - B->sp_indptr[j]);
    out3[2] = sparse_ip(A->tx_idx + A->tx_indptr[i], A->tx_val + A->tx_indptr[i],
                        A->tx_indptr[i + 1] - A->tx_indptr[i],
                        B->tx_idx + B->tx_indptr[j], B->tx_val + B->tx_indptr[j],
                        B->tx_indptr[j + 1] - B->tx_indptr[j]);
}

static double fuse(const double s[3], const float w[3]) {
    return (double)w[0] * s[0] + (double)w[1] * s[1] + (double)w[2] * s[2];
}

static float hybrid_fused(const orc_vecset *A, int64_t i, const orc_vecset *B, int64_t j, const float w[3]) {
    double s[3];
    hybrid3(A, i, B, j, s);
    return (float)fuse(s, w);
}

/* For every a in a_ids (na of them) and each of its c candidates in B:
 * out4[(x*c + y)*4 + {0,1,2,3}] = sim_d, sim_s, sim_f, M_w.  w is na x 3.
 * A candidate id of -1 gives four -INFINITY.                           */
void orc_hybrid_block(const orc_vecset *A, int64_t na, const int64_t *a_ids, const orc_vecset *B,
                      int64_t c, const int32_t *cand, const float *w, float *out4) {
    int64_t x, y;
    for (x = 0; x < na; x++)
        for (y = 0; y < c; y++) {
            float *o = out4 + (x * c + y) * 4;
            int32_t j = cand[x * c + y];
            if (j < 0) { o[0] = o[1] = o[2] = o[3] = -INFINITY; continue; }
            double s[3];
            hybrid3(A, a_ids[x], B, j, s);
            o[0] = (float)s[0]; o[1] = (float)s[1]; o[2] = (float)s[2];
            o[3] = (float)fuse(s, w + x * 3);
        }
}

/* Exact top-k of all documents for each query under that query's weights
 * (the maximum-inner-product problem of Theorem 1 solved by enumeration).
 * skip_same != 0 leaves out document i for query i (k-NN among documents).
 * Missing results: id -1, score -INFINITY.                              */
void orc_bruteforce_topk(const orc_vecset *Q, int64_t nq, const int64_t *q_ids, const orc_vecset *D,
                         const float *w, int32_t k, int32_t skip_same, int32_t *out_ids,
                         float *out_scores) {
    int64_t x, j, n = D->n;
    scored *all = (scored *)malloc(sizeof(scored) * (size_t)(n > 0 ? n : 1));
    for (x = 0; x < nq; x++) {
        int64_t cnt = 0, r;
        for (j = 0; j < n; j++) {
            if (skip_same && j == q_ids[x]) continue;
            all[cnt].s = hybrid_fused(Q, q_ids[x], D, j, w + x * 3);
            all[cnt].id = (int32_t)j;
            cnt++;
        }
        qsort(all, (size_t)cnt, sizeof(scored), cmp_scored);
        for (r = 0; r < k; r++) {
            out_ids[x * k + r] = r < cnt ? all[r].id : -1;
            out_scores[x * k + r] = r < cnt ? all[r].s : -INFINITY;
        }
    }
    free(all);
}

/* fused self-similarity M_w(v, v) of every listed document */
void orc_self_sim(const orc_vecset *D, int64_t nn, const int64_t *ids, const float w[3], float *out) {
    int64_t x;
    for (x = 0; x < nn; x++) out[x] = hybrid_fused(D, ids[x], D, ids[x], w);
}

/* ------------------------------------------------------------------ */
/* S2: seed neighbour lists.  Algorithm 1 starts from random lists; this build
 * starts from the exact top-K by dense inner product (v != u), which any
 * number of refinement rounds then improves under the fused metric.      */
void orc_seed_knn(const orc_vecset *D, int64_t nn, const int64_t *node_ids, int32_t K,
                  int32_t *out_ids, float *out_scores) {
    int64_t x, j, n = D->n;
    scored *all = (scored *)malloc(sizeof(scored) * (size_t)(n > 0 ? n : 1));
    for (x = 0; x < nn; x++) {
        int64_t u = node_ids[x], cnt = 0, r;
        for (j = 0; j < n; j++) {
            if (j == u) continue;
            all[cnt].s = (float)dense_ip(D->dense + u * D->dim, D->dense + j * D->dim, D->dim);
            all[cnt].id = (int32_t)j;
            cnt++;
        }
        qsort(all, (size_t)cnt, sizeof(scored), cmp_scored);
        for (r = 0; r < K; r++) {
            out_ids[x * K + r] = r < cnt ? all[r].id : -1;
            out_scores[x * K + r] = r < cnt ? all[r].s : -INFINITY;
        }
    }
    free(all);
}

/* ------------------------------------------------------------------ */
/* S3: one synchronous refinement round (Algorithm 1, the NN-Descent loop:
 * look at the neighbours of u's neighbours and keep the best K).
 *   C(u) = N(u)  U  { N(v)[j] : v in N(u)[0:S], j < S }  \ {u}, duplicates removed
 *   N'(u) = top-K of C(u) under the fused build metric
 * Alongside, three per-path lists of length P keep the best candidates ever
 * scored for u by sim_d, sim_s and sim_f alone (the single-path neighbours
 * of Step 2's last sentence).  sp_* arrays are [3][N][P]; outputs are written
 * for the nn listed nodes only: out_* [nn][K], out_sp_* [3][nn][P].       */
void orc_refine_round(const orc_vecset *D, const float w[3], int32_t K, int32_t S, int32_t P,
                      const int32_t *knn_ids /* N x K */, const int32_t *sp_ids /* 3 x N x P */,
                      const float *sp_sc, int64_t nn, const int64_t *node_ids, int32_t *out_ids,
                      float *out_scores, int32_t *out_sp_ids, float *out_sp_sc) {
    int64_t N = D->n, x;
    int64_t cap = (int64_t)K + (int64_t)S * S;
    int32_t *cand = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap);
    scored *sc = (scored *)malloc(sizeof(scored) * (size_t)(cap + P));
    double *comp = (double *)malloc(sizeof(double) * 3 * (size_t)cap);
    int32_t s_lim = S < K ? S : K;
    for (x = 0; x < nn; x++) {
        int64_t u = node_ids[x], cnt = 0, i, j, m;
        const int32_t *Nu = knn_ids + u * K;
        for (i = 0; i < K; i++) if (Nu[i] >= 0 && Nu[i] != u) cand[cnt++] = Nu[i];
        for (i = 0; i < s_lim; i++) {
            int32_t v = Nu[i];
            if (v < 0) continue;
            for (j = 0; j < s_lim; j++) {
                int32_t t = knn_ids[(int64_t)v * K + j];
                if (t >= 0 && t != u) cand[cnt++] = t;
            }
        }
        qsort(cand, (size_t)cnt, sizeof(int32_t), cmp_i32);
        m = 0;
        for (i = 0; i < cnt; i++) if (i == 0 || cand[i] != cand[i - 1]) cand[m++] = cand[i];
        cnt = m;
        for (i = 0; i < cnt; i++) {
            hybrid3(D, u, D, cand[i], comp + 3 * i);
            sc[i].s = (float)fuse(comp + 3 * i, w);
            sc[i].id = cand[i];
        }
        qsort(sc, (size_t)cnt, sizeof(scored), cmp_scored);
        for (i = 0; i < K; i++) {
            out_ids[x * K + i] = i < cnt ? sc[i].id : -1;
            out_scores[x * K + i] = i < cnt ? sc[i].s : -INFINITY;
        }
        /* per-path lists: previous list U this round's candidates, by that path's similarity */
        for (int p = 0; p < 3; p++) {
            const int32_t *old_i = sp_ids + ((int64_t)p * N + u) * P;
            const float *old_s = sp_sc + ((int64_t)p * N + u) * P;
            int64_t tot = 0;
            for (i = 0; i < cnt; i++) { sc[tot].s = (float)comp[3 * i + p]; sc[tot].id = cand[i]; tot++; }
            for (i = 0; i < P; i++) {
                int dup = 0;
                if (old_i[i] < 0) continue;
                for (j = 0; j < cnt; j++) if (cand[j] == old_i[i]) { dup = 1; break; }
                if (!dup) { sc[tot].s = old_s[i]; sc[tot].id = old_i[i]; tot++; }
            }
            qsort(sc, (size_t)tot, sizeof(scored), cmp_scored);
            for (i = 0; i < P; i++) {
                out_sp_ids[((int64_t)p * nn + x) * P + i] = i < tot ? sc[i].id : -1;
                out_sp_sc[((int64_t)p * nn + x) * P + i] = i < tot ? sc[i].s : -INFINITY;
            }
        }
    }
    free(cand); free(sc); free(comp);
}

/* ------------------------------------------------------------------ */
/* S4: similarities inside one neighbourhood.  Pm[i*K+j] = M_w(ids[i], ids[j]),
 * -INFINITY where either id is -1.  The diagonal holds self-similarities.  */
void orc_pairwise(const orc_vecset *D, const float w[3], int32_t K, const int32_t *ids, float *Pm) {
    int32_t i, j;
    for (i = 0; i < K; i++)
        for (j = 0; j < K; j++)
            Pm[i * K + j] = (ids[i] < 0 || ids[j] < 0) ? -INFINITY : hybrid_fused(D, ids[i], D, ids[j], w);
}

/* S4: detourable routes (Section 3.3, the RNG phase borrowed from the
 * backbone).  With dis = -sim, the two-hop route A -> X -> Y detours the edge
 * A -> Y when max(dis(A,X), dis(X,Y)) < dis(A,Y), i.e.
 *   min(sim(A,X), sim(X,Y)) > sim(A,Y).
 * count[y] = number of such X among the other neighbours.  Then the list is
 * stably sorted by count ascending (Algorithm 1): order[r] = original
 * position of the neighbour that ends up at rank r.  Empty slots (id -1) go
 * last and count 0 routes.                                              */
void orc_detour_sort(int32_t K, const int32_t *ids, const float *simA, const float *Pm,
                     int32_t *count, int32_t *order) {
    int32_t x, y, r, pos = 0, c;
    for (y = 0; y < K; y++) {
        count[y] = 0;
        if (ids[y] < 0) continue;
        for (x = 0; x < K; x++) {
            float a, b, mn;
            if (x == y || ids[x] < 0) continue;
            a = simA[x];
            b = Pm[x * K + y];
            mn = a < b ? a : b;
            if (mn > simA[y]) count[y] += 1;
        }
    }
    for (c = 0; c <= K; c++)
        for (r = 0; r < K; r++)
            if (ids[r] >= 0 && count[r] == c) order[pos++] = r;
    for (r = 0; r < K; r++) if (ids[r] < 0) order[pos++] = r;
}

/* ------------------------------------------------------------------ */
/* S5: inner-product pruning with keyword recycling (Algorithm 1, the loop over
 * v in N(u); Section 3.3 for the keyword rule).
 *
 * Walk the neighbours in detour order.  The first one opens SE.  A later v
 * joins SE when |SE| < R and IP(w, v) < IP(v, v) for every w already in SE;
 * otherwise, if its keyword flag is set (and KE has room), it is recycled
 * into KE.  The flag follows Section 3.3: X may be dropped for good only if
 * some current neighbour Y covers every keyword X shares with A, so
 *   flag(X) = [ K(A) n K(X) != {} ]  and  for every Y in SE now:
 *             K(A) n K(X) is NOT a subset of K(Y).
 * K(.) is the set of term ids of the lexical vector.
 * Positions index the ORIGINAL neighbour array (ids, Pm, self).
 * Ablation of the joint strategy (Section 5, effectiveness of RNG-IP joint
 * pruning): use_ip = 0 drops the IP test, so SE is simply the first R
 * neighbours in detour order ("RNG alone"); "IP alone" is this routine with
 * use_ip = 1 fed the neighbours in their original similarity order.      */
static int contains(const int32_t *a, int64_t n, int32_t t) {
    int64_t i;
    for (i = 0; i < n; i++) if (a[i] == t) return 1;
    return 0;
}

void orc_ip_prune(const orc_vecset *D, int64_t A, int32_t K, int32_t R, int32_t ke_cap,
                  const int32_t *ids, const int32_t *order, const float *Pm, const float *self, int32_t use_ip,
                  int32_t *se_pos, int32_t *n_se, int32_t *ke_pos, int32_t *n_ke, int32_t *flag) {
    int32_t r, nse = 0, nke = 0, i;
    const int32_t *KA = D->tx_idx + D->tx_indptr[A];
    int64_t nA = D->tx_indptr[A + 1] - D->tx_indptr[A];
    for (r = 0; r < K; r++) flag[r] = 0;
    for (r = 0; r < K; r++) {
        int32_t pv = order[r], v = ids[pv], ok;
        if (v < 0) continue;
        if (nse == 0) { se_pos[nse++] = pv; continue; }
        /* keyword flag of v against the SE of this moment */
        {
            const int32_t *KX = D->tx_idx + D->tx_indptr[v];
            int64_t nX = D->tx_indptr[v + 1] - D->tx_indptr[v], e;
            int shared = 0, covered_by_some = 0;
            for (e = 0; e < nX; e++) if (contains(KA, nA, KX[e])) { shared = 1; break; }
            if (shared) {
                for (i = 0; i < nse && !covered_by_some; i++) {
                    int32_t y = ids[se_pos[i]];
                    const int32_t *KY = D->tx_idx + D->tx_indptr[y];
                    int64_t nY = D->tx_indptr[y + 1] - D->tx_indptr[y];
                    int all_in = 1;
                    for (e = 0; e < nX; e++)
                        if (contains(KA, nA, KX[e]) && !contains(KY, nY, KX[e])) { all_in = 0; break; }
                    if (all_in) covered_by_some = 1;
                }
                flag[pv] = covered_by_some ? 0 : 1;
            }
        }
        ok = nse < R;
        for (i = 0; i < nse && ok && use_ip; i++)
            if (!(Pm[se_pos[i] * K + pv] < self[pv])) ok = 0;
        if (ok) se_pos[nse++] = pv;
        else if (flag[pv] && nke < ke_cap) ke_pos[nke++] = pv;
    }
    *n_se = nse;
    *n_ke = nke;
}

/* ------------------------------------------------------------------ */
/* S6: final edge lists (last sentences of Step 2; Algorithm 1's two lines
 * after the loop).  For node u, in this order and without duplicates or u:
 *   1. up to R/4 pruned neighbours: SE(u)[0 : R/4]            ("Fwd")
 *   2. up to R/4 reverse neighbours: nodes x with u in Fwd(x), ordered by
 *      (position of u in Fwd(x), x)
 *   3. up to R/2 single-path neighbours, taken round-robin dense, sparse,
 *      lexical from the per-path lists in rank order
 *   4. padding to exactly R: rest of SE(u), then the detour-sorted K-list,
 *      then -1.
 * se: N x R (-1 padded), sorted: N x K, sp_ids: 3 x N x P; rows are written
 * for the nn listed nodes.                                              */
static int present(const int32_t *row, int32_t len, int32_t v) {
    int32_t i;
    for (i = 0; i < len; i++) if (row[i] == v) return 1;
    return 0;
}

void orc_assemble(int64_t N, int32_t R, int32_t K, int32_t P, const int32_t *se, const int32_t *sorted,
                  const int32_t *sp_ids, int64_t nn, const int64_t *node_ids, int32_t *out /* nn x R */) {
    int32_t q = R / 4, h = R / 2;
    int64_t u, x, y;
    for (y = 0; y < nn; y++) {
        int32_t *row = out + y * R, len = 0, i, added, pos, ptr[3] = {0, 0, 0}, turn, idle;
        u = node_ids[y];
        for (i = 0; i < q; i++) {
            int32_t v = se[u * R + i];
            if (v >= 0 && v != u && !present(row, len, v)) row[len++] = v;
        }
        /* reverse neighbours, by (position, x) */
        added = 0;
        for (pos = 0; pos < q && added < q; pos++)
            for (x = 0; x < N && added < q; x++) {
                if (x == u || se[x * R + pos] != (int32_t)u) continue;
                if (!present(row, len, (int32_t)x)) { row[len++] = (int32_t)x; added++; }
            }
        /* single-path neighbours, round-robin */
        added = 0; turn = 0; idle = 0;
        while (added < h && idle < 3) {
            const int32_t *lst = sp_ids + ((int64_t)turn * N + u) * P;
            int took = 0;
            while (ptr[turn] < P) {
                int32_t v = lst[ptr[turn]++];
                if (v < 0 || v == u || present(row, len, v)) continue;
                row[len++] = v; added++; took = 1;
                break;
            }
            idle = took ? 0 : idle + 1;
            turn = (turn + 1) % 3;
        }
        for (i = q; i < R && len < R; i++) {
            int32_t v = se[u * R + i];
            if (v >= 0 && v != u && !present(row, len, v)) row[len++] = v;
        }
        for (i = 0; i < K && len < R; i++) {
            int32_t v = sorted[u * K + i];
            if (v >= 0 && v != u && !present(row, len, v)) row[len++] = v;
        }
        while (len < R) row[len++] = -1;
    }
}

/* Entry points (Section 4.2.1: nodes with the largest vector norms): the E
 * documents with the largest fused self-similarity.                      */
void orc_entry_points(int64_t N, const float *self, int32_t E, int32_t *out) {
    scored *all = (scored *)malloc(sizeof(scored) * (size_t)(N > 0 ? N : 1));
    int64_t i;
    for (i = 0; i < N; i++) { all[i].s = self[i]; all[i].id = (int32_t)i; }
    qsort(all, (size_t)N, sizeof(scored), cmp_scored);
    for (i = 0; i < E; i++) out[i] = i < N ? all[i].id : -1;
    free(all);
}

/* ------------------------------------------------------------------ */
/* S7-S9: best-first search on the semantic edges (Algorithm 2 without the
 * keyword and entity branches).  One pool of capacity L plays both cand and
 * topk.  Each iteration expands the best `width` not-yet-expanded pool
 * entries; every neighbour seen for the first time is scored and inserted if
 * the pool has room or it ranks before the pool's worst entry (which is then
 * evicted).  Stops when nothing is left to expand or after max_iters
 * iterations (0 = no limit).  score_table, if not NULL, supplies the fused
 * score of every document for this query (length N) instead of computing it:
 * used to replay the selection logic on another implementation's scores.
 * deleted, if not NULL, marks documents (one byte each) that are removed from
 * the answer but not from the search.
 * visit_log (optional, capacity log_cap) receives the ids in scoring order.
 * Returns the number of scored documents.                               */
int64_t orc_search(const orc_vecset *D, const int32_t *graph, int32_t R, const int32_t *entry,
                   int32_t E, const orc_vecset *Q, int64_t qi, const float w[3], int32_t k, int32_t L,
                   int32_t max_iters, int32_t width, const float *score_table, const unsigned char *deleted,
                   int32_t *out_ids, float *out_scores, int32_t *visit_log, int64_t log_cap) {
    int64_t N = D->n, nscored = 0;
    unsigned char *visited = (unsigned char *)calloc((size_t)(N > 0 ? N : 1), 1);
    scored *pool = (scored *)malloc(sizeof(scored) * (size_t)(L + 1));
    unsigned char *expanded = (unsigned char *)malloc((size_t)(L + 1));
    int32_t *parents = (int32_t *)malloc(sizeof(int32_t) * (size_t)(width > 0 ? width : 1));
    int32_t len = 0, it = 0, i, e, nout = 0;

#define ORC_SCORE(v) (score_table ? score_table[(v)] : hybrid_fused(Q, qi, D, (v), w))
#define ORC_INSERT(v, s)                                                                       \
    do {                                                                                       \
        int32_t p_;                                                                            \
        if (len == L && !ranks_before((s), (v), pool[len - 1].s, pool[len - 1].id)) break;      \
        if (len == L) len--;                                                                   \
        p_ = len;                                                                              \
        while (p_ > 0 && ranks_before((s), (v), pool[p_ - 1].s, pool[p_ - 1].id)) {            \
            pool[p_] = pool[p_ - 1]; expanded[p_] = expanded[p_ - 1]; p_--;                    \
        }                                                                                      \
        pool[p_].s = (s); pool[p_].id = (v); expanded[p_] = 0; len++;                          \
    } while (0)

    for (e = 0; e < E; e++) {
        int32_t v = entry[e];
        float s;
        if (v < 0 || visited[v]) continue;
        visited[v] = 1;
        s = ORC_SCORE(v);
        if (visit_log && nscored < log_cap) visit_log[nscored] = v;
        nscored++;
        ORC_INSERT(v, s);
    }
    while (max_iters <= 0 || it < max_iters) {
        int32_t np = 0;
        for (i = 0; i < len && np < width; i++)
            if (!expanded[i]) { expanded[i] = 1; parents[np++] = pool[i].id; }
        if (np == 0) break;
        for (i = 0; i < np; i++) {
            const int32_t *nb = graph + (int64_t)parents[i] * R;
            for (e = 0; e < R; e++) {
                int32_t v = nb[e];
                float s;
                if (v < 0 || visited[v]) continue;
                visited[v] = 1;
                s = ORC_SCORE(v);
                if (visit_log && nscored < log_cap) visit_log[nscored] = v;
                nscored++;
                ORC_INSERT(v, s);
            }
        }
        it++;
    }
    /* mark-deletion (Section 4.1, updates): deleted documents take part in the search like any other and are
     * left out of the answer */
    for (i = 0; i < len && nout < k; i++) {
        if (deleted && deleted[pool[i].id]) continue;
        out_ids[nout] = pool[i].id; out_scores[nout] = pool[i].s; nout++;
    }
    for (i = nout; i < k; i++) { out_ids[i] = -1; out_scores[i] = -INFINITY; }
#undef ORC_SCORE
#undef ORC_INSERT
    free(visited); free(pool); free(expanded); free(parents);
    return nscored;
}

/* ------------------------------------------------------------------ */
/* Keyword-constrained search (Section 4.2.2 and the keyword branches of
 * Algorithm 2).  KW = the required term ids; K(v) = the terms of document
 * v's text.  A document "satisfies" the constraint when K(v) meets KW
 * (kw_all = 0, the condition Algorithm 2 writes) or contains all of KW
 * (kw_all = 1).  Differences from the base search:
 *  - a parent that satisfies the constraint also expands its keyword edges
 *    (after its semantic edges; off when use_kw_edges = 0);
 *  - every satisfying document that is scored but not kept by the pool --
 *    rejected on arrival or evicted later -- goes to a secondary pool that
 *    keeps the k best of them;
 *  - the result is the k best satisfying documents of pool and secondary
 *    pool together.
 * n_kw = 0 means "no constraint": the base search.  Deleted documents
 * (see orc_search) still expand their keyword edges when they satisfy the
 * constraint, but enter neither the secondary pool nor the answer.      */
static int kw_satisfied(const orc_vecset *D, int64_t v, const int32_t *kw, int32_t n_kw, int32_t kw_all) {
    int32_t hits = 0, j;
    int64_t p;
    for (j = 0; j < n_kw; j++) {
        int found = 0;
        for (p = D->tx_indptr[v]; p < D->tx_indptr[v + 1]; p++)
            if (D->tx_idx[p] == kw[j]) found = 1;
        hits += found;
    }
    return kw_all ? hits == n_kw : hits > 0;
}

int64_t orc_search_kw(const orc_vecset *D, const int32_t *graph, int32_t R, const int32_t *kw_edges, int32_t KR,
                      const int32_t *kw_count, const int32_t *entry, int32_t E, const orc_vecset *Q, int64_t qi,
                      const float w[3], int32_t k, int32_t L, int32_t max_iters, int32_t width, const int32_t *kw,
                      int32_t n_kw, int32_t kw_all, int32_t use_kw_edges, const float *score_table,
                      const unsigned char *deleted, int32_t *out_ids, float *out_scores, int32_t *visit_log,
                      int64_t log_cap) {
    int64_t N = D->n, nscored = 0;
    unsigned char *visited = (unsigned char *)calloc((size_t)(N > 0 ? N : 1), 1);
    scored *pool = (scored *)malloc(sizeof(scored) * (size_t)(L + 1));
    unsigned char *expanded = (unsigned char *)malloc((size_t)(L + 1));
    unsigned char *sat = (unsigned char *)malloc((size_t)(L + 1));      /* pool entry satisfies the constraint */
    scored *second = (scored *)malloc(sizeof(scored) * (size_t)(k + 1)); /* secondary pool, best first */
    scored *all = (scored *)malloc(sizeof(scored) * (size_t)(L + k + 1));
    int32_t *parents = (int32_t *)malloc(sizeof(int32_t) * (size_t)(width > 0 ? width : 1));
    unsigned char *psat = (unsigned char *)malloc((size_t)(width > 0 ? width : 1));   /* parent satisfies the constraint */
    int32_t len = 0, nsec = 0, it = 0, i, e, nall = 0;

    if (n_kw <= 0) {
        free(visited); free(pool); free(expanded); free(sat); free(second); free(all); free(parents); free(psat);
        return orc_search(D, graph, R, entry, E, Q, qi, w, k, L, max_iters, width, score_table, deleted, out_ids,
                          out_scores, visit_log, log_cap);
    }
    /* one newly seen document: score it, offer it to the pool, pass what the pool does not keep to the secondary pool */
#define KW_VISIT(v)                                                                                   \
    do {                                                                                              \
        scored out_;                                                                                  \
        int out_sat_ = 0, have_out_ = 0, p_;                                                          \
        float s_ = score_table ? score_table[(v)] : hybrid_fused(Q, qi, D, (v), w);                   \
        int sat_ = kw_satisfied(D, (v), kw, n_kw, kw_all);                                            \
        if (visit_log && nscored < log_cap) visit_log[nscored] = (v);                                 \
        nscored++;                                                                                    \
        if (len == L && !ranks_before(s_, (v), pool[len - 1].s, pool[len - 1].id)) {                  \
            out_.s = s_; out_.id = (v); out_sat_ = sat_; have_out_ = 1;                               \
        } else {                                                                                      \
            if (len == L) { out_ = pool[len - 1]; out_sat_ = sat[len - 1]; have_out_ = 1; len--; }    \
            p_ = len;                                                                                 \
            while (p_ > 0 && ranks_before(s_, (v), pool[p_ - 1].s, pool[p_ - 1].id)) {                \
                pool[p_] = pool[p_ - 1]; expanded[p_] = expanded[p_ - 1]; sat[p_] = sat[p_ - 1]; p_--; \
            }                                                                                         \
            pool[p_].s = s_; pool[p_].id = (v); expanded[p_] = 0; sat[p_] = (unsigned char)sat_; len++; \
        }                                                                                             \
        if (have_out_ && out_sat_ && !(deleted && deleted[out_.id]) &&                                \
            (nsec < k || ranks_before(out_.s, out_.id, second[nsec - 1].s, second[nsec - 1].id))) {   \
            if (nsec == k) nsec--;                                                                    \
            p_ = nsec;                                                                                \
            while (p_ > 0 && ranks_before(out_.s, out_.id, second[p_ - 1].s, second[p_ - 1].id)) {    \
                second[p_] = second[p_ - 1]; p_--;                                                    \
            }                                                                                         \
            second[p_] = out_; nsec++;                                                                \
        }                                                                                             \
    } while (0)

    for (e = 0; e < E; e++) {
        int32_t v = entry[e];
        if (v < 0 || visited[v]) continue;
        visited[v] = 1;
        KW_VISIT(v);
    }
    while (max_iters <= 0 || it < max_iters) {
        int32_t np = 0;
        for (i = 0; i < len && np < width; i++)
            if (!expanded[i]) { expanded[i] = 1; psat[np] = sat[i]; parents[np++] = pool[i].id; }
        if (np == 0) break;
        for (i = 0; i < np; i++) {
            const int32_t u = parents[i];
            const int32_t *nb = graph + (int64_t)u * R;
            for (e = 0; e < R; e++) {
                int32_t v = nb[e];
                if (v < 0 || visited[v]) continue;
                visited[v] = 1;
                KW_VISIT(v);
            }
            /* the keyword edges of a parent that itself satisfies the constraint */
            if (use_kw_edges && psat[i]) {
                const int32_t *ke = kw_edges + (int64_t)u * KR;
                for (e = 0; e < kw_count[u] && e < KR; e++) {
                    int32_t v = ke[e];
                    if (v < 0 || visited[v]) continue;
                    visited[v] = 1;
                    KW_VISIT(v);
                }
            }
        }
        it++;
    }
#undef KW_VISIT
    /* merge both pools, keep the satisfying documents, best k */
    for (i = 0; i < len; i++) if (sat[i] && !(deleted && deleted[pool[i].id])) all[nall++] = pool[i];
    for (i = 0; i < nsec; i++) all[nall++] = second[i];
    qsort(all, (size_t)nall, sizeof(scored), cmp_scored);
    for (i = 0; i < k; i++) {
        out_ids[i] = i < nall ? all[i].id : -1;
        out_scores[i] = i < nall ? all[i].s : -INFINITY;
    }
    free(visited); free(pool); free(expanded); free(sat); free(second); free(all); free(parents); free(psat);
    return nscored;
}

/* ------------------------------------------------------------------ */
/* Search with knowledge-graph augmentation (Section 4.2.3 and the entity
 * branches of Algorithm 2), one parent per iteration.
 *   V(x)   = entities of document x          (doc_ent_indptr / doc_ent, ascending)
 *   KG     = undirected relations of entities (kg_indptr / kg_idx, ascending)
 *   nodes(e) = documents that mention e       (en_indptr / en_idx, ascending)
 *   logical edges of x: le_count[x] triples (s, y, t) in le[x*le_cap*3 ..]: s in V(x), (s,t) in KG, t not in V(x),
 *   y mentions t.
 * Every pool entry carries (ent, hop): the entity through which it is tied to the query's entities and the
 * number of relations in between; ent = -1 when there is no such tie.
 *  - With query entities, the search starts from the documents that mention them (in the order of the query's
 *    entities, then ascending document id, at most E of them), each with hop 0 and that entity; otherwise from
 *    the usual entry points with no entity.
 *  - Expanding u: its semantic edges, then -- if u has an entity and u.hop < max_hops -- the targets of its
 *    logical edges whose source is u.ent.
 *  - A newly seen o gets ent = the smallest entity of V(o) related to u.ent (none if u has no entity or V(o) holds
 *    no such entity); with an entity, hop = u.hop + 1 and the score is raised by w_k / hop.
 * ann_log (optional, capacity log_cap x 2): (ent, hop) of every scored document in scoring order.               */
static int32_t related_entity(const int64_t *de_ip, const int32_t *de, const int64_t *kg_ip, const int32_t *kg,
                              int64_t o, int32_t eu) {
    int64_t p, r;
    for (p = de_ip[o]; p < de_ip[o + 1]; p++)
        for (r = kg_ip[eu]; r < kg_ip[eu + 1]; r++)
            if (kg[r] == de[p]) return de[p];          /* V(o) is ascending: the first hit is the smallest */
    return -1;
}

int64_t orc_search_kg(const orc_vecset *D, const int32_t *graph, int32_t R, const int32_t *entry, int32_t E,
                      const orc_vecset *Q, int64_t qi, const float w[3], int32_t k, int32_t L, int32_t max_iters,
                      const int64_t *de_ip, const int32_t *de, const int64_t *kg_ip, const int32_t *kg,
                      const int64_t *en_ip, const int32_t *en, const int32_t *le, int32_t le_cap,
                      const int32_t *le_count, const int32_t *q_ent, int32_t n_qe, float w_k, int32_t max_hops,
                      const float *score_table, const unsigned char *deleted, int32_t *out_ids, float *out_scores,
                      int32_t *visit_log, int32_t *ann_log, int64_t log_cap) {
    int64_t N = D->n, nscored = 0;
    unsigned char *visited = (unsigned char *)calloc((size_t)(N > 0 ? N : 1), 1);
    scored *pool = (scored *)malloc(sizeof(scored) * (size_t)(L + 1));
    unsigned char *expanded = (unsigned char *)malloc((size_t)(L + 1));
    int32_t *p_ent = (int32_t *)malloc(sizeof(int32_t) * (size_t)(L + 1));
    int32_t *p_hop = (int32_t *)malloc(sizeof(int32_t) * (size_t)(L + 1));
    int32_t len = 0, it = 0, i, e, started = 0;

    /* one newly seen document o reached from a parent with (eu, hu); eu = -2: an initial document that carries
     * (ent0, 0) itself */
#define KG_VISIT(o, eu, hu, ent0)                                                                      \
    do {                                                                                               \
        int32_t ent_ = -1, hop_ = 0, p_;                                                               \
        float s_ = score_table ? score_table[(o)] : hybrid_fused(Q, qi, D, (o), w);                    \
        if ((eu) == -2) { ent_ = (ent0); hop_ = 0; }                                                   \
        else if ((eu) >= 0) {                                                                          \
            ent_ = related_entity(de_ip, de, kg_ip, kg, (o), (eu));                                    \
            if (ent_ >= 0) { hop_ = (hu) + 1; s_ = s_ + w_k / (float)hop_; }                           \
        }                                                                                              \
        if (visit_log && nscored < log_cap) visit_log[nscored] = (o);                                  \
        if (ann_log && nscored < log_cap) { ann_log[2 * nscored] = ent_; ann_log[2 * nscored + 1] = hop_; } \
        nscored++;                                                                                     \
        if (len == L && !ranks_before(s_, (o), pool[len - 1].s, pool[len - 1].id)) break;               \
        if (len == L) len--;                                                                           \
        p_ = len;                                                                                      \
        while (p_ > 0 && ranks_before(s_, (o), pool[p_ - 1].s, pool[p_ - 1].id)) {                     \
            pool[p_] = pool[p_ - 1]; expanded[p_] = expanded[p_ - 1];                                  \
            p_ent[p_] = p_ent[p_ - 1]; p_hop[p_] = p_hop[p_ - 1]; p_--;                                \
        }                                                                                              \
        pool[p_].s = s_; pool[p_].id = (o); expanded[p_] = 0; p_ent[p_] = ent_; p_hop[p_] = hop_; len++; \
    } while (0)

    for (e = 0; e < n_qe && started < E; e++) {
        int64_t p;
        int32_t ent = q_ent[e];
        if (ent < 0) continue;
        for (p = en_ip[ent]; p < en_ip[ent + 1] && started < E; p++) {
            int32_t v = en[p];
            if (visited[v]) continue;
            visited[v] = 1; started++;
            KG_VISIT(v, -2, 0, ent);
        }
    }
    if (started == 0) {
        for (e = 0; e < E; e++) {
            int32_t v = entry[e];
            if (v < 0 || visited[v]) continue;
            visited[v] = 1;
            KG_VISIT(v, -1, 0, -1);
        }
    }
    while (max_iters <= 0 || it < max_iters) {
        int32_t u = -1, eu = -1, hu = 0;
        for (i = 0; i < len; i++)
            if (!expanded[i]) { expanded[i] = 1; u = pool[i].id; eu = p_ent[i]; hu = p_hop[i]; break; }
        if (u < 0) break;
        for (e = 0; e < R; e++) {
            int32_t v = graph[(int64_t)u * R + e];
            if (v < 0 || visited[v]) continue;
            visited[v] = 1;
            KG_VISIT(v, eu, hu, -1);
        }
        if (eu >= 0 && hu < max_hops) {
            const int32_t *t3 = le + (int64_t)u * le_cap * 3;
            for (e = 0; e < le_count[u] && e < le_cap; e++) {
                int32_t v = t3[3 * e + 1];
                if (t3[3 * e] != eu || v < 0 || visited[v]) continue;
                visited[v] = 1;
                KG_VISIT(v, eu, hu, -1);
            }
        }
        it++;
    }
#undef KG_VISIT
    /* mark-deletion (Section 4.1, updates): as in the plain search, deleted documents were searched through
     * like any other and are only left out of the answer */
    {
        int32_t o = 0;
        for (i = 0; i < len && o < k; i++) {
            if (deleted && deleted[pool[i].id]) continue;
            out_ids[o] = pool[i].id; out_scores[o] = pool[i].s; o++;
        }
        for (; o < k; o++) { out_ids[o] = -1; out_scores[o] = -INFINITY; }
    }
    free(visited); free(pool); free(expanded); free(p_ent); free(p_hop);
    return nscored;
}
