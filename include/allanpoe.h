/*
 * allanpoe.h -- C ABI of the MI355X (gfx950) hybrid graph index.
 *
 * The library computes, entirely in hand-written HIP kernels, the hot path of
 * the all-in-one hybrid index: the hybrid similarity of Definition 1
 *     M_w(q,d) = w_d <q_d,d_d> + w_s <q_s,d_s> + w_f <q_f,d_f>
 * (dense inner product, learned-sparse inner product over ascending
 * (term id, weight) lists, BM25 full-text score as a lexical sparse inner
 * product, Section 3.2), the index construction it drives (Algorithm 1,
 * Steps 1-3 of Section 4.1) and the batched best-first search on the semantic
 * edges with per-query fusion weights (Algorithm 2, Section 4.2.1).
 *
 * General rules
 *  - Every pointer is a DEVICE pointer owned by the caller unless the comment
 *    says "host".  `stream` is a hipStream_t passed as void* (NULL = the null
 *    stream).  Calls enqueue work on `stream`; outputs are valid once the
 *    caller has synchronised it.  Calls that create an index (build, ingest,
 *    import) synchronise the stream themselves before returning.
 *  - An index BORROWS the corpus arrays (dense rows and both CSR structures):
 *    they must stay alive and unchanged until ap_free_index.  Everything else
 *    the index needs (BM25 weights, self-similarities, graph, workspaces) it
 *    allocates with hipMalloc and releases in ap_free_index.
 *  - Return value: 0 on success, a negative AP_E* code otherwise; the message
 *    of the last failure on the calling thread is at ap_last_error().  Nothing
 *    here throws or aborts.
 *  - Scores are similarities: larger is better (the paper's dis is -score).
 *    Every ranking is by (score descending, id ascending).  A missing result
 *    has id -1 and score -inf.
 *  - CSR rows must hold strictly ascending term ids in [0, vocab) and finite
 *    values, with row offsets ascending from 0.  ids of documents must fit 30
 *    bits (n < 2^30); the two CSR parts together hold fewer than 2^32 entries
 *    and no list more than 65,535.  A corpus is checked for all of this when
 *    an index is made from it (AP_EINVAL); query batches are not checked.
 *  - With ALLANPOE_PROGRESS set in the environment, ap_build_index reports on
 *    stderr how far its seed stage has come (minutes on millions of documents).
 *  - Calls on one index from several host threads at once are not supported
 *    (the search workspace is per index).
 */
#ifndef ALLANPOE_H
#define ALLANPOE_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AP_OK 0
#define AP_EINVAL (-1)   /* bad argument (null pointer, unsupported size, bad enum) */
#define AP_ENOMEM (-2)   /* hipMalloc failed */
#define AP_EHIP (-3)     /* a HIP runtime call or kernel launch failed */
#define AP_ESTATE (-4)   /* the index lacks what the call needs (e.g. no graph yet) */

#define AP_F32 0
#define AP_BF16 1

typedef struct ap_index ap_index; /* opaque */

/* The corpus: n fused vectors (Section 3.2: dense part, learned sparse part,
 * and the text as a bag of (term id, term count) from which the lexical
 * sparse vector is derived at ingest). */
typedef struct {
    int64_t n;
    int32_t dim;          /* dense dimension; multiple of 4 (f32) or 8 (bf16); <= 1024 (f32) / 2048 (bf16) */
    int32_t dense_dtype;  /* AP_F32 or AP_BF16 (accumulation is always f32) */
    const void *dense;    /* n x dim, row-major, 16-byte aligned */
    const int64_t *sp_indptr; /* n+1 */
    const int32_t *sp_idx;
    const float *sp_val;
    int32_t sp_vocab;
    const int64_t *tx_indptr; /* n+1 */
    const int32_t *tx_idx;
    const float *tx_tf;   /* term counts */
    int32_t tx_vocab;
} ap_corpus;

/* Construction parameters (Algorithm 1 names `it` and `d`; the rest are the
 * quantities it leaves open). */
typedef struct {
    int32_t degree;     /* d: length of every semantic edge list; multiple of 4, <= 128 */
    int32_t knn_k;      /* K: k-NN list length during construction; degree <= K <= 256 */
    int32_t nd_rounds;  /* it: refinement rounds */
    int32_t nd_sample;  /* S: neighbours (and neighbours of each) explored per round; <= 32 */
    int32_t n_entry;    /* E: number of entry points; <= 256 */
    int32_t sp_len;     /* P: length of each per-path list; <= 32; 0 = ceil(degree/6) */
    float bm25_k1, bm25_b;
    float build_w[3];   /* fusion weights used during construction */
    int32_t prune_mode; /* AP_PRUNE_JOINT (0, Algorithm 1), or one of the two ablations of the joint strategy
                           (Section 5, effectiveness of RNG-IP joint pruning): AP_PRUNE_RNG_ONLY keeps the first d
                           neighbours of the detour order without the inner-product test, AP_PRUNE_IP_ONLY applies
                           the test to the list in its similarity order without the detour sort */
    uint64_t seed;      /* reserved (construction is deterministic) */
} ap_build_params;
#define AP_PRUNE_JOINT 0
#define AP_PRUNE_RNG_ONLY 1
#define AP_PRUNE_IP_ONLY 2

/* A batch of queries.  tx_cnt holds term counts of the query text. */
typedef struct {
    int32_t nq;
    const float *dense;   /* nq x dim f32 */
    const int64_t *sp_indptr; const int32_t *sp_idx; const float *sp_val;
    const int64_t *tx_indptr; const int32_t *tx_idx; const float *tx_cnt;
} ap_queries;

#define AP_MAX_BEAM 16384
typedef struct {
    int32_t k;            /* results per query; k <= beam */
    int32_t beam;         /* L: candidate pool capacity; <= AP_MAX_BEAM, as far as the pool (8 bytes per entry) and the
                             call's other per-query arrays fit a workgroup's 160 KB of LDS (else AP_EINVAL) */
    int32_t max_iters;    /* 0 = until the pool is fully expanded */
    int32_t search_width; /* p: pool entries expanded per iteration; 1..16 */
} ap_search_params;

/* ---- the three calls of the problem statement -------------------------- */

/* Algorithm 1 (Steps 1-3): S0 lexical encoding, seed lists, refinement rounds
 * under the hybrid metric, detour sort, IP pruning with keyword recycling,
 * edge-list assembly, entry points.  Synchronises `stream`. */
int ap_build_index(const ap_corpus *corpus, const ap_build_params *params, void *stream, ap_index **out);

/* Default fusion weights [w_d, w_s, w_f] (host pointer) used by searches that
 * pass no per-query weights.  O(1): the index is never rebuilt for a change of
 * weights (Theorem 1; Section 4.2.1).  A blocking 12-byte copy: call it when
 * no search that relies on the default weights is still in flight. */
int ap_set_weights(ap_index *index, const float w[3]);

/* Algorithm 2 on the semantic edges for nq queries at once.  per_query_w is
 * nq x 3 (device) or NULL for the index default.  out_ids / out_scores are
 * nq x k.  The call sizes a per-index workspace (one visited bit per document
 * for every query in flight, at most 2 GiB: larger batches run in slabs of
 * queries, one launch each) and may allocate on first use or when nq grows. */
int ap_search_batch(ap_index *index, const ap_queries *queries, const float *per_query_w,
                    const ap_search_params *params, int32_t *out_ids, float *out_scores, void *stream);

/* ap_search_batch for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same results bit for bit; the visited
 * sets live in a static device array of AP_NOALLOC_WORKSPACE_BYTES (64 MiB, held by every GPU the library runs
 * on until the process ends) instead of the index's workspace, and batches beyond it run in slabs of queries.
 * The call allocates nothing, records no events and writes nothing into the index: ap_search_stats does not
 * report on it.  A corpus of more than 8 * AP_NOALLOC_WORKSPACE_BYTES documents (one query's visited bits
 * would not fit) is refused with AP_EINVAL.  All such calls on one GPU share the array: calls that overlap
 * (different streams, different host threads, different indexes) race; calls on one stream are ordered.  Not for
 * indexes with mark-deleted documents when n >= 2^29 (as ap_search_batch). */
#define AP_NOALLOC_WORKSPACE_BYTES ((size_t)64 << 20)
int ap_search_batch_noalloc(const ap_index *index, const ap_queries *queries, const float *per_query_w,
                            const ap_search_params *params, int32_t *out_ids, float *out_scores, void *stream);

/* Keyword-constrained search (Section 4.2.2; the keyword branches of
 * Algorithm 2).  kw_terms (device): nq x kw_stride term ids of the lexical
 * vocabulary that a result's text must contain, -1 = unused slot, kw_stride in
 * [1, 16]; a query whose slots are all unused runs the plain search.  A
 * document satisfies the constraint when its text holds at least one required
 * term (the condition Algorithm 2 writes), or all of them with AP_KW_ALL.
 * While searching, a parent that satisfies the constraint also expands its
 * keyword edges (unless AP_KW_NO_EDGES), every scored satisfying document the
 * pool does not keep -- rejected on arrival or evicted later -- goes to a
 * secondary pool of the k best, and the result is the k best satisfying
 * documents of both pools (-1 / -inf padded when fewer were met).  Satisfying
 * candidates are always scored in full.  Needs n < 2^29 and an index with
 * keyword edges (built here or imported).  Other arguments as ap_search_batch;
 * ap_search_stats reports on this search as well. */
#define AP_KW_ALL 1u
#define AP_KW_NO_EDGES 2u
int ap_search_batch_keywords(ap_index *index, const ap_queries *queries, const float *per_query_w,
                             const ap_search_params *params, const int32_t *kw_terms, int32_t kw_stride,
                             uint32_t kw_flags, int32_t *out_ids, float *out_scores, void *stream);

/* Mark-deletion (Section 4.1, updates of the hybrid index): the count listed
 * documents (device ids) are marked deleted, or restored when restore != 0.
 * Deleted documents stay in the graph and are searched through like any
 * other; ap_search_batch, ap_search_batch_keywords and
 * ap_search_batch_entities leave them out of their answers (and out of the
 * secondary pool), so an answer holds the best k live documents the search
 * met.  The marks carry over to the index ap_insert_documents returns.  Synchronises `stream`; ids outside [0, n) are
 * skipped and reported as AP_EINVAL after the others were applied. */
int ap_mark_deleted(ap_index *index, const int32_t *ids, int64_t count, int restore, void *stream);

/* Insertion of new documents (Section 4.1, updates of the hybrid index).
 * `enlarged` is the corpus after the insertion: its first n0 documents are
 * those of `old`, unchanged and in the same order, the rest are new; same
 * dimension, dense type and vocabularies.  Produces a new index over the
 * enlarged corpus (which it borrows like ap_build_index does); `old` stays
 * valid and is not modified.  Steps: S0 over the enlarged corpus (lexical
 * weights follow the new corpus statistics); candidate set one = the K best
 * old documents for each new one, found by the search of Algorithm 2 on the
 * old semantic edges with the new document as the query, the construction
 * weights and a pool of `beam` (0 = 2K); candidate set two = K-lists among the
 * new documents alone (seed + the refinement rounds of the parameters); the
 * K-list of a new document = the best K of both sets; pruning and keyword
 * recycling for the new documents only; edge-list assembly over all documents
 * (old documents gain reverse neighbours among the new ones); entry points
 * from all self-similarities.  Mark-deleted documents of `old` stay deleted
 * (and, being part of the graph, stay eligible as neighbours of new
 * documents); a knowledge graph set on `old` is not carried over (its
 * arrays describe the old corpus: call ap_set_knowledge_graph on the new
 * index).  Needs an index produced by ap_build_index or
 * ap_insert_documents (AP_ESTATE for an imported graph).  Synchronises
 * `stream`.  trace (may be NULL): optional device buffers that receive the
 * intermediates for the m = n1 - n0 new documents, any of them NULL. */
typedef struct {
    int32_t *cand1_ids; float *cand1_sc;       /* m x K: candidate set one */
    int32_t *cand2_ids; float *cand2_sc;       /* m x K: candidate set two (global ids) */
    int32_t *cand2_sp_ids; float *cand2_sp_sc; /* 3 x m x P: per-path lists that came with set two */
    int32_t *merged_ids; float *merged_sc;     /* m x K: best K of both sets */
    int32_t *knn_ids; float *knn_sc;           /* m x K: the list handed to pruning */
} ap_insert_trace;
int ap_insert_documents(const ap_index *old, const ap_corpus *enlarged, int32_t beam, const ap_insert_trace *trace,
                        void *stream, ap_index **out);

/* What the construction keeps for later insertions (any pointer may be NULL):
 * pruned lists n x degree, detour-sorted lists n x knn_k, per-path lists
 * 3 x n x sp_len and their scores. */
int ap_export_build_state(const ap_index *index, int32_t *se, int32_t *sorted_ids, int32_t *sp_ids, float *sp_sc,
                          void *stream);

/* Knowledge-graph augmentation (Section 3.4; the last step of Algorithm 1).
 * doc_ent_indptr (n+1) / doc_ent: the entities each document mentions, ids in
 * [0, n_ent), ascending per document.  kg_indptr (n_ent+1) / kg_idx: the
 * relations, as a symmetric adjacency of entities, ascending per row, no
 * self-relation.  All four are device arrays the index borrows until it is
 * freed or the call is repeated.  Derives the entity-to-document mapping and
 * the logical edges of every document x: triples (s, y, t) with s an entity
 * of x, (s, t) a relation, t not an entity of x and y != x a document that
 * mentions t, in ascending (s, t, y) order, the first le_cap (<= 128) of them.
 * Synchronises `stream`; row offsets that do not ascend from 0 to the total
 * (< 2^31 each) or malformed ids give AP_EINVAL. */
int ap_set_knowledge_graph(ap_index *index, int32_t n_ent, const int64_t *doc_ent_indptr, const int32_t *doc_ent,
                           const int64_t *kg_indptr, const int32_t *kg_idx, int32_t le_cap, void *stream);

/* Copies out what ap_set_knowledge_graph derived (any pointer may be NULL):
 * le n x le_cap x 3 (-1 padded), le_count n, en_indptr n_ent+1 and en_idx
 * (documents per entity, ascending). */
int ap_export_logical_edges(const ap_index *index, int32_t *le, int32_t *le_count, int64_t *en_indptr, int32_t *en_idx,
                            void *stream);

/* Search with knowledge-graph augmentation (Section 4.2.3; the entity
 * branches of Algorithm 2).  q_ent (device): nq x ent_stride entity ids the
 * query names, ent_stride in [1, 16]; a negative id or one >= n_ent is an
 * unused slot.  Every pool entry carries the entity that ties it to the
 * query's entities and the number of relations in between (hop).  With query entities the search starts from the
 * documents that mention them (order of the query's entities, then ascending
 * id, at most n_entry; hop 0), otherwise from the usual entry points.
 * Expanding u: its semantic edges, then -- if u has an entity and
 * hop(u) < max_hops -- the targets of its logical edges whose source is that
 * entity.  A newly seen document o gets the smallest of its entities related
 * to u's entity (none if u has none); with an entity, hop(o) = hop(u) + 1 and
 * the score is raised by w_k / hop(o).  One parent per iteration
 * (params->search_width must be 1).  Other arguments as ap_search_batch. */
int ap_search_batch_entities(ap_index *index, const ap_queries *queries, const float *per_query_w,
                             const ap_search_params *params, const int32_t *q_ent, int32_t ent_stride, float w_k,
                             int32_t max_hops, int32_t *out_ids, float *out_scores, void *stream);

void ap_free_index(ap_index *index);
const char *ap_last_error(void); /* host string, thread-local */

/* ---- measurement / test surface: the same kernels, exposed stage by stage - */

/* S0 only: an index with lexical weights and self-similarities but no graph. */
int ap_ingest(const ap_corpus *corpus, const ap_build_params *params, void *stream, ap_index **out);

/* Copies out what S0 computed.  Any pointer may be NULL.  tx_w: one f32 per
 * lexical CSR entry; df: tx_vocab int32; avgdl: 1 f32; self_sim: n f32 (fused
 * self-similarity under build_w). */
int ap_export_ingest(const ap_index *index, float *tx_w, int32_t *df, float *avgdl, float *self_sim, void *stream);

/* Definition 1 for explicit pairs: for query x and its c candidates
 * cand_ids[x*c + y] (document ids; anything outside [0, n) is a hole) writes
 * out4[(x*c + y)*4 + {0,1,2,3}] = sim_d, sim_s, sim_f, M_w (holes: -inf). */
int ap_hybrid_scores(const ap_index *index, const ap_queries *queries, const int32_t *cand_ids, int32_t c,
                     const float *per_query_w, float *out4, void *stream);

/* Same with documents on the query side (construction's document-document
 * similarities): a_ids[na] document ids (one outside [0, n) gives a line of
 * holes), w3 three host floats. */
int ap_hybrid_scores_docs(const ap_index *index, const int32_t *a_ids, int32_t na, const int32_t *cand_ids,
                          int32_t c, const float w3[3], float *out4, void *stream);

/* Exact top-k by enumeration of all documents (Theorem 1's MIPS solved by
 * brute force): ground truth for recall. */
int ap_bruteforce_topk(const ap_index *index, const ap_queries *queries, const float *per_query_w, int32_t k,
                       int32_t *out_ids, float *out_scores, void *stream);

/* S2: exact top-K by dense inner product among the other documents for the
 * nn listed nodes (NULL = all n, nn ignored).  out_*: nn x K. */
int ap_stage_seed_knn(const ap_index *index, const int32_t *node_ids, int64_t nn, int32_t K, int32_t *out_ids,
                      float *out_scores, void *stream);

/* S3: one refinement round for the nn listed nodes (NULL = all).  knn_ids is
 * n x K; sp_ids / sp_sc are 3 x n x P (per-path lists so far).  Outputs:
 * out_ids/out_sc nn x K, out_sp_ids/out_sp_sc 3 x nn x P. */
int ap_stage_refine(const ap_index *index, int32_t K, int32_t S, int32_t P, const int32_t *knn_ids,
                    const int32_t *sp_ids, const float *sp_sc, const int32_t *node_ids, int64_t nn,
                    int32_t *out_ids, float *out_sc, int32_t *out_sp_ids, float *out_sp_sc, void *stream);

/* S4 + S5 for the nn listed nodes (NULL = all): neighbourhood similarities,
 * detourable-route counts and sort, IP pruning with keyword flags.
 * knn_ids / knn_sc: n x K lists ranked by fused score.  Outputs (any may be
 * NULL): pm nn x K x K, count nn x K, sorted_ids nn x K, se nn x R (-1 padded),
 * ke nn x R/2 (-1 padded), ke_count nn, flag nn x K (indexed by position in
 * the input list). */
int ap_stage_prune(const ap_index *index, int32_t K, int32_t R, const int32_t *knn_ids, const float *knn_sc,
                   const int32_t *node_ids, int64_t nn, float *pm, int32_t *count, int32_t *sorted_ids,
                   int32_t *se, int32_t *ke, int32_t *ke_count, int32_t *flag, void *stream);

/* S6 for all nodes: se n x R, sorted_ids n x K, sp_ids 3 x n x P -> graph n x R. */
int ap_stage_assemble(const ap_index *index, int32_t R, int32_t K, int32_t P, const int32_t *se,
                      const int32_t *sorted_ids, const int32_t *sp_ids, int32_t *out_graph, void *stream);

/* Entry points: the E documents of largest fused self-similarity. */
int ap_stage_entry_points(const ap_index *index, int32_t E, int32_t *out_entry, void *stream);

/* Graph exchange: lets the search run on a graph built elsewhere and a graph
 * built here be checked elsewhere.  semantic n x degree, keyword n x degree/2,
 * kw_count n, entry n_entry.  Export pointers may be NULL. */
int ap_export_graph(const ap_index *index, int32_t *semantic, int32_t *keyword, int32_t *kw_count, int32_t *entry,
                    void *stream);
int ap_import_graph(const ap_corpus *corpus, const ap_build_params *params, const int32_t *semantic,
                    const int32_t *keyword, const int32_t *kw_count, const int32_t *entry, void *stream,
                    ap_index **out);

/* Counters of the last search (plain or keyword-constrained) on this index (synchronises on that
 * search).  out_counts (device, may be NULL): nq x 3 int32 = per query the
 * number of candidates scored, the number of iterations, and the number of
 * scored candidates whose dense row was not read (their sparse + lexical parts
 * plus the largest possible dense part could not reach the pool).
 * kernel_ms (host, may be NULL): duration of the search kernel alone, measured
 * with events on the stream it ran on. */
int ap_search_stats(const ap_index *index, int32_t *out_counts, int32_t nq, float *kernel_ms, void *stream);

/* Measurement aid: a plain streaming copy kernel (reads and writes `bytes`
 * bytes once each; 16-byte aligned device buffers, bytes % 16 == 0).  Profiler
 * byte counters are scaled by what they report for this copy of known size. */
int ap_calibration_copy(void *dst, const void *src, size_t bytes, void *stream);

/* Timings of the last ap_build_index on this index, host floats in seconds:
 * [0] ingest, [1] seed, [2] refinement, [3] prune, [4] assemble+entry, [5] total. */
int ap_build_timings(const ap_index *index, float out6[6]);

/* Work counters of the construction stages run on this index so far (host array; synchronises `stream`):
 * [0] hybrid similarities evaluated by refinement rounds (whole builds, insertions and ap_stage_refine calls),
 * [1] FLOPs (2 per multiply-add; padded tiles included) of the dense products of the seed stages (the sampled columns,
 *     the sweeps, the exact rows). */
int ap_build_counters(const ap_index *index, uint64_t out2[2], void *stream);

/* Debug settings, for tests: they drive small inputs through the code paths of large ones and never change a
 * result.  One process-wide value per name (host string), 0 = the library's own choice:
 *   "seed_sample_cols"        columns sampled for the seed threshold (forces the thresholded sweep on small corpora)
 *   "seed_buffer_cap"         capacity of a row's candidate buffer in that sweep (forces the overflow fallback)
 *   "seed_tau_ulps"           raises every row's threshold by this many ulps (forces the short-row fallback)
 *   "seed_one_sided"          1: whole-corpus seed lists by the one-sided sweep instead of the symmetric one
 *   "max_launch_threads"      a multiple of 1024: launches that grow with the corpus run in slices of this many threads
 *   "search_workspace_bytes"  cap of the searches' visited-set workspace (forces searches in several slabs of queries)
 *   "search_visited_global"   1: visited sets stay in the global workspace even where the search would keep them in LDS
 *   "search_query_lists"      1: the plain and keyword searches look query terms up in the query's lists, not in LDS tables
 * Unknown names and negative values give AP_EINVAL.  Not thread-safe against running calls. */
int ap_debug_set(const char *name, int64_t value);

#ifdef __cplusplus
}
#endif
#endif
