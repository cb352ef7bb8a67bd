/*
 * tsdg_ann.h -- C ABI of the MI355X (gfx950) library for graph-based approximate
 * nearest-neighbour search on a two-stage diversified k-NN graph (TSDG).
 *
 * Problem statement (paper Sec. 1): given a query q and a metric m, return the
 * top-k nearest neighbours of q from a candidate set.  The work is split, as in
 * Sec. 2.2, into an offline graph build and an online search:
 *
 *   ann_build_graph  exact k-NN graph -> relaxed diversification (Sec. 3.2,
 *                    Eq. 2) -> reverse edges -> soft diversification with an
 *                    occlusion factor lambda per edge (Sec. 3.3, Eq. 1)
 *   ann_search       best-first search from 32 random seeds over that graph,
 *                    visiting in each neighbour list only the prefix whose
 *                    lambda is below a threshold (Sec. 3.3, Sec. 4, Sec. 5.4)
 *
 * Conventions for every call
 *   - ALL data pointers are DEVICE pointers on the current HIP device, row-major,
 *     rows contiguous; base and query rows must start on 16-byte boundaries
 *     (d a multiple of 4 for fp32 rows, of 16 for uint8 rows).
 *   - The metric is L2; every distance taken or returned is the SQUARED L2
 *     distance in fp32, computed as fl32( sum_j (double)(fl32(a_j - b_j))^2 ).
 *   - Order is (distance, id): of two equal distances the smaller id comes first.
 *   - The caller owns base, queries and the output arrays.  A graph object owns
 *     its adjacency memory until ann_graph_free; it keeps NO pointer to base.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream).  ann_search* return after enqueueing; ann_build_graph*,
 *     ann_knn, ann_bruteforce, import and export synchronise the stream before
 *     returning because they size or free temporary device memory (hipFree also
 *     waits for work on the caller's other streams).  The search calls
 *     (ann_search_ex, ann_search_alg2, ann_search_multi with the caller's
 *     workspace, ann_search_multi_static) allocate nothing and only read the graph.
 *   - Errors: a status code is returned, never an exception or abort; outputs
 *     are untouched when argument validation fails; ann_last_error() gives a
 *     thread-local message for the last failing call.
 *   - Limits: 1 <= K <= 64, N > K, N < 2^27, 1 <= k <= L <= 512,
 *     d <= 2048 (fp32) / d <= 1024 (uint8), 0 <= lambda0 <= 30, at most 2^22
 *     queries per search call.
 */
#ifndef TSDG_ANN_H
#define TSDG_ANN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ann_graph ann_graph; /* opaque; owns the packed adjacency in device memory */

typedef enum {
    ANN_OK = 0,
    ANN_EINVAL = 1,      /* bad argument (null pointer, size out of range, misaligned row) */
    ANN_ENOMEM = 2,      /* device or host allocation failed */
    ANN_EDEVICE = 3,     /* a HIP call or kernel launch failed */
    ANN_EUNSUPPORTED = 4 /* valid request outside the limits above */
} ann_status;

/* Element type of base rows.  ANN_F16 (IEEE binary16, d a multiple of 8) is a STORAGE type for the
 * search entry points only: distances are the canonical ones of the stored values (each converts
 * exactly to fp32); the graph is built from fp32 or uint8 rows. */
typedef enum { ANN_F32 = 0, ANN_U8 = 1, ANN_F16 = 2 } ann_dtype;

/* Dissimilarity m(.,.) of Sec. 2 / Table 1.
 *   ANN_L2:     squared Euclidean distance s (what every call returns); Eq. 2's alpha acts on
 *               the distance, i.e. alpha^2 on s.
 *   ANN_COSINE: m = 1 - cos.  Base rows and queries must be UNIT vectors in fp32 (the caller
 *               normalises once, e.g. with ann_normalize_rows; this is not checked).  Then
 *               m = s/2: the k-NN graph and every walk are those of s, Eq. 2's alpha acts on m
 *               (alpha on s), and the distances returned are m = s/2. */
typedef enum { ANN_L2 = 0, ANN_COSINE = 1 } ann_metric;

/* Progress of a long build: called on the calling thread, between launches, after the build's
 * stream has been synchronised (so a build that reports progress is slower than one that does
 * not).  step names what was finished ("knn-sweep": done/total = base columns swept for the current
 * block of rows; "knn-rows": rows finished; "descent": iterations done / the limit), user is
 * passed through.  The callback must not call back into the library on the same graph. */
typedef void (*ann_progress_fn)(void* user, const char* step, int64_t done, int64_t total);

/* Optional report of a build, filled on the host when ann_build_params.stats points at one:
 * device time of the four steps (events on the build's stream) and the work they did. */
typedef struct {
    float knn_ms;            /* k-NN lists (exact contraction + re-scoring, or the propagation) */
    float stage1_ms;         /* Eq. 2 pruning */
    float reverse_ms;        /* reverse edges: count scan, scatter, per-node merge and cut */
    float stage2_ms;         /* lambda by Eq. 1, order, cuts, packing */
    uint64_t stage1_rows;    /* base rows stage 1 reads: every node's own row and its K list entries */
    uint64_t stage2_rows;    /* likewise for stage 2: own row + list length after the reverse edges and the cut */
    uint64_t reverse_edges;  /* edges that survive stage 1 (each is scattered once as a reverse edge) */
    int gather_row_bytes;    /* bytes of one gathered row in stages 1 and 2 (d for the centred int8 copy of
                                integer-valued rows, else d * element size) */
    int knn_contraction;     /* 0: int8 matrix cores (exact), 1: one binary16 part, 2: bf16 hi + lo parts,
                                3: integer rows wider than 128 as one bf16 part (exact), 4: propagation */
    uint32_t knn_plain_scan_rows; /* rows whose list the re-scoring pass could not certify and a plain scan redid */
} ann_build_stats;

/* Build parameters.  Defaults (ann_build_params_default): fp32 rows,
 * alpha = 1.2 (Sec. 3.2 recommends values above 1.1), lambda0 = 9 (so that the
 * small-batch prefix of Sec. 5.4, lambda below 10, means every stored edge),
 * rev_cap = 0 meaning 2*K (length to which a list is cut after the reverse
 * edges are appended; the paper leaves it unbounded), stream NULL. */
typedef struct {
    ann_dtype dtype;
    float alpha;
    int lambda0;
    int rev_cap;
    void* stream;
    ann_metric metric; /* default ANN_L2 */
    /* Which k-NN graph the diversification starts from (Sec. 3 allows an approximate one;
     * the default here is the exact one).  knn_mode 0 = exact (MFMA contraction);
     * 1 = neighbourhood propagation, see ann_knn_descent, with the four parameters below
     * (0 = defaults: S = largest power of two <= min(16, K/2), 12 iterations, delta 0.001, seed 0). */
    int knn_mode;
    int descent_S;
    int descent_iters;
    float descent_delta;
    uint64_t descent_seed;
    /* Form of the exact contraction for real-valued rows: 0 = one scaled binary16 part per row, falling back
     * to two bf16 parts (hi + lo) when too many rows fail the re-scoring pass's acceptance test; 1 = hi + lo
     * from the start.  Both give the exact lists; integer-valued rows ignore it. */
    int knn_filter;
    /* Query rows per sweep of the exact contraction; 0 = 2^21 (bounds the candidate buffers to a few GB).
     * A multiple of 256; smaller values only cost time (a hook for tests of the multi-sweep path). */
    int64_t knn_row_block;
    ann_progress_fn progress; /* NULL = no reports and no extra synchronisation */
    void* progress_user;
    ann_build_stats* stats;   /* host pointer or NULL */
} ann_build_params;

/* Search parameters.  Defaults (ann_search_params_default): fp32 rows, mode 0
 * (auto: small-batch kernel below a batch-size threshold, large-batch kernel
 * above; the threshold was measured per row length: 1,024 queries for rows of up
 * to 128 bytes, 4,096 up to 512 bytes, 16,384 up to 2,048 bytes, 32,768 beyond), lambda_visit 0 meaning "by mode" (Sec. 5.4: 10 for small batches, 5
 * for large ones), n_seeds 32 (Alg. 2), seed 0, max_hops 0 = unbounded (the hop
 * limit T of Alg. 2), visited_slots 0 = chosen from mode, L and the row length, waves_per_query 0 =
 * chosen from the row length and the batch size (8 wavefronts up to 512 queries, 4 for rows of at most 128
 * bytes; beyond, 2 for rows of 129..512 bytes and 4 otherwise), qi_offset 0, stream NULL.
 *   mode: 1 = large batch (one 64-lane wavefront per query),
 *         2 = small batch (one workgroup of several wavefronts per query).
 *   lambda_visit: edges with lambda < lambda_visit are followed; values above
 *         31 mean every stored edge.  RESULTS DEPEND ON IT.
 *   visited_slots: capacity (a multiple of 64 in 64..16384) of the per-query hashed
 *         visited set.  It is lossy without false positives: results do not
 *         depend on it, only the number of distance evaluations does.
 *   qi_offset: added to the query's index in the seed generator, so that a
 *         batch split over several calls draws the seeds of the whole batch. */
typedef struct {
    ann_dtype dtype;
    int mode;
    int lambda_visit;
    int n_seeds;
    uint64_t seed;
    int max_hops;
    int visited_slots;
    int waves_per_query;
    int64_t qi_offset;
    void* stream;
    ann_metric metric; /* default ANN_L2; must be the metric the graph was built with */
} ann_search_params;

/* Optional per-query counters written by ann_search_ex ([nq] on the device). */
typedef struct {
    uint32_t hops;       /* nodes expanded */
    uint32_t dist_evals; /* distances computed, seeds included */
    uint32_t dedup_hits; /* neighbours skipped because the visited set held them */
} ann_query_stats;

void ann_build_params_default(ann_build_params* p);
void ann_search_params_default(ann_search_params* p);

/* Offline phase (Sec. 3).  base: [N,d] device rows.  On success *out is a new
 * graph of N rows and K columns: row i lists at most K neighbours of i sorted by
 * (lambda, distance, id), each with lambda <= lambda0.
 *   1. exact K nearest neighbours of every row (MFMA distance contraction with a
 *      fused threshold filter, candidates re-scored with the canonical distance);
 *   2. stage 1, Eq. 2 with the checking order of Sec. 3.1;
 *   3. reverse edges appended, duplicates removed, list cut to rev_cap by (s,id);
 *   4. stage 2: lambda_j = number of other edges of the list that occlude edge j
 *      by Eq. 1; sort by (lambda, s, id); drop lambda > lambda0; cut to K.
 * ann_build_graph uses the default parameters. */
ann_status ann_build_graph(const void* base, int64_t N, int d, int K, ann_graph** out);
ann_status ann_build_graph_ex(const void* base, int64_t N, int d, int K,
                              const ann_build_params* params, ann_graph** out);

/* Step 1 of the build alone: knn_ids [N,K] int32 and knn_dists [N,K] fp32 (device),
 * row i = the K nearest other rows by (distance, id). */
ann_status ann_knn(const void* base, int64_t N, int d, int K, ann_dtype dtype, void* stream,
                   int32_t* knn_ids, float* knn_dists);
/* The same with build parameters: of params it reads dtype, stream, knn_filter, knn_row_block,
 * progress / progress_user and stats (knn_ms, knn_contraction, knn_plain_scan_rows). */
ann_status ann_knn_ex(const void* base, int64_t N, int d, int K, const ann_build_params* params,
                      int32_t* knn_ids, float* knn_dists);

/* Exact top-k of each query against the whole base set (the definition the
 * search approximates; used for ground truth, Eq. 3).  queries [nq,d] fp32.
 * out_ids [nq,k] int32, out_dists [nq,k] fp32; 1 <= k <= 128; k <= N. */
ann_status ann_bruteforce(const void* base, int64_t N, int d, ann_dtype dtype,
                          const float* queries, int nq, int k, void* stream,
                          int32_t* out_ids, float* out_dists);

/* Online phase (Sec. 4).  queries [nq,d] fp32 (also for uint8 base rows).
 * out_ids [nq,k] int32, out_dists [nq,k] fp32 squared L2; when fewer than k
 * nodes were reached the tail is id -1 / distance +inf.  ann_search uses the
 * default parameters; ann_search_ex takes them explicitly and optionally
 * writes stats[nq] (NULL to skip).  nq = 0 is valid and does nothing. */
ann_status ann_search(const ann_graph* graph, const void* base, const void* queries, int nq,
                      int k, int L, int32_t* out_ids, float* out_dists);
ann_status ann_search_ex(const ann_graph* graph, const void* base, const void* queries, int nq,
                         int k, int L, const ann_search_params* params, int32_t* out_ids,
                         float* out_dists, ann_query_stats* stats);

/* Small-batch multi-search (Sec. 4.1, Alg. 1): t0 independent greedy searches per query, each
 * on its own workgroup from its own 32 random start nodes, merged into the top-k.  It trades
 * distance evaluations for latency (a search converges in a handful of hops) and lets a batch
 * of one use many compute units; its result is NOT the best-first result of ann_search.
 * 1 <= k <= 32, 1 <= t0 <= 1024, nq <= 65535.  Of params it reads dtype, lambda_visit
 * (0 = 10), seed, max_hops (the hop limit T; 0 = 16), qi_offset and stream.
 * The t0 rankings of every query pass through `workspace`, device memory of the caller of at
 * least ann_search_multi_workspace_bytes(nq, t0) = nq * t0 * 264 bytes, 8-byte aligned, which
 * the call may overwrite and which must stay untouched until the work enqueued on the stream has
 * run; calls with different workspaces may overlap.  workspace = NULL: the call allocates one,
 * waits for the stream and frees it (convenient, not for latency-critical callers). */
size_t ann_search_multi_workspace_bytes(int nq, int t0);
ann_status ann_search_multi(const ann_graph* graph, const void* base, const void* queries, int nq, int k,
                            int t0, const ann_search_params* params, void* workspace,
                            size_t workspace_bytes, int32_t* out_ids, float* out_dists,
                            ann_query_stats* stats);

/* ann_search_multi for callers that can neither allocate device memory nor bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * kernels and the same result as ann_search_multi, but the t0 rankings go to a scratch array that
 * is part of the library's device image (540,672 bytes on every GPU the library runs on, held until
 * the process ends) instead of a workspace, and the call never calls hipMalloc, hipFree or any
 * allocating routine.  Limit: nq * t0 <= 2048 searches per call (ANN_EUNSUPPORTED
 * beyond, outputs untouched).  The first call on a device looks the array's address up once.
 * Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two
 * threads) race and must be serialised by the caller; consecutive calls on one stream are safe.
 * Nothing in the array needs clearing between calls (every word a call reads it has written). */
ann_status ann_search_multi_static(const ann_graph* graph, const void* base, const void* queries, int nq,
                                   int k, int t0, const ann_search_params* params, int32_t* out_ids,
                                   float* out_dists, ann_query_stats* stats);

/* Large-batch search with the structures of Alg. 2 / Sec. 4.2 as printed: a ranking array R of
 * fixed size k (k <= 64), an expansion queue C of m_c segments of 32 sorted entries (segment =
 * id mod m_c; a push into a full segment drops its most distant entry; pop = smallest head), a
 * look-up table V of m_v segments of 32 slots holding only expanded nodes (round-robin
 * overwrite), start from the closest of 32 seeds, stop when the popped candidate u is further
 * than the furthest f of R by more than delta ON THE MEASURE ITSELF, m(u,q) > m(f,q) + delta as
 * Alg. 2 prints it: for ANN_L2 delta is an L2 distance (sqrt(s_u) > sqrt(s_f) + delta, evaluated
 * as (s_u - s_f) - delta^2 > 0 and its square above 4 delta^2 s_f in fp64, so that no square root is
 * taken), for ANN_COSINE a difference of 1 - cos; or when C is empty or at the hop limit.  The
 * distances returned stay squared L2 (or 1 - cos).  1 <= m_c, m_v <= 64.  Unlike ann_search its result depends on m_c and m_v.
 * Of params it reads dtype, lambda_visit (0 = 5), seed, max_hops (0 = unbounded), qi_offset,
 * stream; stats->dedup_hits counts neighbours skipped because V or C held them. */
ann_status ann_search_alg2(const ann_graph* graph, const void* base, const void* queries, int nq, int k,
                           float delta, int m_c, int m_v, const ann_search_params* params,
                           int32_t* out_ids, float* out_dists, ann_query_stats* stats);

/* Flat copies of a graph, N*K entries each (device pointers): adj = neighbour
 * id or -1 for an unused slot, lam = occlusion factor or 255 for an unused
 * slot.  Import validates ids (range, no self loop, no repeats in a row,
 * unused slots only at the end, lambda <= 30) and returns ANN_EINVAL otherwise;
 * d is the row length of the base set the graph describes (a graph remembers
 * it, which is how ann_search knows the row shape of `base`).
 * Together they serve as save/load. */
ann_status ann_graph_export(const ann_graph* graph, int32_t* adj, uint8_t* lam, void* stream);
ann_status ann_graph_import(const int32_t* adj, const uint8_t* lam, int64_t N, int K, int d,
                            void* stream, ann_graph** out);
ann_status ann_graph_info(const ann_graph* graph, int64_t* N, int* K, int* d);
void ann_graph_free(ann_graph* graph);

/* Inner product (Table 1, m = IP) by the standard reduction of maximum-inner-product search to L2:
 * with M >= every base norm a base row x becomes [x, sqrt(M^2 - |x|^2), 0, 0, 0] and a query q
 * becomes [q, 0, 0, 0, 0]; on these rows of d + 4 columns s = |q|^2 + M^2 - 2<q,x>, so every build
 * and search call with ANN_L2 ranks by -<q,x>, and <q,x> = (|q|^2 + M^2 - s) / 2.
 * ann_max_row_norm writes the largest row norm fl32(sqrt(sum x^2 in fp64)) of src[n,d] to *M (host;
 * the call synchronises `stream`).  ann_ip_augment_rows writes dst[n, d+4] (device, 16-byte aligned;
 * not in place); is_query = 0 needs M > 0, and a row longer than M gets 0 as its extra coordinate.
 * src: device fp32 rows, d a multiple of 4, d + 4 <= 2048. */
ann_status ann_max_row_norm(const float* src, int64_t n, int d, void* stream, float* M);
ann_status ann_ip_augment_rows(const float* src, int64_t n, int d, float M, int is_query, float* dst, void* stream);

/* Approximate k-NN lists by neighbourhood propagation (the published NN-descent idea in a form
 * where every node pulls its candidates from the previous iteration's lists, so the result does
 * not depend on execution order; Sec. 3 starts from an approximate k-NN graph and names no
 * builder).  base[N,d] device rows of `dtype`; K in 1..64, K < N; S = sample size, a
 * power of two in 2..16; at most max_iters iterations, stopping early once an iteration changes
 * no more than delta*N*K list entries; `seed` draws the start lists (2K draws per node from the
 * generator of the search's seeds), or init_ids[N,K] (device, may be NULL; -1 = none) gives them.
 * Outputs knn_ids[N,K] int32 / knn_dists[N,K] fp32 (device) in (s,id) order, padded -1 / +inf;
 * iters_done and last_changed (host, may be NULL).  Work per iteration is O(N * S^2) distance
 * evaluations instead of the exact build's N^2.  Synchronises `stream` once per iteration. */
ann_status ann_knn_descent(const void* base, int64_t N, int d, int K, ann_dtype dtype, int S, int max_iters,
                           float delta, uint64_t seed, const int32_t* init_ids, void* stream, int32_t* knn_ids,
                           float* knn_dists, int* iters_done, int64_t* last_changed);

/* Unit rows for ANN_COSINE (Table 1, m = Cos): dst[i,:] = src[i,:] / |src[i,:]| for n rows of d
 * fp32 elements (d a multiple of 4, at most 2048; both device, 16-byte aligned, may be the same
 * buffer).  The norm is fl32(sqrt(sum of squares in fp64)), each quotient is formed in fp64 and
 * rounded once; a zero row stays zero.  Asynchronous on `stream`. */
ann_status ann_normalize_rows(const float* src, int64_t n, int d, float* dst, void* stream);

/* Message of the last failing call on this thread ("" if none). */
const char* ann_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TSDG_ANN_H */
