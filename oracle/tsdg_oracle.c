/*
 * CPU oracle for the two-stage diversified graph (TSDG) build and the
 * best-first k-NN search over it.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
 * statement of what the GPU path must compute.  Only the tests, the smoke
 * check and the benchmark's "cpu_baseline" leg may call it.  It shares no
 * code, header, table or helper with the HIP library, and the HIP library
 * never calls it.
 *
 * What is followed, and where the paper fixes it:
 *   - k-NN graph: the plain definition (all pairs, sort, keep K).  The paper
 *     starts from an approximate k-NN graph built by another method (Sec. 5.2);
 *     this build uses the exact one.
 *   - stage 1, relaxed diversification: Sec. 3.2, Eq. 2, with the checking
 *     order of Sec. 3.1 (closest first, each next edge against all kept ones).
 *   - reverse edges, then stage 2 (occlusion factor lambda by Eq. 1, sort by
 *     (lambda, distance), drop lambda > lambda0): Sec. 3.3.
 *   - search: best-first walk over one bounded sorted rank-list that serves
 *     as result list and expansion queue (the CPU procedure named in Sec. 4 /
 *     Sec. 5.3, started from 32 random seeds as in Alg. 2), visiting only the
 *     prefix of each neighbour list whose lambda is below a threshold
 *     (Sec. 3.3 last paragraph, Sec. 5.4).
 *   - recall: Eq. 3.
 *
 * Deterministic readings where the paper is silent (ties, seeds, caps) are
 * listed at each function.  Order everywhere: key (s, id), smaller id first.
 *
 * Distances are SQUARED L2.  The canonical value is
 *     s(a,b) = fl32( sum_j (double)( fl32(a_j - b_j) )^2 )
 * i.e. the difference is rounded once to fp32, its square (exact in fp64) is
 * accumulated in fp64 and the sum is rounded once to fp32.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * (closed forms, brute force written independently in numpy, invariants,
 * and hand-worked examples under tests/golden/: Eq. 1 / Eq. 2 / lambda in 2-D,
 * a hop of Alg. 2 that overflows a queue segment, two iterations of the
 * neighbourhood propagation on eight points).  No function is left unpinned.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (see build.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_F32 0
#define ORC_U8 1
#define ORC_F16 2 /* rows stored as IEEE binary16; every value converts exactly to fp32 */

typedef struct {
    float s;
    int32_t id;
} pair_t;

/* (s, id) order: smaller distance first, then smaller id. */
static int pair_less(pair_t a, pair_t b)
{
    if (a.s < b.s) return 1;
    if (a.s > b.s) return 0;
    return a.id < b.id;
}

static int pair_cmp(const void* pa, const void* pb)
{
    pair_t a = *(const pair_t*)pa, b = *(const pair_t*)pb;
    if (pair_less(a, b)) return -1;
    if (pair_less(b, a)) return 1;
    return 0;
}

/* IEEE binary16 bit pattern -> fp32 (exact): sign, 5 exponent bits (bias 15), 10 fraction bits;
 * exponent 0 = zero / subnormal (fraction * 2^-24), exponent 31 = infinity / NaN. */
float orc_half_to_float(uint16_t h)
{
    const int sign = (h >> 15) & 1, e = (h >> 10) & 31, f = h & 1023;
    float v;
    if (e == 0) v = ldexpf((float)f, -24);
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = ldexpf((float)(1024 + f), e - 25);
    return sign ? -v : v;
}

/* Row i of the base set as fp32 (uint8 and binary16 convert exactly). */
static const float* row_f32(const void* base, int dtype, int64_t i, int d, float* tmp)
{
    if (dtype == ORC_F32) return (const float*)base + i * (int64_t)d;
    if (dtype == ORC_F16) {
        const uint16_t* r = (const uint16_t*)base + i * (int64_t)d;
        for (int j = 0; j < d; ++j) tmp[j] = orc_half_to_float(r[j]);
        return tmp;
    }
    const uint8_t* r = (const uint8_t*)base + i * (int64_t)d;
    for (int j = 0; j < d; ++j) tmp[j] = (float)r[j];
    return tmp;
}

/* Canonical squared L2 distance (see the header). */
float orc_sqdist(const float* a, const float* b, int d)
{
    double acc = 0.0;
    for (int j = 0; j < d; ++j) {
        float t = a[j] - b[j];
        acc += (double)t * (double)t;
    }
    return (float)acc;
}

static float sqdist_rows(const void* base, int dtype, int d, int64_t i, int64_t j,
                         float* tmp_i, float* tmp_j)
{
    const float* a = row_f32(base, dtype, i, d, tmp_i);
    const float* b = row_f32(base, dtype, j, d, tmp_j);
    return orc_sqdist(a, b, d);
}

static int use_threads(int threads)
{
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
    return threads;
#else
    (void)threads;
    return 1;
#endif
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------
 * Exact top-k of each query against the whole base set (plain definition).
 * exclude_self != 0: query i is base row i and id i is left out (k-NN graph).
 * out_ids/out_s are [nq,k]; missing entries (N too small) are -1 / +inf.
 * ---------------------------------------------------------------------- */
int orc_bruteforce(const void* base, int dtype, int64_t N, int d,
                   const float* queries, int64_t nq, int k, int exclude_self,
                   int32_t* out_ids, float* out_s, int threads)
{
    if (!base || N <= 0 || d <= 0 || k <= 0 || nq < 0) return 1;
    threads = use_threads(threads);
    int failed = 0;
#pragma omp parallel num_threads(threads)
    {
        pair_t* all = (pair_t*)malloc(sizeof(pair_t) * (size_t)N);
        float* tq = (float*)malloc(sizeof(float) * (size_t)d);
        float* tb = (float*)malloc(sizeof(float) * (size_t)d);
        if (!all || !tq || !tb) {
#pragma omp atomic write
            failed = 1;
        } else {
#pragma omp for schedule(dynamic, 4)
            for (int64_t qi = 0; qi < nq; ++qi) {
                const float* q = exclude_self ? row_f32(base, dtype, qi, d, tq)
                                              : queries + qi * (int64_t)d;
                int64_t m = 0;
                for (int64_t j = 0; j < N; ++j) {
                    if (exclude_self && j == qi) continue;
                    const float* b = row_f32(base, dtype, j, d, tb);
                    all[m].s = orc_sqdist(q, b, d);
                    all[m].id = (int32_t)j;
                    ++m;
                }
                qsort(all, (size_t)m, sizeof(pair_t), pair_cmp);
                for (int t = 0; t < k; ++t) {
                    if (t < m) {
                        out_ids[qi * k + t] = all[t].id;
                        out_s[qi * k + t] = all[t].s;
                    } else {
                        out_ids[qi * k + t] = -1;
                        out_s[qi * k + t] = INFINITY;
                    }
                }
            }
        }
        free(all);
        free(tq);
        free(tb);
    }
    return failed ? 2 : 0;
}

/* Exact k-NN graph: row i = the K nearest other points by (s, id). */
int orc_knn(const void* base, int dtype, int64_t N, int d, int K,
            int32_t* knn_id, float* knn_s, int threads)
{
    return orc_bruteforce(base, dtype, N, d, NULL, N, K, 1, knn_id, knn_s, threads);
}

/* ------------------------------------------------------------------------
 * Stage 1 (Sec. 3.2, Eq. 2; order rule of Sec. 3.1).
 * The list of x0 is in (s,id) order.  The closest neighbour is kept; edge j
 * is dropped iff some already-kept edge i has
 *      alpha2 * s(x0,xi) < s(x0,xj)   and   alpha2 * s(xi,xj) < s(x0,xj)
 * with alpha2 = fl32(alpha*alpha) (the paper states the rule on the L2
 * distance m; squaring both sides gives alpha^2 on squared distances) and
 * each product one fp32 multiply.  Output g1_* is [N,K], kept edges first in
 * their original order, padded with -1 / +inf; g1_deg[N] = number kept.
 *
 * Cosine metric (Sec. 5, Table 1: m = Cos): rows are unit vectors (see
 * orc_normalize_rows) and m(a,b) = 1 - cos(a,b) = s(a,b)/2.  Eq. 2 is stated
 * on m itself, alpha*m(..) < m(..), and m is proportional to s, so the factor
 * on the squared distances is alpha, not alpha^2.  metric: 0 = L2, 1 = cosine.
 * ---------------------------------------------------------------------- */
int orc_stage1_m(const void* base, int dtype, int64_t N, int d, int K,
                 const int32_t* knn_id, const float* knn_s, float alpha, int metric,
                 int32_t* g1_id, float* g1_s, int32_t* g1_deg, int threads)
{
    if (!base || !knn_id || !knn_s || N <= 0 || K <= 0 || (metric != 0 && metric != 1)) return 1;
    threads = use_threads(threads);
    const float alpha2 = metric == 1 ? alpha : alpha * alpha;
#pragma omp parallel num_threads(threads)
    {
        float* ti = (float*)malloc(sizeof(float) * (size_t)d);
        float* tj = (float*)malloc(sizeof(float) * (size_t)d);
#pragma omp for schedule(dynamic, 64)
        for (int64_t x0 = 0; x0 < N; ++x0) {
            const int32_t* ids = knn_id + x0 * K;
            const float* ss = knn_s + x0 * K;
            int32_t* oid = g1_id + x0 * K;
            float* os = g1_s + x0 * K;
            int nk = 0;
            for (int j = 0; j < K; ++j) {
                if (ids[j] < 0) break;
                int occluded = 0;
                for (int t = 0; t < nk && !occluded; ++t) {
                    float s0i = os[t];
                    float s0j = ss[j];
                    if (alpha2 * s0i < s0j) {
                        float sij = sqdist_rows(base, dtype, d, oid[t], ids[j], ti, tj);
                        if (alpha2 * sij < s0j) occluded = 1;
                    }
                }
                if (!occluded) {
                    oid[nk] = ids[j];
                    os[nk] = ss[j];
                    ++nk;
                }
            }
            g1_deg[x0] = nk;
            for (int t = nk; t < K; ++t) {
                oid[t] = -1;
                os[t] = INFINITY;
            }
        }
        free(ti);
        free(tj);
    }
    return 0;
}

int orc_stage1(const void* base, int dtype, int64_t N, int d, int K,
               const int32_t* knn_id, const float* knn_s, float alpha,
               int32_t* g1_id, float* g1_s, int32_t* g1_deg, int threads)
{
    return orc_stage1_m(base, dtype, N, d, K, knn_id, knn_s, alpha, 0, g1_id, g1_s, g1_deg, threads);
}

/* ------------------------------------------------------------------------
 * Unit rows for the cosine metric.  norm = fl32( sqrt( sum (double)x_j^2 ) )
 * (the sum in fp64, in index order), out_j = fl32( (double)x_j / (double)norm );
 * a zero row stays zero.  With unit rows, 1 - cos(a,b) = s(a,b) / 2.
 * ---------------------------------------------------------------------- */
int orc_normalize_rows(const float* src, int64_t n, int d, float* dst)
{
    if (!src || !dst || n < 0 || d <= 0) return 1;
    for (int64_t i = 0; i < n; ++i) {
        double ss = 0.0;
        for (int j = 0; j < d; ++j) ss += (double)src[i * d + j] * (double)src[i * d + j];
        const float norm = (float)sqrt(ss);
        for (int j = 0; j < d; ++j)
            dst[i * d + j] = norm > 0.0f ? (float)((double)src[i * d + j] / (double)norm) : 0.0f;
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Inner product (Table 1 lists m = IP for one dataset; the paper says no more).
 * Reading: the standard reduction of maximum-inner-product search to L2.  With
 * M >= every base norm, a base row x becomes [x, sqrt(M^2 - |x|^2), 0, 0, 0]
 * and a query q becomes [q, 0, 0, 0, 0] (d + 4 columns, so rows stay 16-byte
 * multiples); then  s(q~, x~) = |q|^2 + M^2 - 2 <q,x>,  which orders the base
 * rows of one query exactly as -<q,x> does, and the graph is the L2 graph of
 * the augmented rows.  extra = fl32( sqrt( max(0, (double)M*M - sum (double)x_j^2) ) ).
 * ---------------------------------------------------------------------- */
int orc_ip_augment_rows(const float* src, int64_t n, int d, float M, int is_query, float* dst)
{
    if (!src || !dst || n < 0 || d <= 0 || (!is_query && !(M > 0.0f))) return 1;
    const int dp = d + 4;
    for (int64_t i = 0; i < n; ++i) {
        double ss = 0.0;
        for (int j = 0; j < d; ++j) {
            dst[i * dp + j] = src[i * d + j];
            ss += (double)src[i * d + j] * (double)src[i * d + j];
        }
        double rest = (double)M * (double)M - ss;
        if (rest < 0.0) rest = 0.0;
        dst[i * dp + d] = is_query ? 0.0f : (float)sqrt(rest);
        dst[i * dp + d + 1] = dst[i * dp + d + 2] = dst[i * dp + d + 3] = 0.0f;
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Reverse edges (Sec. 3.3, second sentence): list(x0) = kept(x0) united with
 * { y : x0 in kept(y) }.  Reading where the paper is silent: duplicates are
 * removed by id, the list is sorted by (s,id) with s = s(x0,y) computed
 * directly, and it is cut to rev_cap entries (hub nodes have unbounded
 * in-degree).  Output g2_* is [N,rev_cap] padded -1 / +inf, g2_deg[N].
 * ---------------------------------------------------------------------- */
int orc_reverse(const void* base, int dtype, int64_t N, int d, int K,
                const int32_t* g1_id, const int32_t* g1_deg, int rev_cap,
                int32_t* g2_id, float* g2_s, int32_t* g2_deg, int threads)
{
    if (!base || !g1_id || !g1_deg || N <= 0 || K <= 0 || rev_cap <= 0) return 1;
    threads = use_threads(threads);
    int64_t* start = (int64_t*)calloc((size_t)N + 1, sizeof(int64_t));
    if (!start) return 2;
    for (int64_t y = 0; y < N; ++y)
        for (int t = 0; t < g1_deg[y]; ++t) start[g1_id[y * K + t] + 1]++;
    for (int64_t i = 0; i < N; ++i) start[i + 1] += start[i];
    int64_t total = start[N];
    int32_t* src = (int32_t*)malloc(sizeof(int32_t) * (size_t)(total > 0 ? total : 1));
    int64_t* cur = (int64_t*)malloc(sizeof(int64_t) * (size_t)N);
    if (!src || !cur) {
        free(start); free(src); free(cur);
        return 2;
    }
    memcpy(cur, start, sizeof(int64_t) * (size_t)N);
    for (int64_t y = 0; y < N; ++y)
        for (int t = 0; t < g1_deg[y]; ++t) src[cur[g1_id[y * K + t]]++] = (int32_t)y;

#pragma omp parallel num_threads(threads)
    {
        float* ti = (float*)malloc(sizeof(float) * (size_t)d);
        float* tj = (float*)malloc(sizeof(float) * (size_t)d);
#pragma omp for schedule(dynamic, 64)
        for (int64_t x0 = 0; x0 < N; ++x0) {
            int64_t nin = start[x0 + 1] - start[x0];
            int64_t cap = g1_deg[x0] + nin;
            pair_t* lst = (pair_t*)malloc(sizeof(pair_t) * (size_t)(cap > 0 ? cap : 1));
            int64_t m = 0;
            for (int t = 0; t < g1_deg[x0]; ++t) lst[m++].id = g1_id[x0 * K + t];
            for (int64_t t = start[x0]; t < start[x0 + 1]; ++t) {
                int32_t y = src[t];
                int dup = 0;
                for (int64_t u = 0; u < m && !dup; ++u) dup = (lst[u].id == y);
                if (!dup) lst[m++].id = y;
            }
            for (int64_t t = 0; t < m; ++t)
                lst[t].s = sqdist_rows(base, dtype, d, x0, lst[t].id, ti, tj);
            qsort(lst, (size_t)m, sizeof(pair_t), pair_cmp);
            int keep = (int)(m < rev_cap ? m : rev_cap);
            for (int t = 0; t < rev_cap; ++t) {
                g2_id[x0 * rev_cap + t] = t < keep ? lst[t].id : -1;
                g2_s[x0 * rev_cap + t] = t < keep ? lst[t].s : INFINITY;
            }
            g2_deg[x0] = keep;
            free(lst);
        }
        free(ti);
        free(tj);
    }
    free(start);
    free(src);
    free(cur);
    return 0;
}

/* ------------------------------------------------------------------------
 * Stage 2 (Sec. 3.3): occlusion factor of edge j of node x0
 *   lambda_j = #{ i != j in the list : s(x0,xi) < s(x0,xj) and s(xi,xj) < s(x0,xj) }
 * (Eq. 1, counted over the whole list, strict comparisons), then the list is
 * sorted by (lambda, s, id), entries with lambda > lambda0 are removed, the
 * list is cut to K and padded with id -1 / lambda 255.
 * ---------------------------------------------------------------------- */
typedef struct {
    int32_t lam;
    float s;
    int32_t id;
} lam_t;

static int lam_cmp(const void* pa, const void* pb)
{
    const lam_t* a = (const lam_t*)pa;
    const lam_t* b = (const lam_t*)pb;
    if (a->lam != b->lam) return a->lam < b->lam ? -1 : 1;
    if (a->s < b->s) return -1;
    if (a->s > b->s) return 1;
    if (a->id != b->id) return a->id < b->id ? -1 : 1;
    return 0;
}

int orc_stage2(const void* base, int dtype, int64_t N, int d, int rev_cap,
               const int32_t* g2_id, const float* g2_s, const int32_t* g2_deg,
               int lambda0, int K, int32_t* adj, uint8_t* lam, int threads)
{
    if (!base || !g2_id || !g2_s || !g2_deg || N <= 0 || K <= 0 || rev_cap <= 0) return 1;
    threads = use_threads(threads);
#pragma omp parallel num_threads(threads)
    {
        float* ti = (float*)malloc(sizeof(float) * (size_t)d);
        float* tj = (float*)malloc(sizeof(float) * (size_t)d);
        lam_t* lst = (lam_t*)malloc(sizeof(lam_t) * (size_t)rev_cap);
#pragma omp for schedule(dynamic, 64)
        for (int64_t x0 = 0; x0 < N; ++x0) {
            const int32_t* ids = g2_id + x0 * rev_cap;
            const float* ss = g2_s + x0 * rev_cap;
            int m = g2_deg[x0];
            for (int j = 0; j < m; ++j) {
                int cnt = 0;
                for (int i = 0; i < m; ++i) {
                    if (i == j) continue;
                    if (ss[i] < ss[j]) {
                        float sij = sqdist_rows(base, dtype, d, ids[i], ids[j], ti, tj);
                        if (sij < ss[j]) ++cnt;
                    }
                }
                lst[j].lam = cnt;
                lst[j].s = ss[j];
                lst[j].id = ids[j];
            }
            qsort(lst, (size_t)m, sizeof(lam_t), lam_cmp);
            int out = 0;
            for (int j = 0; j < m && out < K; ++j) {
                if (lst[j].lam > lambda0) break;
                adj[x0 * K + out] = lst[j].id;
                lam[x0 * K + out] = (uint8_t)lst[j].lam;
                ++out;
            }
            for (; out < K; ++out) {
                adj[x0 * K + out] = -1;
                lam[x0 * K + out] = 255;
            }
        }
        free(ti);
        free(tj);
        free(lst);
    }
    return 0;
}

/* Whole build: exact k-NN -> stage 1 -> reverse edges -> stage 2.
 * Optional outputs (may be NULL): knn_id/knn_s [N,K] and g1_id [N,K],
 * g1_deg [N], g2_id/g2_s [N,rev_cap], g2_deg [N] for per-stage parity. */
int orc_build_m(const void* base, int dtype, int64_t N, int d, int K, float alpha, int metric,
                int lambda0, int rev_cap, int32_t* adj, uint8_t* lam,
                int32_t* knn_id_out, float* knn_s_out, int32_t* g1_id_out, int32_t* g1_deg_out,
                int32_t* g2_id_out, float* g2_s_out, int32_t* g2_deg_out, int threads)
{
    if (!base || !adj || !lam || N <= K || K <= 0 || rev_cap <= 0) return 1;
    size_t nk = (size_t)N * (size_t)K, nr = (size_t)N * (size_t)rev_cap;
    int32_t* knn_id = (int32_t*)malloc(sizeof(int32_t) * nk);
    float* knn_s = (float*)malloc(sizeof(float) * nk);
    int32_t* g1_id = (int32_t*)malloc(sizeof(int32_t) * nk);
    float* g1_s = (float*)malloc(sizeof(float) * nk);
    int32_t* g1_deg = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    int32_t* g2_id = (int32_t*)malloc(sizeof(int32_t) * nr);
    float* g2_s = (float*)malloc(sizeof(float) * nr);
    int32_t* g2_deg = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    int rc = 2;
    if (knn_id && knn_s && g1_id && g1_s && g1_deg && g2_id && g2_s && g2_deg) {
        rc = orc_knn(base, dtype, N, d, K, knn_id, knn_s, threads);
        if (!rc) rc = orc_stage1_m(base, dtype, N, d, K, knn_id, knn_s, alpha, metric, g1_id, g1_s, g1_deg, threads);
        if (!rc) rc = orc_reverse(base, dtype, N, d, K, g1_id, g1_deg, rev_cap, g2_id, g2_s, g2_deg, threads);
        if (!rc) rc = orc_stage2(base, dtype, N, d, rev_cap, g2_id, g2_s, g2_deg, lambda0, K, adj, lam, threads);
        if (!rc) {
            if (knn_id_out) memcpy(knn_id_out, knn_id, sizeof(int32_t) * nk);
            if (knn_s_out) memcpy(knn_s_out, knn_s, sizeof(float) * nk);
            if (g1_id_out) memcpy(g1_id_out, g1_id, sizeof(int32_t) * nk);
            if (g1_deg_out) memcpy(g1_deg_out, g1_deg, sizeof(int32_t) * (size_t)N);
            if (g2_id_out) memcpy(g2_id_out, g2_id, sizeof(int32_t) * nr);
            if (g2_s_out) memcpy(g2_s_out, g2_s, sizeof(float) * nr);
            if (g2_deg_out) memcpy(g2_deg_out, g2_deg, sizeof(int32_t) * (size_t)N);
        }
    }
    free(knn_id); free(knn_s); free(g1_id); free(g1_s); free(g1_deg);
    free(g2_id); free(g2_s); free(g2_deg);
    return rc;
}

int orc_build(const void* base, int dtype, int64_t N, int d, int K, float alpha,
              int lambda0, int rev_cap, int32_t* adj, uint8_t* lam,
              int32_t* knn_id_out, float* knn_s_out, int32_t* g1_id_out, int32_t* g1_deg_out,
              int32_t* g2_id_out, float* g2_s_out, int32_t* g2_deg_out, int threads)
{
    return orc_build_m(base, dtype, N, d, K, alpha, 0, lambda0, rev_cap, adj, lam, knn_id_out, knn_s_out,
                       g1_id_out, g1_deg_out, g2_id_out, g2_s_out, g2_deg_out, threads);
}

/* ------------------------------------------------------------------------
 * Seed generator.  The paper draws 32 random start nodes (Alg. 2, first
 * line) and names no generator.  Reading: a counter-based one, so the seeds
 * of query qi do not depend on scheduling.  Seed j of query qi:
 *     x = seed + GOLDEN*(qi*2^32 + j + 1)            (mod 2^64)
 *     x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9
 *     x = (x ^ (x >> 27)) * 0x94D049BB133111EB
 *     x =  x ^ (x >> 31)
 *     id = floor( x * N / 2^64 )                      (high half of the product)
 * GOLDEN = 0x9E3779B97F4A7C15.  (The three-step finaliser is the published
 * splitmix64 output function.)
 * ---------------------------------------------------------------------- */
int64_t orc_seed_id(uint64_t seed, uint64_t qi, uint64_t j, int64_t N)
{
    uint64_t x = seed + 0x9E3779B97F4A7C15ULL * ((qi << 32) + j + 1ULL);
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ULL;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBULL;
    x = x ^ (x >> 31);
    return (int64_t)(((unsigned __int128)x * (unsigned __int128)(uint64_t)N) >> 64);
}

/* ------------------------------------------------------------------------
 * Best-first search of one query over the diversified graph.
 *
 * One sorted list of at most L entries (s, id, expanded) is both the result
 * list and the expansion queue.
 *   1. the n_seeds seed nodes (repeats skipped) are scored and inserted;
 *   2. u = first entry not yet expanded; none -> stop; hop limit T reached
 *      (max_hops > 0 and hops == max_hops) -> stop; mark u expanded;
 *   3. the neighbours of u are taken in stored order while id >= 0 and
 *      lambda < lambda_visit (prefix rule of Sec. 3.3 / Sec. 5.4); one already
 *      visited is skipped; otherwise it is marked visited, scored, and
 *      inserted if the list has room or (s,id) precedes the last entry; the
 *      last entry is dropped when the list exceeds L; an id already present
 *      in the list is never inserted twice;
 *   4. the first k entries are returned (id -1 / s +inf when fewer exist).
 *
 * visited_cap == 0: exact visited bitmap.  visited_cap > 0: a lossy
 * direct-mapped table of that many slots (id % cap, overwritten on conflict)
 * -- results must not depend on it; only the evaluation counts do.
 * reverse_hop != 0 scores each hop's neighbours in reverse stored order --
 * results must not depend on that either.
 * ---------------------------------------------------------------------- */
typedef struct {
    float s;
    int32_t id;
    int expanded;
} entry_t;

static void search_one(const int32_t* adj, const uint8_t* lam, int64_t N, int K,
                       const void* base, int dtype, int d, const float* q, int k, int L,
                       int lambda_visit, int n_seeds, uint64_t seed, uint64_t qi,
                       int max_hops, int visited_cap, int reverse_hop,
                       uint8_t* bitmap, int32_t* vtab, entry_t* lst, float* tmp,
                       int32_t* out_ids, float* out_s, uint32_t* stats,
                       int32_t* trace, int trace_cap)
{
    int n = 0;
    uint32_t hops = 0, evals = 0, dedup = 0;
    if (visited_cap == 0) memset(bitmap, 0, (size_t)((N + 7) / 8));
    else for (int t = 0; t < visited_cap; ++t) vtab[t] = -1;

    /* returns 1 if e was already visited, else marks it and returns 0 */
#define VISIT(e, was)                                                        \
    do {                                                                     \
        if (visited_cap == 0) {                                              \
            was = (bitmap[(e) >> 3] >> ((e) & 7)) & 1;                       \
            bitmap[(e) >> 3] |= (uint8_t)(1u << ((e) & 7));                  \
        } else {                                                             \
            was = (vtab[(e) % visited_cap] == (e));                          \
            vtab[(e) % visited_cap] = (e);                                   \
        }                                                                    \
    } while (0)

#define SCORE_AND_INSERT(e)                                                  \
    do {                                                                     \
        const float* xb = row_f32(base, dtype, (e), d, tmp);                 \
        pair_t c;                                                            \
        c.s = orc_sqdist(q, xb, d);                                          \
        c.id = (e);                                                          \
        ++evals;                                                             \
        int present = 0;                                                     \
        for (int t = 0; t < n && !present; ++t) present = (lst[t].id == c.id); \
        if (!present) {                                                      \
            pair_t last = {0.0f, -1};                                        \
            if (n > 0) { last.s = lst[n - 1].s; last.id = lst[n - 1].id; }   \
            if (n < L || pair_less(c, last)) {                               \
                int pos = n;                                                 \
                while (pos > 0) {                                            \
                    pair_t p; p.s = lst[pos - 1].s; p.id = lst[pos - 1].id;  \
                    if (pair_less(c, p)) --pos; else break;                  \
                }                                                            \
                int end = n < L ? n : L - 1;                                 \
                for (int t = end; t > pos; --t) lst[t] = lst[t - 1];         \
                lst[pos].s = c.s; lst[pos].id = c.id; lst[pos].expanded = 0; \
                if (n < L) ++n;                                              \
            }                                                                \
        }                                                                    \
    } while (0)

    for (int j = 0; j < n_seeds; ++j) {
        int32_t e = (int32_t)orc_seed_id(seed, qi, (uint64_t)j, N);
        int was;
        VISIT(e, was);
        if (was) { ++dedup; continue; }
        SCORE_AND_INSERT(e);
    }
    for (;;) {
        int ui = -1;
        for (int t = 0; t < n; ++t)
            if (!lst[t].expanded) { ui = t; break; }
        if (ui < 0) break;
        if (max_hops > 0 && (int)hops == max_hops) break;
        lst[ui].expanded = 1;
        int32_t u = lst[ui].id;
        if (trace && (int)hops < trace_cap) trace[hops] = u;
        ++hops;
        int deg = 0;
        while (deg < K && adj[(int64_t)u * K + deg] >= 0 &&
               (int)lam[(int64_t)u * K + deg] < lambda_visit) ++deg;
        for (int t = 0; t < deg; ++t) {
            int tt = reverse_hop ? deg - 1 - t : t;
            int32_t e = adj[(int64_t)u * K + tt];
            int was;
            VISIT(e, was);
            if (was) { ++dedup; continue; }
            SCORE_AND_INSERT(e);
        }
    }
    for (int t = 0; t < k; ++t) {
        out_ids[t] = t < n ? lst[t].id : -1;
        out_s[t] = t < n ? lst[t].s : INFINITY;
    }
    if (stats) { stats[0] = hops; stats[1] = evals; stats[2] = dedup; }
#undef VISIT
#undef SCORE_AND_INSERT
}

/* Batch of queries.  out_ids/out_s [nq,k]; stats (may be NULL) [nq,3] =
 * hops, distance evaluations, visited hits.  trace (may be NULL) [nq,trace_cap]
 * receives the ids expanded, in order (unused slots untouched). */
int orc_search(const int32_t* adj, const uint8_t* lam, int64_t N, int K,
               const void* base, int dtype, int d, const float* queries, int64_t nq,
               int k, int L, int lambda_visit, int n_seeds, uint64_t seed, int max_hops,
               int visited_cap, int reverse_hop, int64_t qi_offset,
               int32_t* out_ids, float* out_s, uint32_t* stats,
               int32_t* trace, int trace_cap, int threads)
{
    if (!adj || !lam || !base || !queries || !out_ids || !out_s) return 1;
    if (N <= 0 || K <= 0 || d <= 0 || k <= 0 || L < k || n_seeds <= 0 || nq < 0) return 1;
    threads = use_threads(threads);
    int failed = 0;
#pragma omp parallel num_threads(threads)
    {
        uint8_t* bitmap = visited_cap == 0 ? (uint8_t*)malloc((size_t)((N + 7) / 8)) : NULL;
        int32_t* vtab = visited_cap > 0 ? (int32_t*)malloc(sizeof(int32_t) * (size_t)visited_cap) : NULL;
        entry_t* lst = (entry_t*)malloc(sizeof(entry_t) * (size_t)L);
        float* tmp = (float*)malloc(sizeof(float) * (size_t)d);
        if ((visited_cap == 0 && !bitmap) || (visited_cap > 0 && !vtab) || !lst || !tmp) {
#pragma omp atomic write
            failed = 1;
        } else {
#pragma omp for schedule(dynamic, 8)
            for (int64_t qi = 0; qi < nq; ++qi) {
                search_one(adj, lam, N, K, base, dtype, d, queries + qi * (int64_t)d, k, L,
                           lambda_visit, n_seeds, seed, (uint64_t)(qi + qi_offset), max_hops,
                           visited_cap, reverse_hop, bitmap, vtab, lst, tmp,
                           out_ids + qi * k, out_s + qi * k, stats ? stats + qi * 3 : NULL,
                           trace ? trace + qi * (int64_t)trace_cap : NULL, trace_cap);
            }
        }
        free(bitmap);
        free(vtab);
        free(lst);
        free(tmp);
    }
    return failed ? 2 : 0;
}

/* ------------------------------------------------------------------------
 * Small-batch multi-search (Alg. 1 with the merge described in Sec. 4.1).
 *
 * For one query, t0 independent greedy searches are run and their rankings
 * merged.  Search j:
 *   - U = 32 start nodes, seed numbers 32*j .. 32*j+31 of the query; all are
 *     scored and u = the closest by (s,id);  R (32 slots) starts empty;
 *   - while improved and hops < T:
 *       R_temp = 32 empty slots; the neighbours of u are taken in stored order
 *       over the prefix with lambda < lambda_visit; the neighbour at position
 *       p competes only for slot p mod 32 and replaces it when its (s,id) is
 *       smaller ("every 32 neighbours ... R_temp[warp_id]");
 *       update: R <- sort( R[0..16) united with the 16 smallest of R_temp ),
 *       cut to 32 ("the last 16 elements of R are replaced with the top-16
 *       of R_temp", then a complete sort);
 *       u <- the closest node in R_temp;  no neighbours at all -> stop.
 *   - readings where the listing is silent: an id already among the kept 16 is
 *     not entered twice; "R is not updated" means that no id entered the first
 *     16 entries of R that was not among them before the update; order is
 *     (s,id) as everywhere.
 * The t0 rankings are united, repeated ids removed, sorted by (s,id) and cut
 * to k (k <= 32).  stats (may be NULL) [nq,3]: hops summed over the searches,
 * distance evaluations (seeds included), 0.
 * ---------------------------------------------------------------------- */
static int greedy_one(const int32_t* adj, const uint8_t* lam, int64_t N, int K, const void* base,
                      int dtype, int d, const float* q, int lambda_visit, uint64_t seed,
                      uint64_t qi, int j, int T, float* tmp, pair_t* R, uint32_t* hops_out,
                      uint32_t* evals_out)
{
    int nR = 0;
    pair_t best;
    best.s = INFINITY;
    best.id = -1;
    for (int t = 0; t < 32; ++t) {
        pair_t c;
        c.id = (int32_t)orc_seed_id(seed, qi, (uint64_t)(32 * j + t), N);
        c.s = orc_sqdist(q, row_f32(base, dtype, c.id, d, tmp), d);
        ++*evals_out;
        if (best.id < 0 || pair_less(c, best)) best = c;
    }
    int32_t u = best.id;
    int improved = 1, hops = 0;
    while (improved && hops < T) {
        pair_t Rt[32];
        int used[32];
        for (int t = 0; t < 32; ++t) used[t] = 0;
        int deg = 0;
        while (deg < K && adj[(int64_t)u * K + deg] >= 0 && (int)lam[(int64_t)u * K + deg] < lambda_visit) ++deg;
        for (int p = 0; p < deg; ++p) {
            pair_t c;
            c.id = adj[(int64_t)u * K + p];
            c.s = orc_sqdist(q, row_f32(base, dtype, c.id, d, tmp), d);
            ++*evals_out;
            int slot = p % 32;
            if (!used[slot] || pair_less(c, Rt[slot])) { Rt[slot] = c; used[slot] = 1; }
        }
        ++hops;
        pair_t cand[32];
        int nc = 0;
        for (int t = 0; t < 32; ++t) if (used[t]) cand[nc++] = Rt[t];
        if (nc == 0) break;
        qsort(cand, (size_t)nc, sizeof(pair_t), pair_cmp);
        int take = nc < 16 ? nc : 16;
        int keep = nR < 16 ? nR : 16;
        pair_t merged[32];
        int nm = 0;
        for (int t = 0; t < keep; ++t) merged[nm++] = R[t];
        for (int t = 0; t < take; ++t) {
            int dupl = 0;
            for (int a = 0; a < keep && !dupl; ++a) dupl = (R[a].id == cand[t].id);
            if (!dupl) merged[nm++] = cand[t];
        }
        qsort(merged, (size_t)nm, sizeof(pair_t), pair_cmp);
        improved = 0;
        int top = nm < 16 ? nm : 16;
        for (int t = 0; t < top && !improved; ++t) {
            int was = 0;
            for (int a = 0; a < keep && !was; ++a) was = (R[a].id == merged[t].id);
            if (!was) improved = 1;
        }
        nR = nm;
        for (int t = 0; t < nm; ++t) R[t] = merged[t];
        u = cand[0].id;
    }
    *hops_out += (uint32_t)hops;
    return nR;
}

int orc_search_multi(const int32_t* adj, const uint8_t* lam, int64_t N, int K, const void* base, int dtype,
                     int d, const float* queries, int64_t nq, int k, int t0, int T, int lambda_visit,
                     uint64_t seed, int64_t qi_offset, int32_t* out_ids, float* out_s, uint32_t* stats,
                     int threads)
{
    if (!adj || !lam || !base || !queries || !out_ids || !out_s) return 1;
    if (N <= 0 || K <= 0 || d <= 0 || k <= 0 || k > 32 || t0 <= 0 || T < 0 || nq < 0) return 1;
    threads = use_threads(threads);
    int failed = 0;
#pragma omp parallel num_threads(threads)
    {
        float* tmp = (float*)malloc(sizeof(float) * (size_t)d);
        pair_t* all = (pair_t*)malloc(sizeof(pair_t) * (size_t)t0 * 32);
        if (!tmp || !all) {
#pragma omp atomic write
            failed = 1;
        } else {
#pragma omp for schedule(dynamic, 8)
            for (int64_t qi = 0; qi < nq; ++qi) {
                const float* q = queries + qi * (int64_t)d;
                uint32_t hops = 0, evals = 0;
                int n = 0;
                for (int j = 0; j < t0; ++j)
                    n += greedy_one(adj, lam, N, K, base, dtype, d, q, lambda_visit, seed,
                                    (uint64_t)(qi + qi_offset), j, T, tmp, all + n, &hops, &evals);
                qsort(all, (size_t)n, sizeof(pair_t), pair_cmp);
                int out = 0;
                for (int t = 0; t < n && out < k; ++t) {
                    if (t > 0 && all[t].id == all[t - 1].id) continue; /* same id => same key: adjacent */
                    out_ids[qi * k + out] = all[t].id;
                    out_s[qi * k + out] = all[t].s;
                    ++out;
                }
                for (; out < k; ++out) {
                    out_ids[qi * k + out] = -1;
                    out_s[qi * k + out] = INFINITY;
                }
                if (stats) { stats[qi * 3] = hops; stats[qi * 3 + 1] = evals; stats[qi * 3 + 2] = 0; }
            }
        }
        free(tmp);
        free(all);
    }
    return failed ? 2 : 0;
}

/* ------------------------------------------------------------------------
 * Large-batch search with the paper's own structures (Alg. 2 and Sec. 4.2).
 * The loop below takes the listing's statements in the listing's order; this
 * comment only says how its three containers are represented and which
 * readings were taken where the text is silent.
 *
 * R  top ranking array: at most k pairs sorted by (s,id); a push beyond k
 *    removes the furthest.
 * C  expansion queue: m_c segments of at most 32 pairs, each sorted by (s,id);
 *    a pair goes to segment id % m_c; a push into a full segment drops that
 *    segment's most distant pair (possibly the pushed one); pop = the smallest
 *    of the segment heads.
 * V  look-up table: m_v segments of 32 ids written round-robin (the oldest is
 *    overwritten), segment id % m_v; only expanded nodes enter it.
 *
 * Order of the look-ups: the listing tests "e in V, e in C" for one neighbour
 * at a time, after the pushes of the neighbours before it, and so does this
 * loop.  It matters when an earlier neighbour's push into a full segment drops
 * a later neighbour of the same node from C: at its turn that neighbour is in
 * neither container, so it is scored again.  It is never pushed again (it
 * entered R together with C; either R still holds it, or R dropped it as its
 * furthest and every later furthest is at most as far, so the strict test
 * fails), hence R, C and V are what look-ups made before the hop's pushes
 * would give; only the two counters differ, by one each per such event.
 *
 * Readings where the paper is silent:
 *   - the stop test compares the measure m of Table 1, not its square:
 *     L2 (metric 0): m = sqrt(s), stop iff sqrt(s_u) > sqrt(s_f) + Delta.  To keep
 *     every operation a correctly rounded IEEE one (no square root), the test is
 *     taken in the equivalent form, all in fp64:
 *         t = (s_u - s_f) - Delta*Delta;   stop iff t > 0 and t*t > (4*(Delta*Delta))*s_f
 *     (both sides of sqrt(s_u) - sqrt(s_f) > Delta are squared twice; Delta >= 0).
 *     1 - cos on unit rows (metric 1): m = s/2, stop iff s_u > s_f + 2*Delta in fp32;
 *   - an id already in R is pushed neither to R nor to C (R would hold it twice);
 *   - all orders are (s,id); T = 0 means no hop limit.
 * stats [nq,3]: hops t, distance evaluations (seeds included), skips by V or C.
 * ---------------------------------------------------------------------- */
typedef struct {
    pair_t e[32];
    int n;
} cseg_t;

/* stop test of Alg. 2 on the measure itself (see above) */
int orc_alg2_stop(float s_u, float s_f, float delta, int metric)
{
    if (metric == 1) return s_u > s_f + 2.0f * delta;
    const double dd = (double)delta * (double)delta;
    const double t = ((double)s_u - (double)s_f) - dd;
    return t > 0.0 && t * t > (4.0 * dd) * (double)s_f;
}

static void alg2_one(const int32_t* adj, const uint8_t* lam, int64_t N, int K, const void* base, int dtype,
                     int d, const float* q, int k, int m_c, int m_v, float delta, int metric, int T,
                     int lambda_visit, uint64_t seed, uint64_t qi, cseg_t* C, int32_t* V, int* vpos, pair_t* R,
                     float* tmp, int32_t* out_ids, float* out_s, uint32_t* stats)
{
    uint32_t hops = 0, evals = 0, skips = 0;
    int nR = 0;
    for (int g = 0; g < m_c; ++g) C[g].n = 0;
    for (int g = 0; g < m_v * 32; ++g) V[g] = -1;
    for (int g = 0; g < m_v; ++g) vpos[g] = 0;
    pair_t best;
    best.s = INFINITY;
    best.id = -1;
    for (int t = 0; t < 32; ++t) {
        pair_t c;
        c.id = (int32_t)orc_seed_id(seed, qi, (uint64_t)t, N);
        c.s = orc_sqdist(q, row_f32(base, dtype, c.id, d, tmp), d);
        ++evals;
        if (best.id < 0 || pair_less(c, best)) best = c;
    }
    R[nR++] = best;
    C[best.id % m_c].e[0] = best;
    C[best.id % m_c].n = 1;
    for (;;) {
        if (T > 0 && (int)hops >= T) break;
        int gbest = -1;
        for (int g = 0; g < m_c; ++g)
            if (C[g].n > 0 && (gbest < 0 || pair_less(C[g].e[0], C[gbest].e[0]))) gbest = g;
        if (gbest < 0) break;
        ++hops;
        pair_t u = C[gbest].e[0];
        for (int t = 1; t < C[gbest].n; ++t) C[gbest].e[t - 1] = C[gbest].e[t];
        --C[gbest].n;
        if (orc_alg2_stop(u.s, R[nR - 1].s, delta, metric)) break;
        int gv = u.id % m_v;
        V[gv * 32 + vpos[gv]] = u.id;
        vpos[gv] = (vpos[gv] + 1) % 32;
        for (int p = 0; p < K; ++p) {
            const int32_t e = adj[(int64_t)u.id * K + p];
            if (e < 0 || (int)lam[(int64_t)u.id * K + p] >= lambda_visit) break; /* the visited prefix ends */
            int found = 0;
            for (int t = 0; t < 32 && !found; ++t) found = (V[(e % m_v) * 32 + t] == e);
            cseg_t* sg = &C[e % m_c];
            for (int t = 0; t < sg->n && !found; ++t) found = (sg->e[t].id == e);
            if (found) { ++skips; continue; }
            pair_t c;
            c.id = e;
            c.s = orc_sqdist(q, row_f32(base, dtype, e, d, tmp), d);
            ++evals;
            if (!(nR < k || c.s < R[nR - 1].s)) continue;
            int inR = 0;
            for (int t = 0; t < nR && !inR; ++t) inR = (R[t].id == c.id);
            if (inR) continue;
            /* R.push, drop the furthest when over k */
            int pos = nR;
            while (pos > 0 && pair_less(c, R[pos - 1])) --pos;
            int end = nR < k ? nR : k - 1;
            for (int t = end; t > pos; --t) R[t] = R[t - 1];
            if (pos < k) R[pos] = c;
            if (nR < k) ++nR;
            /* C.push into its segment, drop that segment's most distant when over 32 */
            pos = sg->n;
            while (pos > 0 && pair_less(c, sg->e[pos - 1])) --pos;
            end = sg->n < 32 ? sg->n : 31;
            for (int t = end; t > pos; --t) sg->e[t] = sg->e[t - 1];
            if (pos < 32) sg->e[pos] = c;
            if (sg->n < 32) ++sg->n;
        }
    }
    for (int t = 0; t < k; ++t) {
        out_ids[t] = t < nR ? R[t].id : -1;
        out_s[t] = t < nR ? R[t].s : INFINITY;
    }
    if (stats) { stats[0] = hops; stats[1] = evals; stats[2] = skips; }
}

int orc_search_alg2(const int32_t* adj, const uint8_t* lam, int64_t N, int K, const void* base, int dtype, int d,
                    const float* queries, int64_t nq, int k, int m_c, int m_v, float delta, int metric, int T,
                    int lambda_visit, uint64_t seed, int64_t qi_offset, int32_t* out_ids, float* out_s,
                    uint32_t* stats, int threads)
{
    if (!adj || !lam || !base || !queries || !out_ids || !out_s) return 1;
    if (N <= 0 || K <= 0 || d <= 0 || k <= 0 || m_c <= 0 || m_v <= 0 || T < 0 || nq < 0 || !(delta >= 0.0f)) return 1;
    if (metric != 0 && metric != 1) return 1;
    threads = use_threads(threads);
    int failed = 0;
#pragma omp parallel num_threads(threads)
    {
        cseg_t* C = (cseg_t*)malloc(sizeof(cseg_t) * (size_t)m_c);
        int32_t* V = (int32_t*)malloc(sizeof(int32_t) * (size_t)m_v * 32);
        int* vpos = (int*)malloc(sizeof(int) * (size_t)m_v);
        pair_t* R = (pair_t*)malloc(sizeof(pair_t) * (size_t)(k + 1));
        float* tmp = (float*)malloc(sizeof(float) * (size_t)d);
        if (!C || !V || !vpos || !R || !tmp) {
#pragma omp atomic write
            failed = 1;
        } else {
#pragma omp for schedule(dynamic, 8)
            for (int64_t qi = 0; qi < nq; ++qi)
                alg2_one(adj, lam, N, K, base, dtype, d, queries + qi * (int64_t)d, k, m_c, m_v, delta, metric, T,
                         lambda_visit, seed, (uint64_t)(qi + qi_offset), C, V, vpos, R, tmp, out_ids + qi * k,
                         out_s + qi * k, stats ? stats + qi * 3 : NULL);
        }
        free(C); free(V); free(vpos); free(R); free(tmp);
    }
    return failed ? 2 : 0;
}

/* Recall@k (Eq. 3): found[nq,k] against truth[nq,k]; -1 entries never match. */
/* ------------------------------------------------------------------------
 * Approximate k-NN graph by neighbourhood propagation.
 *
 * Sec. 3 (opening) starts from an approximate k-NN graph and names no builder.
 * This one follows the published NN-descent idea -- a neighbour of a neighbour
 * is likely a neighbour; only edges that are new since they were last looked
 * at need looking at again; both directions of an edge count -- in a form in
 * which every node PULLS its candidates from the lists as they stood before
 * the iteration, so that the result does not depend on any order of execution.
 *
 * State: list B[v] of K entries (s, id, new-flag), sorted by (s,id), ids
 * distinct and != v.  S (a power of two, 2..16) is the sample size.
 *
 * Start: draw c_j = seed_id(seed, v, j), j = 0..2K-1 (the generator of the
 * search's seeds), drop v itself and repeats, keep the first K in draw order;
 * score, sort, flag all as new.  (Or the caller's lists, all flagged new.)
 *
 * One iteration, everything read from the lists B of the previous iteration:
 *   newF[v] = the first S entries of B[v], in list order, that are flagged new;
 *   oldF[v] = the first S that are not.
 *   Reverse samples: tables Rnew[w][0..S), Rold[w][0..S), empty at first.  For
 *   every u and every w in newF[u]:  slot = (uint32(u) * 2654435761) >> (32 - log2 S);
 *   Rnew[w][slot] keeps the smallest key (s(u,w), u) offered to it.  Rold
 *   likewise from oldF.  (A fixed-size sample of the reverse edges that does
 *   not depend on the order in which they are offered.)
 *   Node a: L = B[a] with the entries of newF[a] now flagged old (they have
 *   been sampled).  Sources, in this order: newF[a] (edge new), oldF[a] (edge
 *   old), the ids in Rnew[a] by slot (edge new), the ids in Rold[a] (edge old).
 *   From source v the candidates are newF[v], the ids in Rnew[v], and, when the
 *   edge a-v is new, also oldF[v] and the ids in Rold[v]  (a pair is looked at
 *   when at least one of its two edges to the common neighbour is new).  Every
 *   candidate b != a is scored with the canonical distance and put into L
 *   (bounded K, order (s,id), an id already in L is left as it is), flagged new.
 *   B'[a] = L;  changed += entries of B'[a] that were not in B[a].
 * Stop after max_iters iterations or when changed <= delta * N * K.
 *
 * The final list is the K smallest of B[a] united with the scored candidates,
 * whatever the order, so a parallel implementation reproduces it exactly.
 * ---------------------------------------------------------------------- */
typedef struct {
    float s;
    int32_t id;
    int32_t is_new;
} dnode_t;

static int dnode_less(float s, int32_t id, const dnode_t* b)
{
    if (s != b->s) return s < b->s;
    return id < b->id;
}

/* insert (s,id) flagged new into the sorted list l[0..*m) of capacity K; returns 1 if it went in */
static int dlist_insert(dnode_t* l, int* m, int K, float s, int32_t id)
{
    for (int t = 0; t < *m; ++t)
        if (l[t].id == id) return 0;
    if (*m == K && !dnode_less(s, id, &l[K - 1])) return 0;
    int pos = *m < K ? *m : K - 1;
    while (pos > 0 && dnode_less(s, id, &l[pos - 1])) {
        l[pos] = l[pos - 1];
        --pos;
    }
    l[pos].s = s;
    l[pos].id = id;
    l[pos].is_new = 1;
    if (*m < K) ++*m;
    return 1;
}

/* slot of source u in a reverse table of S = 2^log2s cells: the top log2s bits of u * 2654435761 mod 2^32 */
uint32_t orc_descent_slot(uint32_t u, int log2s)
{
    return (uint32_t)(u * 2654435761u) >> (32 - log2s);
}

int orc_knn_descent(const void* base, int dtype, int64_t N, int d, int K, int S, int max_iters, float delta,
                    uint64_t seed, const int32_t* init_ids, int32_t* knn_id, float* knn_s,
                    int32_t* iters_done, int64_t* changed_per_iter, int threads)
{
    if (!base || !knn_id || !knn_s || N <= K || K <= 0 || d <= 0 || max_iters < 0) return 1;
    if (S < 2 || S > 16 || (S & (S - 1)) != 0) return 1;
    threads = use_threads(threads);
    int log2s = 0;
    while ((1 << log2s) < S) ++log2s;
    const size_t nk = (size_t)N * (size_t)K, ns = (size_t)N * (size_t)S;
    dnode_t* B = (dnode_t*)malloc(sizeof(dnode_t) * nk);
    dnode_t* B2 = (dnode_t*)malloc(sizeof(dnode_t) * nk);
    int32_t* cnt = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    int32_t* cnt2 = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    pair_t* Rnew = (pair_t*)malloc(sizeof(pair_t) * ns);
    pair_t* Rold = (pair_t*)malloc(sizeof(pair_t) * ns);
    if (!B || !B2 || !cnt || !cnt2 || !Rnew || !Rold) {
        free(B); free(B2); free(cnt); free(cnt2); free(Rnew); free(Rold);
        return 2;
    }
    /* ---- start lists */
#pragma omp parallel num_threads(threads)
    {
        float* ta = (float*)malloc(sizeof(float) * (size_t)d);
        float* tb = (float*)malloc(sizeof(float) * (size_t)d);
#pragma omp for schedule(dynamic, 256)
        for (int64_t v = 0; v < N; ++v) {
            dnode_t* l = B + v * K;
            int m = 0;
            if (init_ids) {
                for (int t = 0; t < K; ++t) {
                    int32_t c = init_ids[v * K + t];
                    if (c >= 0 && c != v) dlist_insert(l, &m, K, sqdist_rows(base, dtype, d, v, c, ta, tb), c);
                }
            } else {
                int32_t picked[128];
                int np = 0;
                for (int j = 0; j < 2 * K && np < K; ++j) {
                    int32_t c = (int32_t)orc_seed_id(seed, (uint64_t)v, (uint64_t)j, N);
                    int seen = c == v;
                    for (int t = 0; t < np && !seen; ++t) seen = picked[t] == c;
                    if (!seen) picked[np++] = c;
                }
                for (int t = 0; t < np; ++t)
                    dlist_insert(l, &m, K, sqdist_rows(base, dtype, d, v, picked[t], ta, tb), picked[t]);
            }
            cnt[v] = m;
        }
        free(ta);
        free(tb);
    }
    int it = 0;
    for (; it < max_iters; ++it) {
        /* ---- reverse samples from the forward samples of the lists as they stand */
        for (size_t i = 0; i < ns; ++i) {
            Rnew[i].id = -1; Rnew[i].s = INFINITY;
            Rold[i].id = -1; Rold[i].s = INFINITY;
        }
        for (int64_t u = 0; u < N; ++u) {
            const uint32_t slot = orc_descent_slot((uint32_t)u, log2s);
            int nn = 0, no = 0;
            for (int t = 0; t < cnt[u]; ++t) {
                const dnode_t* e = &B[u * K + t];
                pair_t k;
                k.s = e->s;
                k.id = (int32_t)u;
                pair_t* tab = NULL;
                if (e->is_new && nn < S) { tab = Rnew; ++nn; }
                else if (!e->is_new && no < S) { tab = Rold; ++no; }
                if (!tab) continue;
                pair_t* cell = &tab[(size_t)e->id * S + slot];
                if (cell->id < 0 || pair_less(k, *cell)) *cell = k;
            }
        }
        /* ---- every node pulls */
        int64_t changed = 0;
#pragma omp parallel num_threads(threads) reduction(+ : changed)
        {
            float* ta = (float*)malloc(sizeof(float) * (size_t)d);
            float* tb = (float*)malloc(sizeof(float) * (size_t)d);
#pragma omp for schedule(dynamic, 64)
            for (int64_t a = 0; a < N; ++a) {
                dnode_t* L = B2 + a * K;
                int m = cnt[a];
                int32_t src[64];
                int src_new[64];
                int nsrc = 0, nn = 0, no = 0;
                for (int t = 0; t < m; ++t) L[t] = B[a * K + t];
                for (int t = 0; t < m; ++t)       /* newF[a], sampled now: flagged old in L */
                    if (B[a * K + t].is_new && nn < S) { src[nsrc] = B[a * K + t].id; src_new[nsrc++] = 1; L[t].is_new = 0; ++nn; }
                for (int t = 0; t < m; ++t)
                    if (!B[a * K + t].is_new && no < S) { src[nsrc] = B[a * K + t].id; src_new[nsrc++] = 0; ++no; }
                for (int t = 0; t < S; ++t)
                    if (Rnew[(size_t)a * S + t].id >= 0) { src[nsrc] = Rnew[(size_t)a * S + t].id; src_new[nsrc++] = 1; }
                for (int t = 0; t < S; ++t)
                    if (Rold[(size_t)a * S + t].id >= 0) { src[nsrc] = Rold[(size_t)a * S + t].id; src_new[nsrc++] = 0; }
                for (int q = 0; q < nsrc; ++q) {
                    const int64_t v = src[q];
                    int32_t cand[64];
                    int nc = 0, vn = 0, vo = 0;
                    for (int t = 0; t < cnt[v]; ++t) {
                        const dnode_t* e = &B[v * K + t];
                        if (e->is_new && vn < S) { cand[nc++] = e->id; ++vn; }
                        else if (!e->is_new && vo < S) { if (src_new[q]) cand[nc++] = e->id; ++vo; }
                    }
                    for (int t = 0; t < S; ++t)
                        if (Rnew[(size_t)v * S + t].id >= 0) cand[nc++] = Rnew[(size_t)v * S + t].id;
                    if (src_new[q])
                        for (int t = 0; t < S; ++t)
                            if (Rold[(size_t)v * S + t].id >= 0) cand[nc++] = Rold[(size_t)v * S + t].id;
                    for (int t = 0; t < nc; ++t) {
                        if (cand[t] == a) continue;
                        int present = 0;
                        for (int z = 0; z < m && !present; ++z) present = L[z].id == cand[t];
                        if (present) continue;
                        float s = sqdist_rows(base, dtype, d, a, cand[t], ta, tb);
                        dlist_insert(L, &m, K, s, cand[t]);
                    }
                }
                cnt2[a] = m;
                for (int t = 0; t < m; ++t) {
                    int was = 0;
                    for (int z = 0; z < cnt[a] && !was; ++z) was = B[a * K + z].id == L[t].id;
                    changed += !was;
                }
            }
            free(ta);
            free(tb);
        }
        { dnode_t* tmp = B; B = B2; B2 = tmp; }
        { int32_t* tmp = cnt; cnt = cnt2; cnt2 = tmp; }
        if (changed_per_iter) changed_per_iter[it] = changed;
        if ((double)changed <= (double)delta * (double)N * (double)K) { ++it; break; }
    }
    if (iters_done) *iters_done = it;
    for (int64_t v = 0; v < N; ++v)
        for (int t = 0; t < K; ++t) {
            knn_id[v * K + t] = t < cnt[v] ? B[v * K + t].id : -1;
            knn_s[v * K + t] = t < cnt[v] ? B[v * K + t].s : INFINITY;
        }
    free(B); free(B2); free(cnt); free(cnt2); free(Rnew); free(Rold);
    return 0;
}

double orc_recall(const int32_t* found, const int32_t* truth, int64_t nq, int k)
{
    int64_t hit = 0;
    for (int64_t i = 0; i < nq; ++i)
        for (int a = 0; a < k; ++a) {
            int32_t f = found[i * k + a];
            if (f < 0) continue;
            for (int b = 0; b < k; ++b)
                if (truth[i * k + b] == f) { ++hit; break; }
        }
    return nq > 0 ? (double)hit / ((double)nq * (double)k) : 0.0;
}
