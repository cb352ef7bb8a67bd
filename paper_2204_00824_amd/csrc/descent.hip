// Approximate k-NN graph by neighbourhood propagation (the "approximate k-NN graph" that
// Sec. 3 of the paper starts from; the paper names no builder).  The published NN-descent idea
// -- a neighbour of a neighbour is likely a neighbour, only edges that are new need another
// look, reverse edges count too -- in a form in which every node PULLS its candidates from the
// lists of the previous iteration, so that the outcome does not depend on execution order:
//
//   list B[v]: K keys (s, id, flag) in (s,id) order; flag bit 0 set = "old" (already sampled).
//   newF[v] / oldF[v]: the first S new / first S old entries of B[v].
//   Rnew[w][slot(u)] keeps the smallest key (s(u,w), u) over all u with w in newF[u]
//   (slot(u) = (u * 2654435761) >> (32 - log2 S)); Rold likewise from oldF.  An atomic minimum
//   builds them, so they do not depend on the order of the offers either.
//   Node a (one wavefront): its list with newF[a] flagged old; sources newF[a], oldF[a],
//   Rnew[a], Rold[a]; from source v the candidates newF[v] and Rnew[v], plus oldF[v] and
//   Rold[v] when the edge a-v is new.  Candidates are de-duplicated in an LDS hash, scored with
//   the canonical distance and merged into the list (K smallest by (s,id), an id already
//   present stays as it is).  The new list goes to the other buffer.
//
// One source = one step of the same machinery the search uses for a hop: hash test-and-set,
// compaction, row gather + distance, rank merge.
#include <algorithm>
#include <cstring>

#include "dist.hpp"
#include "ranklist.hpp"

namespace tsdg {

constexpr uint64_t kRevEmpty = ~0ull;
constexpr int kDescentSlots = 2048;  // visited hash per node
constexpr int kChangedBins = 1024;

__device__ __forceinline__ uint32_t descent_seed_node(uint64_t seed, uint64_t v, uint32_t j, uint64_t N)
{
    uint64_t x = seed + 0x9E3779B97F4A7C15ull * ((v << 32) + (uint64_t)j + 1ull);
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    x = x ^ (x >> 31);
    return (uint32_t)__umul64hi(x, N);
}

struct DescentArgs {
    const void* base;
    const uint64_t* cur;   // [N,K] lists of the previous iteration
    uint64_t* next;        // [N,K]
    uint64_t* rnew;        // [N,S]
    uint64_t* rold;        // [N,S]
    const int32_t* init_ids;  // optional [N,K] start lists
    unsigned long long* changed;  // [2 * kChangedBins]: list entries changed, then rows scored
    uint64_t N;
    uint64_t seed;
    int d, K, S, log2s;
};

__global__ __launch_bounds__(256) void fill_u64_kernel(uint64_t* p, int64_t n, uint64_t v)
{
    const int64_t i = linear_block() * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// Scores the ids in `id` (one per lane, `valid` lanes only), skipping those the hash has seen,
// and merges them into list[0..K).  cid/ckey: 64 entries each.
template <typename RD, typename T>
__device__ __forceinline__ int score_and_merge(RD& rd, const T* __restrict__ base, uint32_t id, bool valid,
                                                uint64_t* list, int K, uint64_t* ckey, uint32_t* cid,
                                                uint32_t* table, int lane)
{
    using chunk_t = typename RD::chunk_t;
    constexpr int VP = RD::VP;
    constexpr int C = RD::NC;
    bool seen = false;
    if (valid) seen = visited_test_and_set(table, kDescentSlots, id);
    const uint64_t nm = ballot64(valid && !seen);
    const int m = popc64(nm);
    if (m == 0) return 0;
    if (valid && !seen) cid[popc64(nm & lanes_below(lane))] = id;
    __syncthreads();
    for (int b0 = 0; b0 < m; b0 += VP) {
        const int c = b0 + rd.v;
        const bool ok = c < m;
        const uint32_t e = cid[ok ? c : m - 1];
        chunk_t buf[C];
#pragma unroll
        for (int cc = 0; cc < C; ++cc) {
            buf[cc] = chunk_t{};
            if (rd.has(cc)) buf[cc] = rd.load(base, e, cc);
        }
        const float tot = rd.distance(buf);
        if (ok && rd.g == 0) ckey[c] = make_key(tot, e);
    }
    __syncthreads();
    const uint64_t key = lane < m ? ckey[lane] : kKeyEmpty;
    // the hash may have forgotten an id, so one call can carry the same candidate twice
    list_merge<false>(list, K, key, lane, [] { __syncthreads(); });
    __syncthreads();
    return m;
}

// Start lists: 2K draws of the seed generator, self and repeats dropped, the first K kept, or
// the caller's ids; scored and sorted, all flagged new.
template <typename T, int G, int C>
__global__ __launch_bounds__(64) void descent_init_kernel(DescentArgs a)
{
    using RD = RowDist<T, G, C>;
    __shared__ uint64_t list[64];
    __shared__ uint64_t ckey[64];
    __shared__ uint32_t cid[64];
    __shared__ uint32_t table[kDescentSlots];
    const int lane = lane_id();
    const uint64_t v = (uint64_t)linear_block();
    if (v >= a.N) return;  // folded grid: past the last node
    const T* __restrict__ base = static_cast<const T*>(a.base);
    list[lane] = kKeyEmpty;
    for (int i = lane; i < kDescentSlots; i += 64) table[i] = kHashEmpty;
    RD rd;
    rd.init(a.d, lane);
    rd.load_query_row(base, (uint32_t)v);
    __syncthreads();

    uint32_t id = 0;
    bool keep = false;
    if (a.init_ids) {
        const int32_t c = lane < a.K ? a.init_ids[v * a.K + lane] : -1;
        id = (uint32_t)c;
        keep = c >= 0 && (uint64_t)c != v && (uint64_t)c < a.N;
        // repeats inside the caller's list
        for (uint64_t mm = ballot64(keep); mm; mm &= mm - 1) {
            const int o = ctz64(mm);
            const uint32_t ido = readlane32(id, o);
            if (o < lane && ido == id) keep = false;
        }
    } else {
        // draws j = lane and j = 64 + lane (2K <= 128); a draw counts if it is not v and no earlier draw had it
        const uint32_t c0 = descent_seed_node(a.seed, v, (uint32_t)lane, a.N);
        const uint32_t c1 = descent_seed_node(a.seed, v, (uint32_t)(64 + lane), a.N);
        bool ok0 = lane < 2 * a.K && (uint64_t)c0 != v;
        bool ok1 = 64 + lane < 2 * a.K && (uint64_t)c1 != v;
        for (int o = 0; o < 64; ++o) {
            const uint32_t e0 = readlane32(c0, o);
            if (o < 2 * a.K) {
                if (o < lane && e0 == c0) ok0 = false;
                if (e0 == c1) ok1 = false;
            }
            const uint32_t e1 = readlane32(c1, o);
            if (64 + o < 2 * a.K && o < lane && e1 == c1) ok1 = false;
        }
        const uint64_t m0 = ballot64(ok0), m1 = ballot64(ok1);
        const int r0 = popc64(m0 & lanes_below(lane));
        const int r1 = popc64(m0) + popc64(m1 & lanes_below(lane));
        ok0 = ok0 && r0 < a.K;
        ok1 = ok1 && r1 < a.K;
        // at most K survive over both halves; score the first half now, the second below
        score_and_merge(rd, base, c0, ok0, list, a.K, ckey, cid, table, lane);
        id = c1;
        keep = ok1;
    }
    score_and_merge(rd, base, id, keep, list, a.K, ckey, cid, table, lane);
    if (lane < a.K) a.next[v * a.K + lane] = list[lane];
}

// Reverse samples: every node offers itself to the nodes in its forward samples.
__global__ __launch_bounds__(256) void descent_reverse_kernel(DescentArgs a)
{
    const uint64_t u = (uint64_t)linear_block() * 4 + (threadIdx.x >> 6);
    if (u >= a.N) return;
    const int lane = lane_id();
    const uint64_t key = lane < a.K ? a.cur[u * a.K + lane] : kKeyEmpty;
    const bool have = key != kKeyEmpty;
    const bool is_new = have && (key & 1ull) == 0ull;
    const bool is_old = have && (key & 1ull) != 0ull;
    const uint64_t mn = ballot64(is_new), mo = ballot64(is_old);
    const bool in_new = is_new && popc64(mn & lanes_below(lane)) < a.S;
    const bool in_old = is_old && popc64(mo & lanes_below(lane)) < a.S;
    if (in_new || in_old) {
        const uint32_t slot = ((uint32_t)u * 2654435761u) >> (32 - a.log2s);
        const uint64_t offer = ((key >> 32) << 32) | (uint64_t)(uint32_t)u;
        uint64_t* tab = in_new ? a.rnew : a.rold;
        atomicMin(reinterpret_cast<unsigned long long*>(&tab[(uint64_t)key_id(key) * a.S + slot]),
                  (unsigned long long)offer);
    }
}

template <typename T, int G, int C>
__global__ __launch_bounds__(64) void descent_join_kernel(DescentArgs a)
{
    using RD = RowDist<T, G, C>;
    __shared__ uint64_t list[64];
    __shared__ uint64_t ckey[64];
    __shared__ uint32_t cid[64];
    __shared__ uint32_t src[64];       // source id << 1 | edge-is-new
    __shared__ uint32_t table[kDescentSlots];
    const int lane = lane_id();
    const uint64_t v0 = (uint64_t)linear_block();
    if (v0 >= a.N) return;  // folded grid: past the last node
    const T* __restrict__ base = static_cast<const T*>(a.base);
    const int K = a.K, S = a.S;
    for (int i = lane; i < kDescentSlots; i += 64) table[i] = kHashEmpty;
    RD rd;
    rd.init(a.d, lane);
    rd.load_query_row(base, (uint32_t)v0);

    // own list: forward samples, and the list with the sampled new entries flagged old
    const uint64_t own = lane < K ? a.cur[v0 * K + lane] : kKeyEmpty;
    const bool have = own != kKeyEmpty;
    const bool is_new = have && (own & 1ull) == 0ull;
    const bool is_old = have && (own & 1ull) != 0ull;
    const uint64_t mn = ballot64(is_new), mo = ballot64(is_old);
    const bool in_new = is_new && popc64(mn & lanes_below(lane)) < S;
    const bool in_old = is_old && popc64(mo & lanes_below(lane)) < S;
    list[lane] = in_new ? (own | 1ull) : own;
    const uint64_t r = lane < S ? a.rnew[v0 * S + lane] : (lane < 2 * S ? a.rold[v0 * S + (lane - S)] : kRevEmpty);
    const bool rhave = r != kRevEmpty;
    // sources in the order newF, oldF, Rnew, Rold
    const uint64_t m_nf = ballot64(in_new), m_of = ballot64(in_old);
    const uint64_t m_rn = ballot64(rhave && lane < S), m_ro = ballot64(rhave && lane >= S);
    const int n_nf = popc64(m_nf), n_of = popc64(m_of), n_rn = popc64(m_rn), n_ro = popc64(m_ro);
    if (in_new) src[popc64(m_nf & lanes_below(lane))] = (key_id(own) << 1) | 1u;
    if (in_old) src[n_nf + popc64(m_of & lanes_below(lane))] = key_id(own) << 1;
    if (rhave && lane < S) src[n_nf + n_of + popc64(m_rn & lanes_below(lane))] = ((uint32_t)r << 1) | 1u;
    if (rhave && lane >= S) src[n_nf + n_of + n_rn + popc64(m_ro & lanes_below(lane))] = (uint32_t)r << 1;
    const int nsrc = n_nf + n_of + n_rn + n_ro;
    __syncthreads();
    // the node itself and what its list already holds need no scoring
    if (lane == 0) visited_test_and_set(table, kDescentSlots, (uint32_t)v0);
    if (have) visited_test_and_set(table, kDescentSlots, key_id(own));
    __syncthreads();

    const bool one_pass = K + 2 * S <= 64;
    int scored = 0;
    for (int q = 0; q < nsrc; ++q) {
        const uint32_t sv = src[q];
        const uint64_t v = sv >> 1;
        const bool edge_new = (sv & 1u) != 0u;
        // forward part of the source's samples (lanes 0..K-1)
        const uint64_t e = lane < K ? a.cur[v * K + lane] : kKeyEmpty;
        const bool eh = e != kKeyEmpty;
        const bool en = eh && (e & 1ull) == 0ull;
        const bool eo = eh && (e & 1ull) != 0ull;
        const uint64_t bn = ballot64(en), bo = ballot64(eo);
        bool valid = (en && popc64(bn & lanes_below(lane)) < S) ||
                     (edge_new && eo && popc64(bo & lanes_below(lane)) < S);
        uint32_t id = key_id(e);
        // reverse part: Rnew[v] always, Rold[v] when the edge is new
        const int rl = one_pass ? lane - K : lane;
        uint64_t rr = kRevEmpty;
        if (rl >= 0 && rl < S) rr = a.rnew[v * S + rl];
        else if (rl >= S && rl < 2 * S && edge_new) rr = a.rold[v * S + (rl - S)];
        if (one_pass) {
            if (rr != kRevEmpty) {
                valid = true;
                id = (uint32_t)rr;
            }
            valid = valid && (uint64_t)id != v0;
            scored += score_and_merge(rd, base, id, valid, list, K, ckey, cid, table, lane);
        } else {
            valid = valid && (uint64_t)id != v0;
            scored += score_and_merge(rd, base, id, valid, list, K, ckey, cid, table, lane);
            const uint32_t id2 = (uint32_t)rr;
            scored += score_and_merge(rd, base, id2, rr != kRevEmpty && (uint64_t)id2 != v0, list, K, ckey, cid, table, lane);
        }
    }

    const uint64_t fin = lane < K ? list[lane] : kKeyEmpty;
    if (lane < K) a.next[v0 * K + lane] = fin;
    // entries of the new list that the old one did not hold: the old entries that stayed are
    // exactly those not beyond the new list's last key
    const uint64_t fm = ballot64(fin != kKeyEmpty);
    const int nfin = popc64(fm);
    if (nfin > 0) {
        const uint64_t last = list[nfin - 1] | 1ull;
        const int stayed = popc64(ballot64(have && (own | 1ull) <= last));
        const int changed = nfin - stayed;
        if (lane == 0 && changed > 0) atomicAdd(&a.changed[v0 % kChangedBins], (unsigned long long)changed);
    }
    if (lane == 0 && scored > 0) atomicAdd(&a.changed[kChangedBins + v0 % kChangedBins], (unsigned long long)scored);
}

__global__ __launch_bounds__(256) void descent_export_kernel(const uint64_t* __restrict__ keys, int64_t n,
                                                             int32_t* __restrict__ ids, float* __restrict__ s)
{
    const int64_t i = linear_block() * 256 + threadIdx.x;
    if (i >= n) return;
    const uint64_t k = keys[i];
    ids[i] = k != kKeyEmpty ? (int32_t)key_id(k) : -1;
    s[i] = k != kKeyEmpty ? key_dist(k) : __builtin_inff();
}

namespace {
struct DescentLaunch {
    DescentArgs a;
    hipStream_t stream;
    bool init;
    template <typename T, int G, int C> void operator()()
    {
        if (init) TSDG_LAUNCH((descent_init_kernel<T, G, C>), folded_grid((int64_t)a.N), dim3(64), 0, stream, a);
        else TSDG_LAUNCH((descent_join_kernel<T, G, C>), folded_grid((int64_t)a.N), dim3(64), 0, stream, a);
    }
};
}  // namespace

ann_status knn_descent(const void* base, int64_t N, int d, ann_dtype dtype, int K, int S, int max_iters, float delta,
                       uint64_t seed, const int32_t* init_ids, hipStream_t stream, int32_t* out_ids, float* out_s,
                       int* iters_done, int64_t* last_changed, const BuildCtx& ctx)
{
    int log2s = 0;
    while ((1 << log2s) < S) ++log2s;
    uint64_t *b0 = nullptr, *b1 = nullptr, *rnew = nullptr, *rold = nullptr;
    unsigned long long* changed = nullptr;
    auto release = [&] {
        (void)hipFree(b0); (void)hipFree(b1); (void)hipFree(rnew); (void)hipFree(rold); (void)hipFree(changed);
    };
    const size_t nk = (size_t)N * K, ns = (size_t)N * S;
    hipError_t e = hipMalloc(&b0, nk * 8);
    if (e == hipSuccess) e = hipMalloc(&b1, nk * 8);
    if (e == hipSuccess) e = hipMalloc(&rnew, ns * 8);
    if (e == hipSuccess) e = hipMalloc(&rold, ns * 8);
    if (e == hipSuccess) e = hipMalloc(&changed, 2 * kChangedBins * sizeof(unsigned long long));
    if (e != hipSuccess) {
        release();
        set_error("hipMalloc of the neighbourhood-propagation buffers failed: %s", hipGetErrorString(e));
        return ANN_ENOMEM;
    }
    DescentLaunch L;
    L.stream = stream;
    L.a.base = base;
    L.a.cur = nullptr;
    L.a.next = b0;
    L.a.rnew = rnew;
    L.a.rold = rold;
    L.a.init_ids = init_ids;
    L.a.changed = changed;
    L.a.N = (uint64_t)N;
    L.a.seed = seed;
    L.a.d = d;
    L.a.K = K;
    L.a.S = S;
    L.a.log2s = log2s;
    L.init = true;
    ann_status rc = ANN_OK;
    auto fail = [&](ann_status s) { release(); return s; };
    if (!dispatch_row_shape(dtype, d, L)) { set_error("unsupported row shape d=%d", d); return fail(ANN_EUNSUPPORTED); }
    if (launch_error() != hipSuccess) { set_error("launch of the start lists failed"); return fail(ANN_EDEVICE); }
    uint64_t *cur = b0, *nxt = b1;
    int it = 0;
    int64_t ch = 0;
    L.init = false;
    for (; it < max_iters; ++it) {
        TSDG_LAUNCH(fill_u64_kernel, folded_grid((int64_t)((ns + 255) / 256)), dim3(256), 0, stream, rnew, (int64_t)ns, kRevEmpty);
        TSDG_LAUNCH(fill_u64_kernel, folded_grid((int64_t)((ns + 255) / 256)), dim3(256), 0, stream, rold, (int64_t)ns, kRevEmpty);
        TSDG_LAUNCH(fill_u64_kernel, dim3((2 * kChangedBins + 255) / 256), dim3(256), 0, stream,
                           reinterpret_cast<uint64_t*>(changed), (int64_t)(2 * kChangedBins), 0ull);
        L.a.cur = cur;
        L.a.next = nxt;
        TSDG_LAUNCH(descent_reverse_kernel, folded_grid((N + 3) / 4), dim3(256), 0, stream, L.a);
        dispatch_row_shape(dtype, d, L);
        unsigned long long h[2 * kChangedBins];
        hipError_t ce = hipMemcpyAsync(h, changed, sizeof(h), hipMemcpyDeviceToHost, stream);
        if (ce == hipSuccess) ce = hipStreamSynchronize(stream);
        if (ce == hipSuccess) ce = launch_error();
        if (ce != hipSuccess) { set_error("neighbourhood propagation failed on the device: %s", hipGetErrorString(ce)); return fail(ANN_EDEVICE); }
        ch = 0;
        int64_t scored = 0;
        for (int i = 0; i < kChangedBins; ++i) {
            ch += (int64_t)h[i];
            scored += (int64_t)h[kChangedBins + i];
        }
        std::swap(cur, nxt);
        (void)scored;
        ctx.report("descent", it + 1, max_iters);
        if ((double)ch <= (double)delta * (double)N * (double)K) { ++it; break; }
    }
    TSDG_LAUNCH(descent_export_kernel, folded_grid((int64_t)((nk + 255) / 256)), dim3(256), 0, stream, cur, (int64_t)nk,
                       out_ids, out_s);
    hipError_t fe = hipStreamSynchronize(stream);
    if (fe == hipSuccess) fe = launch_error();
    release();
    if (fe != hipSuccess) { set_error("neighbourhood propagation: %s", hipGetErrorString(fe)); return ANN_EDEVICE; }
    if (iters_done) *iters_done = it;
    if (last_changed) *last_changed = ch;
    return rc;
}

}  // namespace tsdg
