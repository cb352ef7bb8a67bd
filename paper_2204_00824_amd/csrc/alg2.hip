// Large-batch search with the paper's own data structures (Alg. 2, Sec. 4.2), one
// wavefront per query -- the counterpart of search.hip's rank-list form, kept so the
// two can be compared at equal recall:
//   R  top ranking array of fixed size k (k <= 64): one entry per lane, in registers,
//      sorted; an insertion is one ballot (rank) and one wave shift;
//   C  expansion queue cut into m_c segments of 32 sorted entries in LDS, segment =
//      id mod m_c; a push into a full segment drops its most distant entry; pop = the
//      smallest of the segment heads;
//   V  look-up table of expanded nodes, m_v segments of 32 slots in LDS written
//      round-robin, segment = id mod m_v;
//   stop when the popped candidate is further than the furthest of R by more than
//   delta on the measure itself (the L2 distance, or 1 - cos), when C is empty, or at
//   the hop limit T.
// Alg. 2 tests one neighbour at a time against V and C, after the pushes of the
// neighbours before it.  Here the look-ups of a hop are made by all lanes at once and the
// survivors' distances are computed together (same gather as search.hip); the pushes then
// run one by one in stored neighbour order, because each acceptance test reads the
// furthest entry of R as left by the previous push.  The two orders differ only when a
// push into a full segment of C drops a LATER neighbour of the same hop: in the listing's
// order that neighbour is then in neither container at its turn and is scored once more,
// but never pushed again (R holds it, or dropped it as its furthest and has only come
// closer since).  So R, C and V are the same either way; the kernel watches for that
// eviction and moves one count from the skips to the evaluations, which keeps both
// counters equal to the listing's.
#include "dist.hpp"
#include "ranklist.hpp"

namespace tsdg {

struct Alg2Args {
    const uint32_t* packed;
    const void* base;
    const float* queries;
    int32_t* out_ids;
    float* out_dists;
    ann_query_stats* stats;
    uint64_t N;
    uint64_t seed;
    int64_t qi_offset;
    float delta;
    int K, d, k, m_c, m_v, T, lambda_visit, metric;
};

// Stop test of Alg. 2 on the measure m itself.  1 - cos on unit rows: m = s/2, so
// s_u > s_f + 2*delta.  L2: sqrt(s_u) > sqrt(s_f) + delta, taken without a square root as
// t = (s_u - s_f) - delta^2 > 0 and t^2 > 4 delta^2 s_f in fp64 (every operation correctly rounded).
__device__ __forceinline__ bool alg2_stop(float s_u, float s_f, float delta, int metric)
{
    if (metric == 1) return s_u > s_f + 2.0f * delta;
    const double dd = (double)delta * (double)delta;
    const double t = ((double)s_u - (double)s_f) - dd;
    return t > 0.0 && t * t > (4.0 * dd) * (double)s_f;
}

__device__ __forceinline__ uint32_t seed_node_alg2(uint64_t seed, uint64_t qi, uint32_t j, uint64_t N)
{
    uint64_t x = seed + 0x9E3779B97F4A7C15ull * ((qi << 32) + (uint64_t)j + 1ull);
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    x = x ^ (x >> 31);
    return (uint32_t)__umul64hi(x, N);
}

// value of lane-1 (lane 0 keeps its own): the wave-wide shift used by the sorted insertions
__device__ __forceinline__ uint64_t from_lane_below(uint64_t v)
{
    const int lo = __builtin_amdgcn_update_dpp((int)(uint32_t)v, (int)(uint32_t)v, 0x138, 0xF, 0xF, false);          // wave_shr:1
    const int hi = __builtin_amdgcn_update_dpp((int)(uint32_t)(v >> 32), (int)(uint32_t)(v >> 32), 0x138, 0xF, 0xF, false);
    return ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo;
}

// smallest key of the wave (all lanes get it)
__device__ __forceinline__ uint64_t wave_min64(uint64_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint64_t other = ((uint64_t)(uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), o, 64) << 32) |
                               (uint32_t)__shfl_xor((int)(uint32_t)v, o, 64);
        v = other < v ? other : v;
    }
    return v;
}

template <typename T, int G, int C>
__global__ __launch_bounds__(64) void alg2_kernel(Alg2Args a)
{
    using RD = RowDist<T, G, C>;
    using chunk_t = typename RD::chunk_t;
    constexpr int VP = RD::VP;
    constexpr int U = (C >= 8) ? 1 : (C >= 3 ? 2 : 4);
    extern __shared__ uint64_t smem[];
    // byte rows: the fp32 query first (RowDist::distance_lds reads it 16 bytes at a time)
    float* qs = reinterpret_cast<float*>(smem);                     // [d] for byte rows, else nothing
    uint64_t* Cseg = smem + (sizeof(T) == 1 ? a.d / 2 : 0);         // [m_c * 32]
    uint64_t* ckey = Cseg + a.m_c * 32;                             // [64]
    uint32_t* cid = reinterpret_cast<uint32_t*>(ckey + 64);         // [64]
    uint32_t* V = cid + 64;                                         // [m_v * 32]
    int* Cn = reinterpret_cast<int*>(V + a.m_v * 32);               // [m_c]
    int* vpos = Cn + a.m_c;                                         // [m_v]

    const int lane = lane_id();
    const int qi = (int)blockIdx.x;
    const T* __restrict__ base = static_cast<const T*>(a.base);

    for (int i = lane; i < a.m_v * 32; i += 64) V[i] = 0xFFFFFFFFu;
    for (int i = lane; i < a.m_c; i += 64) Cn[i] = 0;
    for (int i = lane; i < a.m_v; i += 64) vpos[i] = 0;
    RD rd;
    rd.init(a.d, lane);
    rd.load_query_f32(a.queries + (size_t)qi * (size_t)a.d);
    if constexpr (sizeof(T) == 1)
        if (rd.v == 0) rd.store_query(qs);
    if (lane < 32) cid[lane] = seed_node_alg2(a.seed, (uint64_t)(a.qi_offset + qi), (uint32_t)lane, a.N);
    __syncthreads();

    auto score = [&](int m) {
        for (int b0 = 0; b0 < m; b0 += U * VP) {
            chunk_t buf[U][C];
            uint32_t e[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = b0 + u * VP + rd.v;
                ok[u] = c < m;
                e[u] = ok[u] ? cid[c] : 0u;
#pragma unroll
                for (int cc = 0; cc < C; ++cc) {
                    buf[u][cc] = chunk_t{};
                    if (ok[u] && rd.has(cc)) buf[u][cc] = rd.load(base, e[u], cc);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float tot = rd.distance_lds(buf[u], qs);
                if (ok[u] && rd.g == 0) ckey[b0 + u * VP + rd.v] = make_key(tot, e[u]);
            }
        }
    };

    // R = {u}, C = {u}: the closest of the 32 seeds
    score(32);
    __syncthreads();
    uint64_t rkey = kKeyEmpty;  // R[lane]
    int nR = 1;
    uint32_t hops = 0, evals = 32, skips = 0;
    {
        const uint64_t best = wave_min64(lane < 32 ? ckey[lane] : kKeyEmpty);
        if (lane == 0) {
            rkey = best;
            const int g = (int)(key_id(best) % (uint32_t)a.m_c);
            Cseg[g * 32] = best;
            Cn[g] = 1;
        }
    }
    __syncthreads();

    for (;;) {
        if (a.T > 0 && (int)hops >= a.T) break;
        // pop the nearest head
        uint64_t head = kKeyEmpty;
        if (lane < a.m_c && Cn[lane] > 0) head = Cseg[lane * 32];
        const uint64_t ukey = wave_min64(head);
        if (ukey == kKeyEmpty) break;
        ++hops;
        const uint32_t u = key_id(ukey);
        const int gu = (int)(u % (uint32_t)a.m_c);
        const int nu = Cn[gu];
        uint64_t nxt = kKeyEmpty;
        if (lane + 1 < nu) nxt = Cseg[gu * 32 + lane + 1];
        __syncthreads();
        if (lane < nu - 1) Cseg[gu * 32 + lane] = nxt;
        if (lane == 0) Cn[gu] = nu - 1;
        const float fs = key_dist(readlane64(rkey, nR - 1));
        if (alg2_stop(key_dist(ukey), fs, a.delta, a.metric)) break;
        if (lane == 0) {
            const int gv = (int)(u % (uint32_t)a.m_v);
            const int p = vpos[gv];
            V[gv * 32 + p] = u;
            vpos[gv] = (p + 1) & 31;
        }
        __syncthreads();

        // neighbours: lambda-prefix, then the V and C look-ups
        uint32_t w = kPackPad;
        if (lane < a.K) w = a.packed[(size_t)u * (size_t)a.K + lane];
        const bool okw = w != kPackPad && (int)(w >> kIdBits) < a.lambda_visit;
        const uint64_t bad = ~ballot64(okw);
        const int deg = bad ? ctz64(bad) : 64;
        const uint32_t e = w & kIdMask;
        bool fresh = lane < deg;
        bool only_in_c = false;  // skipped because C holds it (and V does not)
        if (fresh) {
            const int gv = (int)(e % (uint32_t)a.m_v);
            const int gc = (int)(e % (uint32_t)a.m_c);
            bool in_v = false, in_c = false;
            for (int t = 0; t < 32; ++t) in_v = in_v || V[gv * 32 + t] == e;
            const int nc = Cn[gc];
            for (int t = 0; t < nc; ++t) in_c = in_c || key_id(Cseg[gc * 32 + t]) == e;
            fresh = !in_v && !in_c;
            only_in_c = !in_v && in_c;
        }
        const uint64_t fm = ballot64(fresh);
        skips += (uint32_t)(deg - popc64(fm));
        const int m = popc64(fm);
        if (fresh) cid[popc64(fm & lanes_below(lane))] = e;
        __syncthreads();
        if (m == 0) continue;
        evals += (uint32_t)m;
        score(m);
        __syncthreads();

        // pushes, one by one in stored order
        uint64_t rest = fm;
        for (int j = 0; j < m; ++j) {
            const uint64_t c = ckey[j];
            const int p = ctz64(rest);  // position of this neighbour in the row
            rest &= rest - 1;
            const float fcur = key_dist(readlane64(rkey, nR - 1));
            const bool accept = nR < a.k || key_dist(c) < fcur;
            if (!accept) continue;
            if (ballot64(rkey == c)) continue;  // already in R
            // R.push: rank by ballot, shift the tail up by one lane, drop what falls beyond k
            {
                const int pos = popc64(ballot64(rkey < c));
                const uint64_t below = from_lane_below(rkey);
                uint64_t nk = lane < pos ? rkey : (lane == pos ? c : below);
                if (lane >= a.k) nk = kKeyEmpty;
                rkey = nk;
                if (nR < a.k) ++nR;
            }
            // C.push into segment id mod m_c
            {
                const int g = (int)(key_id(c) % (uint32_t)a.m_c);
                const int n = Cn[g];
                const uint64_t sk = (lane < n && lane < 32) ? Cseg[g * 32 + lane] : kKeyEmpty;
                const int pos = popc64(ballot64(sk < c));
                const uint64_t below = from_lane_below(sk);
                const uint64_t nk = lane < pos ? sk : (lane == pos ? c : below);
                if (n == 32 && pos < 32) {
                    // the segment's most distant entry falls out; a later neighbour of this hop that was
                    // skipped because C held it is scored again at its turn in the listing's order
                    const uint32_t gone = key_id(readlane64(sk, 31));
                    const bool again = only_in_c && lane > p && e == gone;
                    if (ballot64(again)) {
                        ++evals;
                        --skips;
                    }
                    if (again) only_in_c = false;
                }
                __syncthreads();
                if (lane < 32 && lane <= n) Cseg[g * 32 + lane] = nk;
                if (lane == 0) Cn[g] = n < 32 ? n + 1 : 32;
                __syncthreads();
            }
        }
    }

    for (int t = lane; t < a.k; t += 64) {
        const bool have = rkey != kKeyEmpty;
        a.out_ids[(size_t)qi * a.k + t] = have ? (int32_t)key_id(rkey) : -1;
        a.out_dists[(size_t)qi * a.k + t] = have ? key_dist(rkey) : __builtin_inff();
    }
    if (a.stats && lane == 0) {
        ann_query_stats st;
        st.hops = hops;
        st.dist_evals = evals;
        st.dedup_hits = skips;
        a.stats[qi] = st;
    }
}

namespace {
struct Alg2Dispatch {
    Alg2Args a;
    int nq;
    hipStream_t stream;
    template <typename T, int G, int C> void operator()()
    {
        const size_t lds = (size_t)a.m_c * 32 * 8 + 64 * 8 + 64 * 4 + (size_t)a.m_v * 32 * 4 + (size_t)(a.m_c + a.m_v) * 4 +
                           (sizeof(T) == 1 ? (size_t)a.d * 4 : 0);
        TSDG_LAUNCH((alg2_kernel<T, G, C>), dim3((unsigned)nq), dim3(64), lds, stream, a);
    }
};
}  // namespace

ann_status launch_search_alg2(const Alg2Launch& s)
{
    if (s.nq == 0) return ANN_OK;
    Alg2Dispatch disp;
    disp.a.packed = s.packed;
    disp.a.base = s.base;
    disp.a.queries = s.queries;
    disp.a.out_ids = s.out_ids;
    disp.a.out_dists = s.out_dists;
    disp.a.stats = s.stats;
    disp.a.N = (uint64_t)s.N;
    disp.a.seed = s.seed;
    disp.a.qi_offset = s.qi_offset;
    disp.a.delta = s.delta;
    disp.a.K = s.K;
    disp.a.d = s.d;
    disp.a.k = s.k;
    disp.a.m_c = s.m_c;
    disp.a.m_v = s.m_v;
    disp.a.T = s.max_hops;
    disp.a.lambda_visit = s.lambda_visit;
    disp.a.metric = s.metric;
    disp.nq = s.nq;
    disp.stream = s.stream;
    if (!dispatch_search_row_shape(s.dtype, s.d, disp)) {
        set_error("unsupported row shape: d=%d dtype=%d", s.d, (int)s.dtype);
        return ANN_EUNSUPPORTED;
    }
    TSDG_HIP(launch_error());
    return ANN_OK;
}

}  // namespace tsdg
