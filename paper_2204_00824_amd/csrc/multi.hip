// Small-batch multi-search (paper Sec. 4.1, Alg. 1): every query is served by t0
// workgroups, each running one cheap greedy search from its own 32 random start
// nodes; the t0 rankings of 32 are merged into the query's top-k by a second,
// tiny kernel.  This is what lets a batch of one occupy many CUs.
//
// One workgroup = 4 wavefronts = 32 groups of 8 lanes (for 128-dim fp32 rows), so
// the 32 neighbours of the current node are scored in a single pass with one
// memory round trip -- the role of the paper's "32 warps, one distance each".
// Per hop: wave 0 reads the adjacency row, all waves score, wave 0 applies the
// slot rule (the neighbour at position p competes only for slot p mod 32),
// keeps the 16 smallest, merges them with the kept half of R (first 16) and
// decides whether the search goes on (an id new to the first 16 entered them).
// No visited set and no expansion queue, as in the paper.
#include <mutex>

#include "dist.hpp"
#include "ranklist.hpp"

namespace tsdg {

struct MultiArgs {
    const uint32_t* packed;
    const void* base;
    const float* queries;
    uint64_t* scratch;  // [nq, t0, 33]: 32 keys of R, then hops << 32 | evaluations
    uint64_t N;
    uint64_t seed;
    int64_t qi_offset;
    int K, d, t0, T, lambda_visit;
};

__device__ __forceinline__ uint32_t seed_node_multi(uint64_t seed, uint64_t qi, uint32_t j, uint64_t N)
{
    uint64_t x = seed + 0x9E3779B97F4A7C15ull * ((qi << 32) + (uint64_t)j + 1ull);
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    x = x ^ (x >> 31);
    return (uint32_t)__umul64hi(x, N);
}

// #{ j in [FIRST, FIRST+COUNT) : key_j < mine }.  Lane indices are compile-time constants, so
// every broadcast is a v_readlane with an immediate lane (no scalar hazard waits); empty keys
// are the largest value and never count.
template <int FIRST, int COUNT>
__device__ __forceinline__ int count_smaller(uint64_t keys, uint64_t mine)
{
    int c = 0;
#pragma unroll
    for (int j = FIRST; j < FIRST + COUNT; ++j) c += readlane64(keys, j) < mine ? 1 : 0;
    return c;
}

template <typename T, int G, int C>
__global__ __launch_bounds__(256) void multi_kernel(MultiArgs a)
{
    using RD = RowDist<T, G, C>;
    using chunk_t = typename RD::chunk_t;
    constexpr int VP = RD::VP;
    constexpr int U = (C >= 8) ? 1 : (C >= 3 ? 2 : 4);
    __shared__ uint64_t ckey[64];
    __shared__ uint64_t R[32];
    __shared__ uint32_t cid[64];
    __shared__ uint32_t nrow[64];  // adjacency row of the next node, fetched while R is updated
    __shared__ int ctl[4];
    // byte rows: the fp32 query for the queries that are not integer-valued (RowDist::distance_lds)
    __shared__ __attribute__((aligned(16))) float qs[sizeof(T) == 1 ? 16 * G * C : 4];

    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const int j = (int)blockIdx.x;
    const int qi = (int)blockIdx.y;
    const T* __restrict__ base = static_cast<const T*>(a.base);

    RD rd;
    rd.init(a.d, lane);
    rd.load_query_f32(a.queries + (size_t)qi * (size_t)a.d);
    if constexpr (sizeof(T) == 1)
        if (wave == 0 && rd.v == 0) rd.store_query(qs);
    if (threadIdx.x < 32) {
        R[threadIdx.x] = kKeyEmpty;
        cid[threadIdx.x] = seed_node_multi(a.seed, (uint64_t)(a.qi_offset + qi), (uint32_t)(32 * j + (int)threadIdx.x), a.N);
    }
    __syncthreads();

    auto score = [&](int m) {  // cid[0..m) -> ckey[0..m); passes of VP rows are dealt to the four waves in turn
        for (int b0 = wave * VP; b0 < m; b0 += 4 * U * VP) {
            chunk_t buf[U][C];
            uint32_t e[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (u > 0 && b0 + u * 4 * VP >= m) break;   // wave-uniform: a pass with no candidate
                const int c = b0 + u * 4 * VP + rd.v;
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
                if (u > 0 && b0 + u * 4 * VP >= m) break;
                const float tot = rd.distance_lds(buf[u], qs);
                if (ok[u] && rd.g == 0) ckey[b0 + u * 4 * VP + rd.v] = make_key(tot, e[u]);
            }
        }
    };

    // start node: the closest of the 32 seeds
    score(32);
    __syncthreads();
    if (wave == 0) {
        const uint64_t key = lane < 32 ? ckey[lane] : kKeyEmpty;
        const uint64_t first = ballot64(lane < 32 && count_smaller<0, 32>(key, key) == 0);
        const int u0 = (int)key_id(readlane64(key, ctz64(first)));
        nrow[lane] = lane < a.K ? a.packed[(size_t)u0 * (size_t)a.K + lane] : kPackPad;
    }
    __syncthreads();
    uint32_t hops = 0, evals = 32;

    while ((int)hops < a.T) {
        if (wave == 0) {
            const uint32_t w = nrow[lane];
            const bool ok = w != kPackPad && (int)(w >> kIdBits) < a.lambda_visit;
            const uint64_t bad = ~ballot64(ok);
            const int deg = bad ? ctz64(bad) : 64;
            if (lane < deg) cid[lane] = w & kIdMask;
            if (lane == 0) ctl[1] = deg;
        }
        __syncthreads();
        const int deg = ctl[1];
        ++hops;
        if (deg == 0) break;
        evals += (uint32_t)deg;
        score(deg);
        __syncthreads();
        if (wave == 1) {
            // the next node is the closest of this hop's neighbours (the minimum over the slots is
            // the minimum over all of them): its row is fetched while wave 0 updates R
            const uint64_t key = lane < deg ? ckey[lane] : kKeyEmpty;
            uint32_t hi = (uint32_t)(key >> 32);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) hi = min(hi, (uint32_t)__shfl_xor((int)hi, o, 64));
            const uint64_t tie = ballot64((uint32_t)(key >> 32) == hi);
            uint32_t lo = (tie >> lane) & 1ull ? (uint32_t)key : 0xFFFFFFFFu;
            if (tie & (tie - 1)) {
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) lo = min(lo, (uint32_t)__shfl_xor((int)lo, o, 64));
            } else {
                lo = readlane32((uint32_t)key, ctz64(tie));
            }
            const uint32_t nu = lo >> 1;
            nrow[lane] = lane < a.K ? a.packed[(size_t)nu * (size_t)a.K + lane] : kPackPad;
        }
        if (wave == 0) {
            // slot rule: positions p and p+32 share slot p
            uint64_t key = kKeyEmpty;
            if (lane < 32) {
                const uint64_t k1 = lane < deg ? ckey[lane] : kKeyEmpty;
                const uint64_t k2 = lane + 32 < deg ? ckey[lane + 32] : kKeyEmpty;
                key = k1 < k2 ? k1 : k2;
            }
            const bool filled = lane < 32 && key != kKeyEmpty;
            const int rt = count_smaller<0, 32>(key, key);            // rank inside R_temp
            // lanes 32..47 carry the kept half of R
            uint64_t mine = key;
            const bool kept = lane >= 32 && lane < 48;
            if (kept) mine = R[lane - 32];
            const uint64_t km = ballot64(kept && mine != kKeyEmpty);
            bool cand = filled && rt < 16;
#pragma unroll
            for (int o = 32; o < 48; ++o)
                if (readlane64(mine, o) == key) cand = false;         // already among the kept 16
            const uint64_t vm = ballot64(cand) | km;
            if (!((vm >> lane) & 1ull)) mine = kKeyEmpty;             // only ranked keys take part
            const int fr = count_smaller<0, 48>(mine, mine);          // rank in the merged ranking
            const bool improved = ballot64(cand && fr < 16) != 0ull;
            const int n = popc64(vm);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if ((vm >> lane) & 1ull) R[fr] = mine;
            if (lane < 32 && lane >= n) R[lane] = kKeyEmpty;
            if (lane == 0) ctl[2] = improved ? 1 : 0;
        }
        __syncthreads();
        if (!ctl[2]) break;
    }

    uint64_t* out = a.scratch + ((size_t)qi * a.t0 + j) * 33;
    if (threadIdx.x < 32) out[threadIdx.x] = R[threadIdx.x];
    if (threadIdx.x == 32) out[32] = ((uint64_t)hops << 32) | (uint64_t)evals;
}

struct MultiMergeArgs {
    const uint64_t* scratch;
    int32_t* out_ids;
    float* out_dists;
    ann_query_stats* stats;
    int t0, k;
};

// Merge of the t0 rankings of one query, one workgroup of 256 threads.
// Only the first k entries of a ranking can reach the merged top-k (an entry further down
// has k distinct closer ids in its own ranking), and none above B = the smallest k-th entry
// of any ranking can (that ranking alone holds k distinct ids at or below B).  So: find B,
// put every key <= B into an LDS hash set (repeated ids collapse: same id, same distance,
// same key), list the distinct keys, and give each its rank by counting.  All of it is
// data-parallel; the step-by-step rank-list merge is kept only as the fallback for the case
// where the distinct survivors do not fit the table.
constexpr int kMergeSlots = 2048;
constexpr int kMergeDistinct = 768;

__device__ __forceinline__ void merge_sequential(const uint64_t* in, int t0, int k, uint64_t* list, uint64_t* stage,
                                                 int stage_cap, int lane)
{
    list[lane] = kKeyEmpty;
    auto sync = [] { wave_sync(); };
    const int total = t0 * k;
    for (int b0 = 0; b0 < total; b0 += stage_cap) {
        const int n = min(stage_cap, total - b0);
        wave_sync();
        for (int x = lane; x < n; x += 64) {
            const int gi = b0 + x;
            stage[x] = in[(size_t)(gi / k) * 33 + (gi % k)];
        }
        wave_sync();
        for (int s0 = 0; s0 < n; s0 += 64) {
            uint64_t key = s0 + lane < n ? stage[s0 + lane] : kKeyEmpty;
            const uint64_t worst = list[k - 1] | 1ull;
            if ((key | 1ull) >= worst) key = kKeyEmpty;
            const uint64_t vm = ballot64(key != kKeyEmpty);
            if (!vm) continue;
            bool dup = false;
            for (uint64_t m = vm; m; m &= m - 1) {
                const int o = ctz64(m);
                dup = dup || (o < lane && readlane64(key, o) == key);
            }
            if (dup) key = kKeyEmpty;
            list_merge(list, k, key, lane, sync);
            wave_sync();
        }
    }
}

__global__ __launch_bounds__(256) void multi_merge_kernel(MultiMergeArgs a)
{
    __shared__ unsigned long long table[kMergeSlots];
    __shared__ unsigned long long dist[kMergeDistinct];
    __shared__ unsigned long long bound;
    __shared__ unsigned ndist, sh_hops, sh_evals, overflow;
    const int tid = (int)threadIdx.x;
    const int qi = (int)blockIdx.x;
    const uint64_t* in = a.scratch + (size_t)qi * a.t0 * 33;
    for (int x = tid; x < kMergeSlots; x += 256) table[x] = kKeyEmpty;
    if (tid == 0) {
        bound = kKeyEmpty;
        ndist = 0u;
        sh_hops = 0u;
        sh_evals = 0u;
        overflow = 0u;
    }
    __syncthreads();
    {
        unsigned long long local = kKeyEmpty;
        unsigned h = 0, e = 0;
        for (int j = tid; j < a.t0; j += 256) {
            const uint64_t kth = in[(size_t)j * 33 + a.k - 1];
            local = kth < local ? kth : local;
            const uint64_t st = in[(size_t)j * 33 + 32];
            h += (unsigned)(st >> 32);
            e += (unsigned)st;
        }
        if (tid < a.t0) {
            atomicMin(&bound, local);
            atomicAdd(&sh_hops, h);
            atomicAdd(&sh_evals, e);
        }
    }
    __syncthreads();
    const unsigned long long B = bound;  // kKeyEmpty when no ranking is full: nothing is filtered
    const int total = a.t0 * a.k;
    for (int gi = tid; gi < total; gi += 256) {
        const unsigned long long key = in[(size_t)(gi / a.k) * 33 + (gi % a.k)];
        if (key == kKeyEmpty || key > B) continue;
        unsigned slot = (unsigned)((key * 0x9E3779B97F4A7C15ull) >> 53);  // top 11 bits
        int probe = 0;
        for (; probe < 128; ++probe) {
            const unsigned long long old = atomicCAS(&table[slot], (unsigned long long)kKeyEmpty, key);
            if (old == kKeyEmpty || old == key) break;
            slot = (slot + 1u) & (kMergeSlots - 1);
        }
        if (probe == 128) overflow = 1u;
    }
    __syncthreads();
    for (int x = tid; x < kMergeSlots; x += 256) {
        const unsigned long long key = table[x];
        if (key != kKeyEmpty) {
            const unsigned p = atomicAdd(&ndist, 1u);
            if (p < (unsigned)kMergeDistinct) dist[p] = key;
        }
    }
    __syncthreads();
    const int nd = (int)ndist;
    if (overflow || nd > kMergeDistinct) {   // does not happen on sane inputs; exact all the same
        if (tid < 64) merge_sequential(in, a.t0, a.k, reinterpret_cast<uint64_t*>(dist),
                                       reinterpret_cast<uint64_t*>(table), kMergeSlots, tid);
        __syncthreads();
        if (tid < a.k) {
            const uint64_t key = dist[tid];
            a.out_ids[(size_t)qi * a.k + tid] = key != kKeyEmpty ? (int32_t)key_id(key) : -1;
            a.out_dists[(size_t)qi * a.k + tid] = key != kKeyEmpty ? key_dist(key) : __builtin_inff();
        }
    } else {
        for (int i = tid; i < nd; i += 256) {
            const unsigned long long key = dist[i];
            int r = 0;
            for (int j = 0; j < nd; ++j) r += dist[j] < key ? 1 : 0;
            if (r < a.k) {
                a.out_ids[(size_t)qi * a.k + r] = (int32_t)key_id(key);
                a.out_dists[(size_t)qi * a.k + r] = key_dist(key);
            }
        }
        if (tid < a.k && tid >= nd) {
            a.out_ids[(size_t)qi * a.k + tid] = -1;
            a.out_dists[(size_t)qi * a.k + tid] = __builtin_inff();
        }
    }
    if (a.stats && tid == 0) {
        ann_query_stats s;
        s.hops = sh_hops;
        s.dist_evals = sh_evals;
        s.dedup_hits = 0;
        a.stats[qi] = s;
    }
}

// ---- scratch of ann_search_multi_static, the entry point that allocates nothing
// The rankings of up to kStaticSearches searches (nq * t0) live in this file-scope array: 540,672
// bytes that every GPU the library runs on holds until the process ends.  In host code the
// array's name is only a handle: the device address comes from hipGetSymbolAddress, asked once
// per device with that device current, and only that pointer is handed to kernels.  Nothing in
// the array has to start at zero: multi_kernel writes all 33 words of every search of a call
// before multi_merge_kernel reads them.
static __device__ __align__(256) unsigned long long scratch[(size_t)kMultiStaticSearches * 33];

ann_status multi_static_scratch(uint64_t** out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static uint64_t* ptr[kMaxDevices] = {};
    int dev = -1;
    TSDG_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) {
        set_error("ann_search_multi_static: device index %d outside 0..%d", dev, kMaxDevices - 1);
        return ANN_EUNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        TSDG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) {
            set_error("ann_search_multi_static: no device address for the static scratch");
            return ANN_EDEVICE;
        }
        ptr[dev] = static_cast<uint64_t*>(p);
    }
    *out = ptr[dev];
    return ANN_OK;
}

namespace {
struct MultiDispatch {
    MultiArgs a;
    int nq;
    hipStream_t stream;
    template <typename T, int G, int C> void operator()()
    {
        TSDG_LAUNCH((multi_kernel<T, G, C>), dim3((unsigned)a.t0, (unsigned)nq), dim3(256), 0, stream, a);
    }
};
}  // namespace

ann_status launch_search_multi(const MultiLaunch& s)
{
    if (s.nq == 0) return ANN_OK;
    MultiDispatch disp;
    disp.a.packed = s.packed;
    disp.a.base = s.base;
    disp.a.queries = s.queries;
    disp.a.scratch = s.scratch;
    disp.a.N = (uint64_t)s.N;
    disp.a.seed = s.seed;
    disp.a.qi_offset = s.qi_offset;
    disp.a.K = s.K;
    disp.a.d = s.d;
    disp.a.t0 = s.t0;
    disp.a.T = s.max_hops;
    disp.a.lambda_visit = s.lambda_visit;
    disp.nq = s.nq;
    disp.stream = s.stream;
    if (!dispatch_search_row_shape(s.dtype, s.d, disp)) {
        set_error("unsupported row shape: d=%d dtype=%d", s.d, (int)s.dtype);
        return ANN_EUNSUPPORTED;
    }
    TSDG_HIP(launch_error());
    MultiMergeArgs m;
    m.scratch = s.scratch;
    m.out_ids = s.out_ids;
    m.out_dists = s.out_dists;
    m.stats = s.stats;
    m.t0 = s.t0;
    m.k = s.k;
    TSDG_LAUNCH(multi_merge_kernel, dim3((unsigned)s.nq), dim3(256), 0, s.stream, m);
    TSDG_HIP(launch_error());
    return ANN_OK;
}

}  // namespace tsdg
