// Best-first k-NN search over the diversified graph (paper Sec. 4; steps S0-S7).
//
// One kernel template serves both batch regimes:
//   WAVES == 1  large batch: one 64-lane wavefront per query, one query per
//               workgroup, so the hardware dispatcher balances queries over CUs
//               (the shape of Alg. 2: all per-query state in on-chip memory,
//               one warp/wave per query);
//   WAVES  > 1  small batch: the same search, with the distance evaluations of a
//               hop (S5) split over the wavefronts of one workgroup, while
//               wavefront 0 keeps the rank-list and the visited set (Sec. 4.1
//               motivates spending more threads per query when few queries are
//               in flight; Alg. 1's independent multi-search is not this kernel).
//
// Per query, in LDS: the rank-list (L keys), the visited hash, and the hop's
// compacted candidate ids / keys.  Global reads per hop: one packed adjacency
// row, then the gathered base rows of the unvisited neighbours.
#include <type_traits>

#include "dist.hpp"
#include "ranklist.hpp"

namespace tsdg {

struct SearchArgs {
    const uint32_t* packed;
    const void* base;
    const float* queries;
    int32_t* out_ids;
    float* out_dists;
    ann_query_stats* stats;
    uint64_t N;
    uint64_t seed;
    int64_t qi_offset;
    int K, d, k, L, lambda_visit, n_seeds, max_hops, slots;
};

__device__ __forceinline__ uint32_t seed_node(uint64_t seed, uint64_t qi, uint32_t j, uint64_t N)
{
    // counter-based: splitmix64 output function of seed + GOLDEN*(qi*2^32 + j + 1), scaled to [0,N)
    uint64_t x = seed + 0x9E3779B97F4A7C15ull * ((qi << 32) + (uint64_t)j + 1ull);
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    x = x ^ (x >> 31);
    return (uint32_t)__umul64hi(x, N);
}

// The list and the visited set belong to wave 0 alone: its LDS accesses are processed in issue order,
// so ordering them takes no barrier.
struct ListSync {
    __device__ __forceinline__ void operator()() const { wave_sync(); }
};

// Byte rows of at most 128 elements need 63 registers once the fp32 query stays out of them: eight waves per
// SIMD.  The bound keeps later changes from losing that silently (the build would show spills).
template <typename T, int C, int WAVES>
constexpr int kSearchMinWaves = (sizeof(T) == 1 && C == 1 && WAVES == 1) ? 8 : 1;

// RL: registers per lane that hold the rank-list in wave 0 (1: L <= 64, 2: L <= 128); 0: the list is in LDS.
template <typename T, int G, int C, int WAVES, int RL>
__global__ __launch_bounds__(64 * WAVES, (kSearchMinWaves<T, C, WAVES>)) void search_kernel(SearchArgs a)
{
    using RD = RowDist<T, G, C>;
    using chunk_t = typename RD::chunk_t;
    constexpr int VP = RD::VP;
    constexpr int U = (C >= 8) ? 1 : (C >= 3 ? 2 : 4);  // passes in flight per wave

    extern __shared__ uint64_t smem[];
    const int L = a.L;
    const int Lp = RL ? 0 : (L + 63) & ~63;
    uint64_t* list = smem;                                   // [Lp]; nothing with the list in registers
    RegList<RL ? RL : 1> rl;                                 // RL: the list (wave 0)
    rl.init(RL ? L : 1);
    uint64_t* ckey = list + Lp;                              // [64]
    uint32_t* cid = reinterpret_cast<uint32_t*>(ckey + 64);  // [64]
    uint32_t* table = cid + 64;                              // [slots]
    int* ctl = reinterpret_cast<int*>(table + a.slots);      // [4]
    float* qs = reinterpret_cast<float*>(ctl + 4);           // [d], byte rows only

    const int lane = lane_id();
    const int wave = WAVES == 1 ? 0 : (int)(threadIdx.x >> 6);
    const int qi = (int)blockIdx.x;
    const T* __restrict__ base = static_cast<const T*>(a.base);

    for (int i = (int)threadIdx.x; i < Lp; i += 64 * WAVES) list[i] = kKeyEmpty;
    for (int i = (int)threadIdx.x; i < a.slots; i += 64 * WAVES) table[i] = kHashEmpty;

    RD rd;
    rd.init(a.d, lane);
    rd.load_query_f32(a.queries + (size_t)qi * (size_t)a.d);  // S0
    if constexpr (sizeof(T) == 1)
        if (wave == 0 && rd.v == 0) rd.store_query(qs);
    // With one wave per query nothing crosses waves: values that the waves of a workgroup hand each other
    // through LDS (the hop's node, its candidate count) stay in registers, and a barrier is a fence.
    auto block_sync = [&]() {
        if constexpr (WAVES == 1) wave_sync(); else __syncthreads();
    };
    block_sync();
    // Byte rows: an integer-valued query is scored on the integer route, and any other reads its fp32 elements
    // from LDS at every use, so that neither keeps them in registers (eight waves per SIMD instead of five).
    auto score = [&]<bool FULL>(const chunk_t (&b)[C], std::bool_constant<FULL>) -> float {
        if constexpr (sizeof(T) == 1)
            return rd.q_int ? rd.template distance_int<FULL>(b) : rd.template distance_from<FULL>(b, qs);
        else
            return rd.template distance<FULL>(b);
    };

    uint32_t hops = 0, evals = 0, dedup = 0;
    ListSync lsync;
    // byte rows only (the fp32 kernels would pay for the second loop with a wave of occupancy)
    const bool full_rows = sizeof(T) == 1 && rd.nchunks == G * C;  // wave-uniform

    // Scores the hop's candidates (ids in `id`, one per lane of wave 0) and merges them.  `stop` (wave 0): there
    // is no hop; the other waves learn it from the candidate count, which is the one thing they wait for, so a
    // hop costs them two barriers.  Returns true when the search is over.
    auto process = [&](uint32_t id, bool valid, bool stop) -> bool {
        int m = 0;
        if (wave == 0) {
            bool seen = false;
            if (valid) seen = visited_test_and_set(table, a.slots, id);  // S4
            const uint64_t nm = ballot64(valid && !seen);
            dedup += (uint32_t)popc64(ballot64(valid && seen));
            if (valid && !seen) cid[popc64(nm & lanes_below(lane))] = id;
            m = stop ? -1 : popc64(nm);
            if (WAVES > 1 && lane == 0) ctl[1] = m;
        }
        block_sync();
        if constexpr (WAVES > 1) m = ctl[1];
        if (m < 0) return true;
        if (m == 0) return false;
        evals += (uint32_t)m;
        // S5: gather + distance.  A pass is VP rows; the passes are dealt to the waves in turn and a wave has
        // U of its passes in flight, so that a short candidate list is spread over all the waves.
        if (full_rows) {
            // every lane owns all its C chunks: no per-chunk test, and a slot past the last
            // candidate re-reads the last one (its result is dropped) instead of being predicated
            for (int b0 = wave * VP; b0 < m; b0 += WAVES * U * VP) {
                chunk_t buf[U][C];
                uint32_t e[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (WAVES > 1 && u > 0 && b0 + u * WAVES * VP >= m) break;  // wave-uniform: a pass with no candidate
                    e[u] = cid[min(b0 + u * WAVES * VP + rd.v, m - 1)];
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) buf[u][cc] = rd.load(base, e[u], cc);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (WAVES > 1 && u > 0 && b0 + u * WAVES * VP >= m) break;
                    const float tot = score(buf[u], std::true_type{});
                    const int c = b0 + u * WAVES * VP + rd.v;
                    if (c < m && rd.g == 0) ckey[c] = make_key(tot, e[u]);
                }
            }
        } else {
            for (int b0 = wave * VP; b0 < m; b0 += WAVES * U * VP) {
                chunk_t buf[U][C];
                uint32_t e[U];
                bool ok[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (u > 0 && b0 + u * WAVES * VP >= m) break;   // wave-uniform: a pass with no candidate
                    const int c = b0 + u * WAVES * VP + rd.v;
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
                    if (u > 0 && b0 + u * WAVES * VP >= m) break;
                    const float tot = score(buf[u], std::false_type{});
                    if (ok[u] && rd.g == 0) ckey[b0 + u * WAVES * VP + rd.v] = make_key(tot, e[u]);
                }
            }
        }
        block_sync();
        if (wave == 0) {
            const uint64_t key = lane < m ? ckey[lane] : kKeyEmpty;
            if constexpr (RL) rl.merge(key, lane);  // S6
            else list_merge(list, L, key, lane, lsync);
        }
        return false;
    };

    // S1: seeds, 64 at a time; repeats inside a group of 64 are dropped here, repeats across
    // groups by the visited set.
    for (int j0 = 0; j0 < a.n_seeds; j0 += 64) {
        const int j = j0 + lane;
        bool valid = j < a.n_seeds;
        uint32_t id = valid ? seed_node(a.seed, (uint64_t)(a.qi_offset + qi), (uint32_t)j, a.N) : 0u;
        if (wave == 0) {
            const uint64_t vm = ballot64(valid);
            for (uint64_t mm = vm; mm; mm &= mm - 1) {
                const int o = ctz64(mm);
                const uint32_t ido = readlane32(id, o);
                if (o < lane && ido == id) valid = false;
            }
        }
        process(id, valid, false);
    }

    for (;;) {
        int u = -1;
        if (wave == 0) {
            uint64_t key = kKeyEmpty;
            int idx;
            if constexpr (RL) idx = rl.first_unexpanded(&key);  // S2
            else idx = list_first_unexpanded(list, L, lane, &key);
            if (a.max_hops > 0 && (int)hops >= a.max_hops) idx = -1;
            if (idx >= 0) {
                u = (int)key_id(key);
                if constexpr (RL) {
                    rl.mark_expanded(idx, lane);
                } else {
                    if (lane == 0) list[idx] = key | 1ull;
                    lsync();
                }
            }
        }
        if (WAVES == 1 && u < 0) break;
        uint32_t id = 0;
        bool valid = false;
        if (wave == 0 && u >= 0) {  // S3: adjacency row, prefix with lambda < lambda_visit
            ++hops;
            uint32_t w = kPackPad;
            if (lane < a.K) w = a.packed[(size_t)u * (size_t)a.K + lane];
            const bool ok = w != kPackPad && (int)(w >> kIdBits) < a.lambda_visit;
            const uint64_t bad = ~ballot64(ok);
            const int deg = bad ? ctz64(bad) : 64;
            valid = lane < deg;
            id = w & kIdMask;
        }
        if (process(id, valid, u < 0)) break;
    }

    // S7
    if (wave == 0) {
        for (int t = lane; t < a.k; t += 64) {
            const uint64_t key = RL ? rl.entry(t) : list[t];
            const bool have = key != kKeyEmpty;
            a.out_ids[(size_t)qi * a.k + t] = have ? (int32_t)key_id(key) : -1;
            a.out_dists[(size_t)qi * a.k + t] = have ? key_dist(key) : __builtin_inff();
        }
        if (a.stats && lane == 0) {
            ann_query_stats st;
            st.hops = hops;
            st.dist_evals = evals;
            st.dedup_hits = dedup;
            a.stats[qi] = st;
        }
    }
}

template <typename T, int G, int C, int WAVES, int RL> static ann_status launch_list_variant(const SearchLaunch& s)
{
    SearchArgs a;
    a.packed = s.packed;
    a.base = s.base;
    a.queries = s.queries;
    a.out_ids = s.out_ids;
    a.out_dists = s.out_dists;
    a.stats = s.stats;
    a.N = (uint64_t)s.N;
    a.seed = s.seed;
    a.qi_offset = s.qi_offset;
    a.K = s.K;
    a.d = s.d;
    a.k = s.k;
    a.L = s.L;
    a.lambda_visit = s.lambda_visit;
    a.n_seeds = s.n_seeds;
    a.max_hops = s.max_hops;
    a.slots = s.visited_slots;
    const int Lp = RL ? 0 : (s.L + 63) & ~63;
    const size_t lds = (size_t)Lp * 8 + 64 * 8 + 64 * 4 + (size_t)s.visited_slots * 4 + 16 +
                       (sizeof(T) == 1 ? (size_t)s.d * 4 : 0);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&search_kernel<T, G, C, WAVES, RL>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) {
            set_error("hipFuncSetAttribute(%zu bytes of LDS) failed: %s", lds, hipGetErrorString(e));
            return ANN_EDEVICE;
        }
    }
    TSDG_LAUNCH((search_kernel<T, G, C, WAVES, RL>), dim3((unsigned)s.nq), dim3(64 * WAVES), lds, s.stream, a);
    TSDG_HIP(launch_error());
    return ANN_OK;
}

template <typename T, int G, int C, int WAVES> static ann_status launch_variant(const SearchLaunch& s)
{
    // a list of at most 128 entries fits one or two per lane (k <= L, so the output comes from the same registers)
    if (s.L <= 64) return launch_list_variant<T, G, C, WAVES, 1>(s);
    if (s.L <= 128) return launch_list_variant<T, G, C, WAVES, 2>(s);
    return launch_list_variant<T, G, C, WAVES, 0>(s);
}

namespace {
struct SearchDispatch {
    const SearchLaunch& s;
    ann_status rc = ANN_EUNSUPPORTED;
    template <typename T, int G, int C> void operator()()
    {
        switch (s.waves) {
            case 1: rc = launch_variant<T, G, C, 1>(s); break;
            case 2: rc = launch_variant<T, G, C, 2>(s); break;
            case 4: rc = launch_variant<T, G, C, 4>(s); break;
            case 8: rc = launch_variant<T, G, C, 8>(s); break;
            default: set_error("waves_per_query must be 1, 2, 4 or 8"); rc = ANN_EINVAL; break;
        }
    }
};
}  // namespace

ann_status launch_search(const SearchLaunch& s)
{
    if (s.nq == 0) return ANN_OK;
    SearchDispatch disp{s};
    if (!dispatch_search_row_shape(s.dtype, s.d, disp)) {
        set_error("unsupported row shape: d=%d dtype=%d (d must be a multiple of %d and at most %d)", s.d,
                  (int)s.dtype, s.dtype == ANN_U8 ? 16 : 4, s.dtype == ANN_U8 ? 1024 : 2048);
        return ANN_EUNSUPPORTED;
    }
    return disp.rc;
}

}  // namespace tsdg
