// Two-stage diversification of the exact k-NN graph (paper Sec. 3.2-3.3;
// build steps B2, B3, B4).  Every node is independent (Sec. 3.3, last paragraph),
// so each kernel gives one wavefront to one node:
//   stage 1   pairwise canonical distances inside the K-list, then the sequential
//             relaxed-occlusion scan of Eq. 2 (closest edge first, each next edge
//             against the kept ones, Sec. 3.1);
//   reverse   in-degree count -> exclusive scan -> scatter of (source, distance),
//             then per node the kept and the reverse edges are merged by (s, id),
//             duplicates dropped, and the list is cut to rev_cap;
//   stage 2   pairwise distances inside that list, lambda_j = number of edges that
//             occlude edge j by Eq. 1, order by (lambda, s, id), cut at lambda0
//             and at K, written as the packed adjacency the search reads.
#include <algorithm>

#include "dist.hpp"
#include "i8rows.hpp"
#include "ranklist.hpp"

namespace tsdg {

constexpr float kInfD = __builtin_inff();

// P[i*stride + j] = s(x_ids[i], x_ids[j]) for i < j < m (canonical distance), one wavefront.
// Four rows i at a time sit in registers as "queries", so that every row j fetched from the
// caches serves four distances (a row would otherwise be fetched once per pair: m^2/2 fetches
// of d elements per node, which is what bounds these kernels).
template <typename RD, typename T>
__device__ __forceinline__ void pairwise(RD& rd, const T* __restrict__ base, const int32_t* ids, int m, float* P,
                                         int stride)
{
    using chunk_t = typename RD::chunk_t;
    constexpr int VP = RD::VP;
    constexpr int C = RD::NC;
    constexpr int QB = 4;
    RD q[QB];
#pragma unroll
    for (int b = 0; b < QB; ++b) q[b] = rd;  // lane geometry
    for (int i0 = 0; i0 + 1 < m; i0 += QB) {
#pragma unroll
        for (int b = 0; b < QB; ++b) q[b].load_query_row(base, (uint32_t)ids[min(i0 + b, m - 1)]);
        for (int p0 = i0 + 1; p0 < m; p0 += VP) {
            const int j = p0 + rd.v;
            const bool ok = j < m;
            const uint32_t e = (uint32_t)ids[ok ? j : m - 1];
            chunk_t buf[C];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) {
                buf[cc] = chunk_t{};
                if (rd.has(cc)) buf[cc] = rd.load(base, e, cc);
            }
#pragma unroll
            for (int b = 0; b < QB; ++b) {
                const float tot = q[b].distance(buf);
                if (ok && rd.g == 0 && i0 + b < j) P[(i0 + b) * stride + j] = tot;
            }
        }
    }
}

// Rows that are integers in [0,255] (uint8 storage, or fp32 that passes the test) take their pairwise distances
// from the integer matrix cores: with the centred int8 copies x' = x - 128, s(x_i, x_j) = |x_i'|^2 + |x_j'|^2 -
// 2 x_i'.x_j' is exact in int32, and its conversion to fp32 is the canonical value (an exact sum rounded once).
struct I8Rows {
    const uint8_t* xc8;   // [N, dp8] centred rows, or null: use the general routine
    const int* xn8;       // [N] |x'|^2
    int dp8;
};

// ------------------------------------------------------------------ stage 1
struct Stage1Args {
    const void* base;
    const int32_t* knn_id;  // [N,K] sorted by (s,id)
    const float* knn_s;
    int32_t* g1_id;         // [N,K] kept edges first, -1 after
    float* g1_s;
    int32_t* g1_deg;        // [N]
    unsigned* indeg;        // [N] in-degree of the kept graph (atomic)
    int64_t N;
    int d, K;
    float alpha2;
    I8Rows i8;
};

template <typename T, int G, int C>
__global__ __launch_bounds__(64) void stage1_kernel(Stage1Args a)
{
    using RD = RowDist<T, G, C>;
    extern __shared__ float sm[];
    const int K = a.K;
    float* P = sm;                                         // [K*K]
    float* s0 = P + K * K;                                 // [K]
    int32_t* ids = reinterpret_cast<int32_t*>(s0 + K);     // [K]
    const int64_t x0 = linear_block();
    if (x0 >= a.N) return;  // folded grid: past the last node
    const int lane = lane_id();
    const T* __restrict__ base = static_cast<const T*>(a.base);

    int32_t id = -1;
    float s = kInfD;
    if (lane < K) {
        id = a.knn_id[x0 * K + lane];
        s = a.knn_s[x0 * K + lane];
        ids[lane] = id;
        s0[lane] = s;
    }
    const uint64_t used = ballot64(id >= 0);
    const int m = used ? 64 - __builtin_clzll(used) : 0;   // lists are prefixes
    __syncthreads();
    {
        RD rd;
        rd.init(a.d, lane);
        pairwise(rd, base, ids, m, P, K);
    }
    __syncthreads();

    // sequential scan: lane i answers "does kept edge i occlude edge j"
    uint64_t kept = m > 0 ? 1ull : 0ull;
    for (int j = 1; j < m; ++j) {
        const float s0j = s0[j];
        bool occ = false;
        if (lane < j && ((kept >> lane) & 1ull)) {
            const float a1 = a.alpha2 * s;
            if (a1 < s0j) {
                const float a2 = a.alpha2 * P[lane * K + j];
                occ = a2 < s0j;
            }
        }
        if (!ballot64(occ)) kept |= 1ull << j;
    }
    const int deg = popc64(kept);
    const bool mine = (kept >> lane) & 1ull;
    const int pos = popc64(kept & lanes_below(lane));
    if (lane < K) {
        // compact kept edges to the front, pad the rest
        if (lane >= deg) {
            a.g1_id[x0 * K + lane] = -1;
            a.g1_s[x0 * K + lane] = kInfD;
        }
    }
    __syncthreads();
    if (mine) {
        a.g1_id[x0 * K + pos] = id;
        a.g1_s[x0 * K + pos] = s;
        atomicAdd(&a.indeg[id], 1u);
    }
    if (lane == 0) a.g1_deg[x0] = deg;
}

// ------------------------------------------------------------------ exclusive scan (uint32 -> uint64)
constexpr int kScanBlock = 1024;
__global__ __launch_bounds__(256) void scan_partial(const unsigned* __restrict__ in, int64_t n,
                                                    uint64_t* __restrict__ block_sums)
{
    __shared__ uint64_t red[256];
    const int64_t b0 = (int64_t)blockIdx.x * kScanBlock;
    uint64_t acc = 0;
    for (int i = threadIdx.x; i < kScanBlock; i += 256)
        if (b0 + i < n) acc += in[b0 + i];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) block_sums[blockIdx.x] = red[0];
}
__global__ void scan_block_sums(uint64_t* block_sums, int64_t nb)
{
    // one thread: nb = N/1024 is at most 131072
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        uint64_t run = 0;
        for (int64_t i = 0; i < nb; ++i) {
            const uint64_t v = block_sums[i];
            block_sums[i] = run;
            run += v;
        }
        block_sums[nb] = run;
    }
}
__global__ __launch_bounds__(256) void scan_final(const unsigned* __restrict__ in, int64_t n,
                                                  const uint64_t* __restrict__ block_sums, uint64_t* __restrict__ out)
{
    __shared__ uint64_t part[256];
    const int64_t b0 = (int64_t)blockIdx.x * kScanBlock;
    const int t = threadIdx.x;
    unsigned v[4];
    uint64_t loc = 0;
    for (int e = 0; e < 4; ++e) {
        const int64_t i = b0 + t * 4 + e;
        v[e] = i < n ? in[i] : 0u;
        loc += v[e];
    }
    part[t] = loc;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {  // inclusive Hillis-Steele over the 256 partials
        const uint64_t add = t >= o ? part[t - o] : 0;
        __syncthreads();
        part[t] += add;
        __syncthreads();
    }
    uint64_t run = block_sums[blockIdx.x] + part[t] - loc;
    for (int e = 0; e < 4; ++e) {
        const int64_t i = b0 + t * 4 + e;
        if (i < n) out[i] = run;
        run += v[e];
    }
    if (blockIdx.x == gridDim.x - 1 && t == 255) out[n] = block_sums[gridDim.x];
}

// ------------------------------------------------------------------ reverse edges
__global__ __launch_bounds__(256) void scatter_kernel(const int32_t* __restrict__ g1_id, const float* __restrict__ g1_s,
                                                      int64_t total, int K, const uint64_t* __restrict__ start,
                                                      unsigned* __restrict__ cursor, int32_t* __restrict__ rev_src,
                                                      float* __restrict__ rev_s)
{
    const int64_t i = linear_block() * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int32_t tgt = g1_id[i];
    if (tgt < 0) return;
    const uint64_t pos = start[tgt] + atomicAdd(&cursor[tgt], 1u);
    rev_src[pos] = (int32_t)(i / K);
    rev_s[pos] = g1_s[i];
}

struct MergeArgs {
    const int32_t* g1_id;
    const float* g1_s;
    const int32_t* g1_deg;
    const uint64_t* start;
    const int32_t* rev_src;
    const float* rev_s;
    int32_t* g2_id;  // [N, rev_cap]
    float* g2_s;
    int32_t* g2_deg;
    int64_t N;
    int K, rev_cap;
};

__global__ __launch_bounds__(64) void merge_kernel(MergeArgs a)
{
    extern __shared__ uint64_t list[];  // [rev_cap rounded to 64]
    const int64_t x0 = linear_block();
    if (x0 >= a.N) return;  // folded grid: past the last node
    const int lane = lane_id();
    const int Lp = (a.rev_cap + 63) & ~63;
    for (int i = lane; i < Lp; i += 64) list[i] = kKeyEmpty;
    __syncthreads();
    auto sync = [] { __syncthreads(); };
    const int deg = a.g1_deg[x0];
    uint64_t key = kKeyEmpty;
    if (lane < deg) key = make_key(a.g1_s[x0 * a.K + lane], (uint32_t)a.g1_id[x0 * a.K + lane]);
    list_merge(list, a.rev_cap, key, lane, sync);
    __syncthreads();
    const uint64_t b = a.start[x0], e = a.start[x0 + 1];
    for (uint64_t p0 = b; p0 < e; p0 += 64) {
        const uint64_t p = p0 + lane;
        key = p < e ? make_key(a.rev_s[p], (uint32_t)a.rev_src[p]) : kKeyEmpty;
        list_merge(list, a.rev_cap, key, lane, sync);
        __syncthreads();
    }
    int cnt = 0;
    for (int i = lane; i < a.rev_cap; i += 64) {
        const uint64_t k = list[i];
        const bool have = k != kKeyEmpty;
        a.g2_id[x0 * a.rev_cap + i] = have ? (int32_t)key_id(k) : -1;
        a.g2_s[x0 * a.rev_cap + i] = have ? key_dist(k) : kInfD;
        cnt += have ? 1 : 0;
    }
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
    if (lane == 0) a.g2_deg[x0] = cnt;
}

// ------------------------------------------------------------------ stage 2
constexpr int kLambdaSlots = 1024;

struct Stage2Args {
    const void* base;
    const int32_t* g2_id;
    const float* g2_s;
    const int32_t* g2_deg;
    uint32_t* packed;  // [N,K]
    int* max_lambda;   // [kLambdaSlots]: a node reports to slot (node % kLambdaSlots), so no address takes every atomic
    int64_t N;
    int d, K, rev_cap, lambda0;
    I8Rows i8;
};

template <typename T, int G, int C>
__global__ __launch_bounds__(64) void stage2_kernel(Stage2Args a)
{
    using RD = RowDist<T, G, C>;
    extern __shared__ float sm[];
    const int R = a.rev_cap;
    float* P = sm;                                         // [R*R], upper triangle used
    float* s0 = P + R * R;                                 // [R]
    int32_t* ids = reinterpret_cast<int32_t*>(s0 + R);     // [R]
    int* lam = reinterpret_cast<int*>(ids + R);            // [R]
    const int64_t x0 = linear_block();
    if (x0 >= a.N) return;  // folded grid: past the last node
    const int lane = lane_id();
    const T* __restrict__ base = static_cast<const T*>(a.base);
    const int m = a.g2_deg[x0];
    for (int i = lane; i < m; i += 64) {
        ids[i] = a.g2_id[x0 * R + i];
        s0[i] = a.g2_s[x0 * R + i];
    }
    for (int i = lane; i < a.K; i += 64) a.packed[x0 * a.K + i] = kPackPad;
    __syncthreads();
    {
        RD rd;
        rd.init(a.d, lane);
        pairwise(rd, base, ids, m, P, R);
    }
    __syncthreads();

    // lambda_j (Eq. 1, counted over the whole list, strict comparisons)
    for (int j = lane; j < m; j += 64) {
        const float sj = s0[j];
        int cnt = 0;
#pragma unroll 8   // eight LDS reads in flight: two waves per SIMD do not hide one read per iteration
        for (int i = 0; i < m; ++i) {
            if (i == j) continue;
            const float pij = i < j ? P[i * R + j] : P[j * R + i];
            cnt += (s0[i] < sj && pij < sj) ? 1 : 0;
        }
        lam[j] = cnt;
    }
    __syncthreads();
    // rank by (lambda, s, id); entries with lambda <= lambda0 form a prefix of that order
    int lmax = 0;
    for (int j = lane; j < m; j += 64) {
        const int lj = lam[j];
        const uint64_t kj = make_key(s0[j], (uint32_t)ids[j]);
        int r = 0;
#pragma unroll 8
        for (int i = 0; i < m; ++i) {
            const int li = lam[i];
            const uint64_t ki = make_key(s0[i], (uint32_t)ids[i]);
            r += (li < lj || (li == lj && ki < kj)) ? 1 : 0;
        }
        if (lj <= a.lambda0 && r < a.K) {
            a.packed[x0 * a.K + r] = (uint32_t)ids[j] | ((uint32_t)lj << kIdBits);
            lmax = max(lmax, lj);
        }
    }
    for (int o = 32; o > 0; o >>= 1) lmax = max(lmax, __shfl_xor(lmax, o, 64));
    if (lane == 0 && lmax > 0) atomicMax(&a.max_lambda[x0 % kLambdaSlots], lmax);
}

// ------------------------------------------------------------------ integer rows: both stages on the accumulators
// For rows that are integers in [0,255] the pairwise distances of a list are a Gram matrix on the integer matrix
// cores (pairwise_i8 above says why that is the canonical value).  These two kernels never write that matrix
// anywhere: each decision of Eq. 2 / Eq. 1 is taken on the accumulator that holds its distance, so a node needs no
// LDS beyond the staged rows (a third of the matrix form's footprint: more waves per CU to hide the two dependent
// round trips ids -> rows), and the lambda counts / the order by (lambda, s, id) become ballots instead of loops
// over LDS.  One wavefront per node, kI8Waves nodes per workgroup; the waves share nothing, so there is no
// barrier.  NB = 1: lists of at most 32 entries (one 32x32 block), NB = 2: up to 64 (three blocks of the upper
// triangle).
//
// What makes the upper triangle enough: both stages receive their list sorted by (s, id), so s0[i] <= s0[j] for
// i < j.  Edge i can occlude edge j only if s0[i] < s0[j] (Eq. 1; Eq. 2 asks alpha^2 s0[i] < s0[j] with alpha >= 1),
// which fails for every i >= j -- the tests below need no index comparison, and pairs below the diagonal never count.
constexpr int kI8Waves = 4;

struct I8Slice {          // one wavefront's part of the workgroup's LDS
    uint8_t* rows;        // [32 * NB][dp8 + 16] centred rows of the list, zero beyond its length
    float* s0;            // [32 * NB] distance of each entry to the node (+inf beyond the list)
    int* nrm;             // [32 * NB] |x'|^2
    int32_t* ids;         // [32 * NB]
    int XS;
};
template <int NB> __host__ __device__ constexpr size_t i8_slice_bytes(int dp8) { return (size_t)32 * NB * (dp8 + 16) + 3 * 32 * NB * 4; }
template <int NB> __device__ __forceinline__ I8Slice i8_slice(uint8_t* smem, int wave, int dp8)
{
    I8Slice z;
    z.XS = dp8 + 16;
    z.rows = smem + (size_t)wave * i8_slice_bytes<NB>(dp8);
    z.s0 = reinterpret_cast<float*>(z.rows + 32 * NB * z.XS);
    z.nrm = reinterpret_cast<int*>(z.s0 + 32 * NB);
    z.ids = z.nrm + 32 * NB;
    return z;
}

// Lane e brings entry e of the list (id < 0: none).  Fills the slice and leaves the Gram blocks (0,0), (0,1), (1,1)
// of the list's centred rows in acc: lane l, register r of block (bi,bj) holds x_i'.x_j' for
// i = 32 bi + 8 (r / 4) + 4 (l / 32) + r % 4 and j = 32 bj + l % 32.
template <int NB>
__device__ __forceinline__ void gram_of_list(const I8Rows& x, const I8Slice& z, int32_t id, float s, int m, int lane,
                                             intx16 (&acc)[2 * NB - 1])
{
    constexpr int ROWS = 32 * NB;
    if (lane < ROWS) {
        z.ids[lane] = id;
        z.s0[lane] = lane < m ? s : kInfD;
        z.nrm[lane] = lane < m ? x.xn8[id] : 0;
    }
    wave_sync();
    const int cpr = x.dp8 / 16;  // 16-byte chunks per row
    // eight of a lane's chunks are requested before the first is stored, so the list's rows arrive in one round trip
    for (int t0 = 0; t0 * 64 < ROWS * cpr; t0 += 8) {
        intx4 v[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int c = lane + 64 * (t0 + t);
            const int r = c / cpr, k = c % cpr;
            v[t] = intx4{0, 0, 0, 0};
            if (r < m) v[t] = *reinterpret_cast<const intx4*>(x.xc8 + (size_t)z.ids[r] * x.dp8 + k * 16);
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int c = lane + 64 * (t0 + t);
            const int r = c / cpr, k = c % cpr;
            if (r < ROWS) *reinterpret_cast<intx4*>(z.rows + r * z.XS + k * 16) = v[t];
        }
    }
    wave_sync();
#pragma unroll
    for (int blk = 0; blk < 2 * NB - 1; ++blk) {
        const int bi = blk >> 1, bj = (blk + 1) >> 1;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[blk][r] = 0;
        if (bj * 32 >= m) continue;   // wave-uniform
        for (int ks = 0; ks < x.dp8 / 32; ++ks) {
            const intx4 A = *reinterpret_cast<const intx4*>(z.rows + (bi * 32 + (lane & 31)) * z.XS + ks * 32 + 16 * (lane >> 5));
            const intx4 B = *reinterpret_cast<const intx4*>(z.rows + (bj * 32 + (lane & 31)) * z.XS + ks * 32 + 16 * (lane >> 5));
            acc[blk] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A, B, acc[blk], 0, 0, 0);
        }
    }
}

// Stage 1 (Sec. 3.2, Eq. 2 with the order rule of Sec. 3.1).  Column j's lane collects the set O_j of entries i that
// would occlude j if kept (alpha^2 s0[i] < s0[j] and alpha^2 s(x_i,x_j) < s0[j], the same fp32 products as the
// general kernel); the sequential part is then  kept_j = (O_j and kept) is empty  on 64-bit masks.
template <int NB>
__global__ __launch_bounds__(64 * kI8Waves) void stage1_i8_kernel(Stage1Args a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_i8[];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const int64_t x0 = linear_block() * kI8Waves + wave;
    if (x0 >= a.N) return;  // no barrier below: a wave past the last node just leaves
    const int K = a.K;
    const I8Slice z = i8_slice<NB>(smem_i8, wave, a.i8.dp8);

    int32_t id = -1;
    float s = kInfD;
    if (lane < K) {
        id = a.knn_id[x0 * K + lane];
        s = a.knn_s[x0 * K + lane];
    }
    const uint64_t used = ballot64(id >= 0);
    const int m = used ? 64 - __builtin_clzll(used) : 0;   // lists are prefixes
    intx16 acc[2 * NB - 1];
    gram_of_list<NB>(a.i8, z, id, s, m, lane, acc);

    uint32_t part[2 * NB - 1];
#pragma unroll
    for (int blk = 0; blk < 2 * NB - 1; ++blk) {
        const int bi = blk >> 1, bj = (blk + 1) >> 1;
        part[blk] = 0u;
        if (bj * 32 >= m) continue;
        const int j = bj * 32 + (lane & 31);
        const float sj = z.s0[j];
        const int nj = z.nrm[j];
        uint32_t bits = 0u;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i0 = bi * 32 + 8 * q + 4 * (lane >> 5);
            const float4 si = *reinterpret_cast<const float4*>(z.s0 + i0);
            const intx4 ni = *reinterpret_cast<const intx4*>(z.nrm + i0);
            const float sv[4] = {si.x, si.y, si.z, si.w};
            const int nv[4] = {ni.x, ni.y, ni.z, ni.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float pij = (float)(nv[t] + nj - 2 * acc[blk][4 * q + t]);
                const float a1 = a.alpha2 * sv[t];
                const float a2 = a.alpha2 * pij;
                bits |= (a1 < sj && a2 < sj) ? (1u << (8 * q + t)) : 0u;
            }
        }
        bits <<= 4 * (lane >> 5);
        part[blk] = bits | (uint32_t)__shfl_xor((int)bits, 32, 64);   // both halves of the rows of this column
    }
    // lane e now assembles O_e: entries 0..31 from block (0,0) (e < 32) or (0,1), entries 32..63 from block (1,1)
    uint64_t occ = part[0];
    if constexpr (NB == 2) occ = lane < 32 ? (uint64_t)part[0] : ((uint64_t)part[1] | ((uint64_t)part[2] << 32));
    uint64_t kept = m > 0 ? 1ull : 0ull;
    for (int j = 1; j < m; ++j) {
        const uint64_t oj = readlane64(occ, j);
        if ((oj & kept) == 0ull) kept |= 1ull << j;
    }
    const int deg = popc64(kept);
    const bool mine = (kept >> lane) & 1ull;
    const int pos = popc64(kept & lanes_below(lane));
    if (lane < K && lane >= deg) {
        a.g1_id[x0 * K + lane] = -1;
        a.g1_s[x0 * K + lane] = kInfD;
    }
    if (mine) {
        a.g1_id[x0 * K + pos] = id;
        a.g1_s[x0 * K + pos] = s;
        atomicAdd(&a.indeg[id], 1u);
    }
    if (lane == 0) a.g1_deg[x0] = deg;
}

// Stage 2 (Sec. 3.3): lambda_j = #{i : s0[i] < s0[j] and s(x_i,x_j) < s0[j]} (Eq. 1 over the whole list), counted by
// column j's two lanes over their sixteen rows of every block; then the order by (lambda, s, id) -- the list is in
// (s, id) order already, so an entry's rank is the number of entries with a smaller lambda plus those of equal
// lambda before it: one ballot per lambda value up to lambda0.
template <int NB>
__global__ __launch_bounds__(64 * kI8Waves) void stage2_i8_kernel(Stage2Args a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_i8[];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const int64_t x0 = linear_block() * kI8Waves + wave;
    if (x0 >= a.N) return;  // no barrier below
    const int R = a.rev_cap;
    const I8Slice z = i8_slice<NB>(smem_i8, wave, a.i8.dp8);

    const int m = a.g2_deg[x0];
    int32_t id = -1;
    float s = kInfD;
    if (lane < m) {
        id = a.g2_id[x0 * R + lane];
        s = a.g2_s[x0 * R + lane];
    }
    intx16 acc[2 * NB - 1];
    gram_of_list<NB>(a.i8, z, id, s, m, lane, acc);

    int part[2 * NB - 1];
#pragma unroll
    for (int blk = 0; blk < 2 * NB - 1; ++blk) {
        const int bi = blk >> 1, bj = (blk + 1) >> 1;
        part[blk] = 0;
        if (bj * 32 >= m) continue;
        const int j = bj * 32 + (lane & 31);
        const float sj = z.s0[j];
        const int nj = z.nrm[j];
        int c = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i0 = bi * 32 + 8 * q + 4 * (lane >> 5);
            const float4 si = *reinterpret_cast<const float4*>(z.s0 + i0);
            const intx4 ni = *reinterpret_cast<const intx4*>(z.nrm + i0);
            const float sv[4] = {si.x, si.y, si.z, si.w};
            const int nv[4] = {ni.x, ni.y, ni.z, ni.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float pij = (float)(nv[t] + nj - 2 * acc[blk][4 * q + t]);
                c += (sv[t] < sj && pij < sj) ? 1 : 0;
            }
        }
        part[blk] = c + __shfl_xor(c, 32, 64);
    }
    int lam = part[0];
    if constexpr (NB == 2) lam = lane < 32 ? part[0] : part[1] + part[2];

    // order by (lambda, s, id); entries with lambda <= lambda0 come first in it, cut to K
    const bool have = lane < m;
    int rank = -1, count = 0, lmax = 0;
    for (int v = 0; v <= a.lambda0 && count < a.K; ++v) {
        const uint64_t mv = ballot64(have && lam == v);
        if (!mv) continue;
        if (have && lam == v) rank = count + popc64(mv & lanes_below(lane));
        count += popc64(mv);
        lmax = v;   // some entry of this lambda has a rank below K
    }
    if (rank >= 0 && rank < a.K) a.packed[x0 * a.K + rank] = (uint32_t)id | ((uint32_t)lam << kIdBits);
    const int filled = min(count, a.K);
    for (int t = filled + lane; t < a.K; t += 64) a.packed[x0 * a.K + t] = kPackPad;
    if (lane == 0 && lmax > 0) atomicMax(&a.max_lambda[x0 % kLambdaSlots], lmax);
}

// ------------------------------------------------------------------ real-valued rows: Gram matrix with an error band
// The canonical distance of real-valued rows (fp32 difference, fp64 sum) has no exact matrix form, but the DECISIONS of
// Eq. 2 / Eq. 1 only compare s(x_i,x_j) with s0[j], and most of those comparisons are not close.  So the pairwise
// values come from the matrix cores as an approximation with a proven error band, and only a comparison that falls
// inside the band is decided by the canonical distance of that one pair (computed by the whole wavefront).  The
// adjacency that results is the one the general kernels (pairwise above) give; what changes is the work: each row
// of a list is read once instead of once per four pairs, and 2,016 canonical distances per node shrink to a handful.
//
// Approximation.  With y_i = fl32(x_i - x_0) (x_0 the node's own row; |y_i|^2 is s0[i] up to rounding),
// s(x_i,x_j) = |y_i|^2 + |y_j|^2 - 2 y_i.y_j up to rounding, and y_i.y_j is taken on v_mfma_f32_32x32x16_bf16 from
// y = hi + lo (bf16 each) as hi.hi + hi.lo + lo.hi with fp32 accumulation.  Error of P~ = s0[i] + s0[j] - 2 dot against
// the canonical s(x_i,x_j):
//   parts dropped or rounded (lo.lo, the remainder of hi + lo):      2 * 1.6 * 2^-18 * sqrt(s0[i] s0[j])
//   fp32 accumulation of 3 dp products:                              2 * 1.5 * dp * 2^-24 * sqrt(s0[i] s0[j])
//   fl32 of the differences x_i - x_j against y_i - y_j, of s0, of P~: below 2^-20 (s0[i] + s0[j])
// and sqrt(ab) <= (a + b) / 2, so |P~ - s| <= err * (s0[i] + s0[j]) with err = 1.5 * (1.6 * 2^-18 + 1.5 dp 2^-24 + 2^-20)
// (1.5: margin), plus a floor of 1e-30 that sends data at the bottom of the fp32 range (flushed by the matrix cores)
// to the exact path.  A value that is not finite (overflow of the products) counts as inside the band.  Both stages
// need s0[i] < s0[j] (times alpha^2 in stage 1) exactly, which they have: the s0 are canonical values.
constexpr int kSlab = 32;                 // elements of k per staging step
constexpr int kSlabStride = kSlab + 8;    // bf16 elements per staged row: 80 bytes, conflict-free 16-byte fragment reads

struct F32Slice {
    uint16_t* hi;      // [32 * NB][kSlabStride]
    uint16_t* lo;
    float* s0;         // [32 * NB], +inf beyond the list
    int32_t* ids;      // [32 * NB]
    uint64_t* fix;     // [32 * NB] what the exact path adds for column j (a count in stage 2, a mask in stage 1)
};
template <int NB> __host__ __device__ constexpr size_t f32_slice_bytes() { return (size_t)32 * NB * (2 * kSlabStride * 2 + 4 + 4 + 8); }
template <int NB> __device__ __forceinline__ F32Slice f32_slice(uint8_t* smem, int wave)
{
    F32Slice z;
    uint8_t* p = smem + (size_t)wave * f32_slice_bytes<NB>();
    z.fix = reinterpret_cast<uint64_t*>(p);
    z.hi = reinterpret_cast<uint16_t*>(p + 32 * NB * 8);
    z.lo = z.hi + 32 * NB * kSlabStride;
    z.s0 = reinterpret_cast<float*>(z.lo + 32 * NB * kSlabStride);
    z.ids = reinterpret_cast<int32_t*>(z.s0 + 32 * NB);
    return z;
}

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 dv_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float dv_floatx16;

__device__ __forceinline__ uint32_t dv_bf16_rne(float v)
{
    const uint32_t b = __float_as_uint(v);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

// canonical s(x_a, x_b) by all 64 lanes: fp32 differences, squares summed in fp64, one rounding
__device__ __forceinline__ float canonical_pair(const float* __restrict__ base, int d, int64_t a, int64_t b, int lane)
{
    double acc = 0.0;
    for (int k = 4 * lane; k < d; k += 256) {
        const float4 u = *reinterpret_cast<const float4*>(base + a * d + k);
        const float4 v = *reinterpret_cast<const float4*>(base + b * d + k);
        const float t0 = u.x - v.x, t1 = u.y - v.y, t2 = u.z - v.z, t3 = u.w - v.w;
        acc += (double)t0 * (double)t0;
        acc += (double)t1 * (double)t1;
        acc += (double)t2 * (double)t2;
        acc += (double)t3 * (double)t3;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += shfl_xor_f64(acc, o);
    return (float)acc;
}

// Lane e brings entry e of the list.  Leaves y_i.y_j of the list's rows (centred at the node) in acc, laid out as in
// gram_of_list: lane l, register r of block (bi,bj) holds the pair i = 32 bi + 8 (r / 4) + 4 (l / 32) + r % 4, j = 32 bj + l % 32.
template <int NB>
__device__ __forceinline__ void gram_of_list_f32(const float* __restrict__ base, int d, int64_t x0, const F32Slice& z,
                                                 int32_t id, float s, int m, int lane, dv_floatx16 (&acc)[2 * NB - 1])
{
    constexpr int ROWS = 32 * NB;
    constexpr int RT = ROWS / 8;   // rows this lane converts per slab
    if (lane < ROWS) {
        z.ids[lane] = lane < m ? id : (int32_t)x0;
        z.s0[lane] = lane < m ? s : kInfD;
        z.fix[lane] = 0ull;
    }
    wave_sync();
#pragma unroll
    for (int blk = 0; blk < 2 * NB - 1; ++blk)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[blk][r] = 0.f;
    const int kc = lane & 7;   // this lane's 16-byte chunk of a slab row
    int64_t rid[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) rid[t] = (int64_t)z.ids[(lane >> 3) + 8 * t];
    for (int k0 = 0; k0 < d; k0 += kSlab) {
        const int k = k0 + 4 * kc;
        const bool in = k < d;
        float4 c0 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (in) c0 = *reinterpret_cast<const float4*>(base + x0 * d + k);
        float4 v[RT];
#pragma unroll
        for (int t = 0; t < RT; ++t) {
            v[t] = c0;   // a row past the list, or a column past d, becomes a zero row / column
            if (in && (lane >> 3) + 8 * t < m) v[t] = *reinterpret_cast<const float4*>(base + rid[t] * d + k);
        }
        wave_sync();   // the fragment reads of the slab before are done
#pragma unroll
        for (int t = 0; t < RT; ++t) {
            const int r = (lane >> 3) + 8 * t;
            const float y[4] = {v[t].x - c0.x, v[t].y - c0.y, v[t].z - c0.z, v[t].w - c0.w};
            uint32_t h[4], l[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                h[e] = dv_bf16_rne(y[e]);
                l[e] = dv_bf16_rne(y[e] - __uint_as_float(h[e] << 16));
            }
            *reinterpret_cast<uint2*>(z.hi + r * kSlabStride + 4 * kc) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
            *reinterpret_cast<uint2*>(z.lo + r * kSlabStride + 4 * kc) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
        }
        wave_sync();
#pragma unroll
        for (int ks = 0; ks < kSlab / 16; ++ks) {
            dv_bf16x8 fh[NB], fl[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int off = (b * 32 + (lane & 31)) * kSlabStride + ks * 16 + 8 * (lane >> 5);
                fh[b] = __builtin_bit_cast(dv_bf16x8, *reinterpret_cast<const uint4*>(z.hi + off));
                fl[b] = __builtin_bit_cast(dv_bf16x8, *reinterpret_cast<const uint4*>(z.lo + off));
            }
#pragma unroll
            for (int blk = 0; blk < 2 * NB - 1; ++blk) {
                const int bi = blk >> 1, bj = (blk + 1) >> 1;
                if (bj * 32 >= m) continue;   // wave-uniform
                acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fh[bi], fh[bj], acc[blk], 0, 0, 0);
                acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fh[bi], fl[bj], acc[blk], 0, 0, 0);
                acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fl[bi], fh[bj], acc[blk], 0, 0, 0);
            }
        }
    }
}

// Decides "s(x_i,x_j) times f below s0[j]" (f = 1 in stage 2, alpha^2 in stage 1) for every pair of the list that
// passes `first` (the exact half of the rule), from the banded approximation; returns per block the pairs that are
// surely true (bit r of sure[blk]) and leaves the undecided ones in open[blk].
template <int NB, typename First>
__device__ __forceinline__ void banded_decisions(const F32Slice& z, const dv_floatx16 (&acc)[2 * NB - 1], int m, int lane, float f,
                                                 float err, First first, uint32_t (&sure)[2 * NB - 1], uint32_t (&open)[2 * NB - 1])
{
#pragma unroll
    for (int blk = 0; blk < 2 * NB - 1; ++blk) {
        const int bi = blk >> 1, bj = (blk + 1) >> 1;
        sure[blk] = 0u;
        open[blk] = 0u;
        if (bj * 32 >= m) continue;
        const float sj = z.s0[bj * 32 + (lane & 31)];
        const bool column = bj * 32 + (lane & 31) < m;   // a column past the list has s0 = +inf: nothing to decide there
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 si = *reinterpret_cast<const float4*>(z.s0 + bi * 32 + 8 * q + 4 * (lane >> 5));
            const float sv[4] = {si.x, si.y, si.z, si.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int r = 4 * q + t;
                const float sum = sv[t] + sj;
                const float p = sum - 2.f * acc[blk][r];
                const float e = err * sum + 1.0e-30f;
                const bool ft = column & first(sv[t], sj);
                const bool yes = f * (p + e) < sj;              // the canonical value is below p + e: surely true
                const bool no = f * fmaxf(p - e, 0.f) >= sj;    // and above p - e: surely false (false too when p is not finite)
                sure[blk] |= (uint32_t)(ft & yes) << r;
                open[blk] |= (uint32_t)(ft & !yes & !no) << r;
            }
        }
    }
}

// Runs `decide(i, j, s)` (wave-uniform arguments, s the canonical distance) for every undecided pair.
template <int NB, typename Decide>
__device__ __forceinline__ void settle_open_pairs(const float* __restrict__ base, int d, const F32Slice& z,
                                                  const uint32_t (&open)[2 * NB - 1], int lane, Decide decide)
{
#pragma unroll
    for (int blk = 0; blk < 2 * NB - 1; ++blk) {
        const int bi = blk >> 1, bj = (blk + 1) >> 1;
        if (!ballot64(open[blk] != 0u)) continue;
#pragma unroll 1
        for (int r = 0; r < 16; ++r) {
            for (uint64_t um = ballot64((open[blk] >> r) & 1u); um; um &= um - 1) {
                const int l = ctz64(um);
                const int i = bi * 32 + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3), j = bj * 32 + (l & 31);
                decide(i, j, canonical_pair(base, d, (int64_t)z.ids[i], (int64_t)z.ids[j], lane));
            }
        }
    }
}

struct F32Extra {
    float err;   // error band of the approximate pairwise distance, as a multiple of s0[i] + s0[j]
};

template <int NB>
__global__ __launch_bounds__(64 * kI8Waves) void stage1_f32_kernel(Stage1Args a, F32Extra x)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_f32[];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const int64_t x0 = linear_block() * kI8Waves + wave;
    if (x0 >= a.N) return;  // no barrier below
    const int K = a.K;
    const F32Slice z = f32_slice<NB>(smem_f32, wave);
    const float* __restrict__ base = static_cast<const float*>(a.base);

    int32_t id = -1;
    float s = kInfD;
    if (lane < K) {
        id = a.knn_id[x0 * K + lane];
        s = a.knn_s[x0 * K + lane];
    }
    const uint64_t used = ballot64(id >= 0);
    const int m = used ? 64 - __builtin_clzll(used) : 0;
    dv_floatx16 acc[2 * NB - 1];
    gram_of_list_f32<NB>(base, a.d, x0, z, id, s, m, lane, acc);

    const float alpha2 = a.alpha2;
    uint32_t sure[2 * NB - 1], open[2 * NB - 1];
    banded_decisions<NB>(z, acc, m, lane, alpha2, x.err, [alpha2](float si, float sj) { return alpha2 * si < sj; }, sure, open);
    settle_open_pairs<NB>(base, a.d, z, open, lane, [&](int i, int j, float sij) {
        if (lane == 0 && alpha2 * sij < z.s0[j]) z.fix[j] |= 1ull << i;
    });
    wave_sync();
    uint32_t part[2 * NB - 1];
#pragma unroll
    for (int blk = 0; blk < 2 * NB - 1; ++blk) {
        // register r of this lane is entry 8 (r / 4) + 4 (lane / 32) + r % 4 of the block's rows
        uint32_t bits = 0u;
#pragma unroll
        for (int r = 0; r < 16; ++r) bits |= ((sure[blk] >> r) & 1u) << (8 * (r >> 2) + (r & 3));
        bits <<= 4 * (lane >> 5);
        part[blk] = bits | (uint32_t)__shfl_xor((int)bits, 32, 64);
    }
    uint64_t occ = part[0];
    if constexpr (NB == 2) occ = lane < 32 ? (uint64_t)part[0] : ((uint64_t)part[1] | ((uint64_t)part[2] << 32));
    if (lane < 32 * NB) occ |= z.fix[lane];
    uint64_t kept = m > 0 ? 1ull : 0ull;
    for (int j = 1; j < m; ++j) {
        const uint64_t oj = readlane64(occ, j);
        if ((oj & kept) == 0ull) kept |= 1ull << j;
    }
    const int deg = popc64(kept);
    const bool mine = (kept >> lane) & 1ull;
    const int pos = popc64(kept & lanes_below(lane));
    if (lane < K && lane >= deg) {
        a.g1_id[x0 * K + lane] = -1;
        a.g1_s[x0 * K + lane] = kInfD;
    }
    if (mine) {
        a.g1_id[x0 * K + pos] = id;
        a.g1_s[x0 * K + pos] = s;
        atomicAdd(&a.indeg[id], 1u);
    }
    if (lane == 0) a.g1_deg[x0] = deg;
}

template <int NB>
__global__ __launch_bounds__(64 * kI8Waves) void stage2_f32_kernel(Stage2Args a, F32Extra x)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_f32[];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const int64_t x0 = linear_block() * kI8Waves + wave;
    if (x0 >= a.N) return;  // no barrier below
    const int R = a.rev_cap;
    const F32Slice z = f32_slice<NB>(smem_f32, wave);
    const float* __restrict__ base = static_cast<const float*>(a.base);

    const int m = a.g2_deg[x0];
    int32_t id = -1;
    float s = kInfD;
    if (lane < m) {
        id = a.g2_id[x0 * R + lane];
        s = a.g2_s[x0 * R + lane];
    }
    dv_floatx16 acc[2 * NB - 1];
    gram_of_list_f32<NB>(base, a.d, x0, z, id, s, m, lane, acc);

    uint32_t sure[2 * NB - 1], open[2 * NB - 1];
    banded_decisions<NB>(z, acc, m, lane, 1.f, x.err, [](float si, float sj) { return si < sj; }, sure, open);
    settle_open_pairs<NB>(base, a.d, z, open, lane, [&](int i, int j, float sij) {
        (void)i;
        if (lane == 0 && sij < z.s0[j]) z.fix[j] += 1ull;
    });
    wave_sync();
    int part[2 * NB - 1];
#pragma unroll
    for (int blk = 0; blk < 2 * NB - 1; ++blk) {
        const int c = __popc(sure[blk]);
        part[blk] = c + __shfl_xor(c, 32, 64);
    }
    int lam = part[0];
    if constexpr (NB == 2) lam = lane < 32 ? part[0] : part[1] + part[2];
    if (lane < 32 * NB) lam += (int)z.fix[lane];

    const bool have = lane < m;
    int rank = -1, count = 0, lmax = 0;
    for (int v = 0; v <= a.lambda0 && count < a.K; ++v) {
        const uint64_t mv = ballot64(have && lam == v);
        if (!mv) continue;
        if (have && lam == v) rank = count + popc64(mv & lanes_below(lane));
        count += popc64(mv);
        lmax = v;
    }
    if (rank >= 0 && rank < a.K) a.packed[x0 * a.K + rank] = (uint32_t)id | ((uint32_t)lam << kIdBits);
    const int filled = min(count, a.K);
    for (int t = filled + lane; t < a.K; t += 64) a.packed[x0 * a.K + t] = kPackPad;
    if (lane == 0 && lmax > 0) atomicMax(&a.max_lambda[x0 % kLambdaSlots], lmax);
}

// ------------------------------------------------------------------ host driver
namespace {
struct DevBuf {
    void* p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 16); }
    template <typename T> T* as() { return static_cast<T*>(p); }
};

struct Stage1Launch {
    Stage1Args a;
    hipStream_t stream;
    hipError_t err = hipSuccess;
    template <typename T, int G, int C> void operator()()
    {
        size_t lds = (size_t)a.K * a.K * 4 + (size_t)a.K * 8;
        if (lds > 64 * 1024)
            err = hipFuncSetAttribute(reinterpret_cast<const void*>(&stage1_kernel<T, G, C>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        TSDG_LAUNCH((stage1_kernel<T, G, C>), folded_grid(a.N), dim3(64), lds, stream, a);
    }
};
struct Stage2Launch {
    Stage2Args a;
    hipStream_t stream;
    hipError_t err = hipSuccess;
    template <typename T, int G, int C> void operator()()
    {
        size_t lds = (size_t)a.rev_cap * a.rev_cap * 4 + (size_t)a.rev_cap * 12;
        if (lds > 64 * 1024)
            err = hipFuncSetAttribute(reinterpret_cast<const void*>(&stage2_kernel<T, G, C>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        TSDG_LAUNCH((stage2_kernel<T, G, C>), folded_grid(a.N), dim3(64), lds, stream, a);
    }
};
}  // namespace

// sum of n 32-bit counts into *out (64-bit): one atomic per workgroup; only run when a build report is asked for
__global__ __launch_bounds__(256) void sum_counts_kernel(const int32_t* __restrict__ v, int64_t n,
                                                         unsigned long long* __restrict__ out)
{
    __shared__ unsigned long long part[4];
    unsigned long long acc = 0;
    const int64_t i0 = linear_block() * 1024, i1 = i0 + 1024 < n ? i0 + 1024 : n;
    for (int64_t i = i0 + threadIdx.x; i < i1; i += 256) acc += (unsigned long long)v[i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const unsigned lo = (unsigned)__shfl_xor((int)(unsigned)acc, o, 64);
        const unsigned hi = (unsigned)__shfl_xor((int)(unsigned)(acc >> 32), o, 64);
        acc += ((unsigned long long)hi << 32) | lo;
    }
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) atomicAdd(out, part[0] + part[1] + part[2] + part[3]);
}

ann_status diversify(const void* base, int64_t N, int d, ann_dtype dtype, int K, const int32_t* knn_id,
                     const float* knn_s, float alpha_on_s, int lambda0, int rev_cap, hipStream_t stream, uint32_t* packed,
                     int* max_lambda, const BuildCtx& ctx)
{
    // device time of the three steps for the caller's report: events on the build's stream
    struct Marks {
        hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
        ~Marks() { for (hipEvent_t e : ev) if (e) (void)hipEventDestroy(e); }
    } marks;
    const bool timed = ctx.stats != nullptr;
    if (timed)
        for (hipEvent_t& e : marks.ev) TSDG_HIP(hipEventCreate(&e));

    DevBuf g1_id, g1_s, g1_deg, indeg, cursor, start, bsums, rev_src, rev_s, g2_id, g2_s, g2_deg, mlam;
    const size_t nk = (size_t)N * K;
    TSDG_HIP(g1_id.alloc(nk * 4));
    TSDG_HIP(g1_s.alloc(nk * 4));
    TSDG_HIP(g1_deg.alloc((size_t)N * 4));
    TSDG_HIP(indeg.alloc((size_t)N * 4));
    TSDG_HIP(cursor.alloc((size_t)N * 4));
    TSDG_HIP(start.alloc(((size_t)N + 1) * 8));
    const int64_t nb = (N + kScanBlock - 1) / kScanBlock;
    TSDG_HIP(bsums.alloc(((size_t)nb + 1) * 8));
    TSDG_HIP(mlam.alloc(kLambdaSlots * sizeof(int)));
    TSDG_HIP(hipMemsetAsync(indeg.p, 0, (size_t)N * 4, stream));
    TSDG_HIP(hipMemsetAsync(cursor.p, 0, (size_t)N * 4, stream));
    TSDG_HIP(hipMemsetAsync(mlam.p, 0, kLambdaSlots * sizeof(int), stream));

    // Rows that are integers in [0,255] (uint8 storage, or fp32 that passes the test) with lists of at
    // most 64 entries take their pairwise distances from the int8 matrix cores.
    DevBuf xc8, xn8, notint;
    I8Rows i8{nullptr, nullptr, 0};
    const int dp8 = (d + 31) / 32 * 32;
    if (K <= 64 && rev_cap <= 64 && dp8 <= 256) {
        TSDG_HIP(xc8.alloc((size_t)N * dp8));
        TSDG_HIP(xn8.alloc((size_t)N * 4));
        TSDG_HIP(notint.alloc(4));
        TSDG_HIP(hipMemsetAsync(notint.p, 0, 4, stream));
        if (dtype == ANN_U8)
            TSDG_LAUNCH((i8_prep_kernel<uint8_t>), folded_grid((N + 31) / 32), dim3(256), 0, stream,
                               static_cast<const uint8_t*>(base), N, d, dp8, xc8.as<uint8_t>(), xn8.as<int>(),
                               notint.as<unsigned>());
        else
            TSDG_LAUNCH((i8_prep_kernel<float>), folded_grid((N + 31) / 32), dim3(256), 0, stream,
                               static_cast<const float*>(base), N, d, dp8, xc8.as<uint8_t>(), xn8.as<int>(),
                               notint.as<unsigned>());
        TSDG_HIP(launch_error());
        unsigned h_notint = 1;
        TSDG_HIP(hipMemcpyAsync(&h_notint, notint.p, 4, hipMemcpyDeviceToHost, stream));
        TSDG_HIP(hipStreamSynchronize(stream));
        if (h_notint == 0) i8 = I8Rows{xc8.as<uint8_t>(), xn8.as<int>(), dp8};
    }

    // stage 1
    if (timed) TSDG_HIP(hipEventRecord(marks.ev[0], stream));
    Stage1Launch s1;
    s1.a.base = base;
    s1.a.knn_id = knn_id;
    s1.a.knn_s = knn_s;
    s1.a.g1_id = g1_id.as<int32_t>();
    s1.a.g1_s = g1_s.as<float>();
    s1.a.g1_deg = g1_deg.as<int32_t>();
    s1.a.indeg = indeg.as<unsigned>();
    s1.a.N = N;
    s1.a.d = d;
    s1.a.K = K;
    s1.a.alpha2 = alpha_on_s;
    s1.a.i8 = i8;
    s1.stream = stream;
    const dim3 i8_grid = folded_grid((N + kI8Waves - 1) / kI8Waves);
    const bool banded = !i8.xc8 && dtype == ANN_F32 && K <= 64 && rev_cap <= 64;
    F32Extra fx;
    {
        const double dpad = (double)((d + kSlab - 1) / kSlab * kSlab);
        fx.err = (float)(1.5 * (1.6 / 262144.0 + 1.5 * dpad / 16777216.0 + 1.0 / 1048576.0));
    }
    if (i8.xc8 && kI8Waves * i8_slice_bytes<2>(dp8) > 64 * 1024) {   // only rows wider than 192 bytes get there
        for (const void* f : {reinterpret_cast<const void*>(&stage1_i8_kernel<2>), reinterpret_cast<const void*>(&stage2_i8_kernel<2>)})
            TSDG_HIP(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kI8Waves * i8_slice_bytes<2>(dp8))));
    }
    if (i8.xc8) {   // integer rows: decisions taken on the matrix cores' accumulators
        if (K <= 32)
            TSDG_LAUNCH(stage1_i8_kernel<1>, i8_grid, dim3(64 * kI8Waves), kI8Waves * i8_slice_bytes<1>(dp8), stream, s1.a);
        else
            TSDG_LAUNCH(stage1_i8_kernel<2>, i8_grid, dim3(64 * kI8Waves), kI8Waves * i8_slice_bytes<2>(dp8), stream, s1.a);
    } else if (banded) {   // real-valued fp32 rows, lists of at most 64: banded Gram matrix, exact only inside the band
        if (K <= 32)
            TSDG_LAUNCH(stage1_f32_kernel<1>, i8_grid, dim3(64 * kI8Waves), kI8Waves * f32_slice_bytes<1>(), stream, s1.a, fx);
        else
            TSDG_LAUNCH(stage1_f32_kernel<2>, i8_grid, dim3(64 * kI8Waves), kI8Waves * f32_slice_bytes<2>(), stream, s1.a, fx);
    } else if (!dispatch_row_shape(dtype, d, s1)) {
        set_error("unsupported row shape d=%d", d);
        return ANN_EUNSUPPORTED;
    }
    TSDG_HIP(s1.err);
    TSDG_HIP(launch_error());

    // reverse edges: scan of in-degrees, scatter, per-node merge
    if (timed) TSDG_HIP(hipEventRecord(marks.ev[1], stream));
    TSDG_LAUNCH(scan_partial, dim3((unsigned)nb), dim3(256), 0, stream, indeg.as<unsigned>(), N,
                       bsums.as<uint64_t>());
    TSDG_LAUNCH(scan_block_sums, dim3(1), dim3(64), 0, stream, bsums.as<uint64_t>(), nb);
    TSDG_LAUNCH(scan_final, dim3((unsigned)nb), dim3(256), 0, stream, indeg.as<unsigned>(), N,
                       bsums.as<uint64_t>(), start.as<uint64_t>());
    TSDG_HIP(launch_error());
    uint64_t total = 0;
    TSDG_HIP(hipMemcpyAsync(&total, start.as<uint64_t>() + N, 8, hipMemcpyDeviceToHost, stream));
    TSDG_HIP(hipStreamSynchronize(stream));
    TSDG_HIP(rev_src.alloc((size_t)total * 4));
    TSDG_HIP(rev_s.alloc((size_t)total * 4));
    TSDG_LAUNCH(scatter_kernel, folded_grid((int64_t)((nk + 255) / 256)), dim3(256), 0, stream, g1_id.as<int32_t>(),
                       g1_s.as<float>(), (int64_t)nk, K, start.as<uint64_t>(), cursor.as<unsigned>(),
                       rev_src.as<int32_t>(), rev_s.as<float>());
    TSDG_HIP(launch_error());

    const size_t nr = (size_t)N * rev_cap;
    TSDG_HIP(g2_id.alloc(nr * 4));
    TSDG_HIP(g2_s.alloc(nr * 4));
    TSDG_HIP(g2_deg.alloc((size_t)N * 4));
    MergeArgs m;
    m.g1_id = g1_id.as<int32_t>();
    m.g1_s = g1_s.as<float>();
    m.g1_deg = g1_deg.as<int32_t>();
    m.start = start.as<uint64_t>();
    m.rev_src = rev_src.as<int32_t>();
    m.rev_s = rev_s.as<float>();
    m.g2_id = g2_id.as<int32_t>();
    m.g2_s = g2_s.as<float>();
    m.g2_deg = g2_deg.as<int32_t>();
    m.N = N;
    m.K = K;
    m.rev_cap = rev_cap;
    TSDG_LAUNCH(merge_kernel, folded_grid(N), dim3(64), (size_t)((rev_cap + 63) & ~63) * 8, stream, m);
    TSDG_HIP(launch_error());

    // stage 2
    if (timed) TSDG_HIP(hipEventRecord(marks.ev[2], stream));
    Stage2Launch s2;
    s2.a.base = base;
    s2.a.g2_id = g2_id.as<int32_t>();
    s2.a.g2_s = g2_s.as<float>();
    s2.a.g2_deg = g2_deg.as<int32_t>();
    s2.a.packed = packed;
    s2.a.max_lambda = mlam.as<int>();
    s2.a.N = N;
    s2.a.d = d;
    s2.a.K = K;
    s2.a.rev_cap = rev_cap;
    s2.a.lambda0 = lambda0;
    s2.a.i8 = i8;
    s2.stream = stream;
    if (i8.xc8) {
        if (rev_cap <= 32)
            TSDG_LAUNCH(stage2_i8_kernel<1>, i8_grid, dim3(64 * kI8Waves), kI8Waves * i8_slice_bytes<1>(dp8), stream, s2.a);
        else
            TSDG_LAUNCH(stage2_i8_kernel<2>, i8_grid, dim3(64 * kI8Waves), kI8Waves * i8_slice_bytes<2>(dp8), stream, s2.a);
    } else if (banded) {
        if (rev_cap <= 32)
            TSDG_LAUNCH(stage2_f32_kernel<1>, i8_grid, dim3(64 * kI8Waves), kI8Waves * f32_slice_bytes<1>(), stream, s2.a, fx);
        else
            TSDG_LAUNCH(stage2_f32_kernel<2>, i8_grid, dim3(64 * kI8Waves), kI8Waves * f32_slice_bytes<2>(), stream, s2.a, fx);
    } else {
        dispatch_row_shape(dtype, d, s2);
    }
    TSDG_HIP(s2.err);
    TSDG_HIP(launch_error());
    if (timed) TSDG_HIP(hipEventRecord(marks.ev[3], stream));
    int h_lam[kLambdaSlots];
    TSDG_HIP(hipMemcpyAsync(h_lam, mlam.p, sizeof(h_lam), hipMemcpyDeviceToHost, stream));
    unsigned long long h_rows[2] = {0, 0};
    DevBuf rows;
    if (timed) {
        TSDG_HIP(rows.alloc(sizeof(h_rows)));
        TSDG_HIP(hipMemsetAsync(rows.p, 0, sizeof(h_rows), stream));
        // stage 1 reads each node's own row and the rows of its k-NN list (its length is K, short only when the
        // propagation left a list unfilled: then the padding -1 entries are not read, counted here as read)
        TSDG_LAUNCH(sum_counts_kernel, folded_grid((N + 1023) / 1024), dim3(256), 0, stream, g2_deg.as<int32_t>(), N,
                    rows.as<unsigned long long>());
        TSDG_HIP(launch_error());
        TSDG_HIP(hipMemcpyAsync(h_rows, rows.p, sizeof(h_rows), hipMemcpyDeviceToHost, stream));
    }
    TSDG_HIP(hipStreamSynchronize(stream));
    *max_lambda = *std::max_element(h_lam, h_lam + kLambdaSlots);
    if (timed) {
        ann_build_stats& st = *ctx.stats;
        TSDG_HIP(hipEventElapsedTime(&st.stage1_ms, marks.ev[0], marks.ev[1]));
        TSDG_HIP(hipEventElapsedTime(&st.reverse_ms, marks.ev[1], marks.ev[2]));
        TSDG_HIP(hipEventElapsedTime(&st.stage2_ms, marks.ev[2], marks.ev[3]));
        st.stage1_rows = (uint64_t)N * (uint64_t)(K + 1);
        st.stage2_rows = (uint64_t)N + (uint64_t)h_rows[0];
        st.reverse_edges = total;
        st.gather_row_bytes = i8.xc8 ? dp8 : d * (dtype == ANN_U8 ? 1 : 4);
    }
    return ANN_OK;
}

}  // namespace tsdg
