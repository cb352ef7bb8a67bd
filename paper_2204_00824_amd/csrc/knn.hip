// Exact k nearest neighbours of a set of query rows against the whole base set
// (build step B1 + B1r; also the brute-force ground truth).
//
// The squared distance is expanded as |q|^2 + |x|^2 - 2 q.x and the cross term is
// a dense contraction on the matrix cores:
//   * rows that are integers in [0,255] with d <= 128 (uint8 rows, SIFT-like fp32 rows) are
//     centred to int8 and go through the integer matrix cores (v_mfma_i32_32x32x32_i8), exact;
//     such rows of 129..1024 elements go through bf16 MFMA with both operands staged in LDS, one
//     MFMA per k-step: centred to x - 128 they are exact in bf16 and every partial sum is an integer
//     of at most 2^24 in magnitude, so the fp32 accumulators are exact and the filter runs in int32;
//   * real-valued rows (and integer rows wider than 1024) are centred and written as one scaled binary16
//     part, one v_mfma_f32_32x32x16_f16 per k-step (relative error 2^-10 of the norms, carried by the
//     acceptance test below); when that margin rejects too many rows the call starts over with bf16
//     hi + lo parts, three v_mfma_f32_32x32x16_bf16 per k-step, an error near that of fp32 accumulation.
//     Either way the query fragments stay in registers up to d = 128 and both operands are staged
//     through LDS beyond.
// The contraction only SELECTS candidates: each query row keeps the K' = 2k
// smallest approximate distances (K' = k + max(8, k/4) where the filter is exact) through a
// threshold filter fused into the tile epilogue.  The base columns are swept in chunks of doubling
// size; after each chunk a per-row pass keeps the K' smallest of the row's buffer and lowers the row's
// threshold, so the expected number of survivors per chunk stays near K' ln 2.
// The kept candidates are then re-scored with the canonical distance, sorted by
// (s, id) and cut to k.  A row is accepted only if its k-th canonical distance
// lies below the final threshold minus a bound on the expansion's rounding
// error (no rejected column can then belong to the answer, ties included);
// rows that fail, or whose buffer overflowed, are redone by a plain scan of
// all base rows with the canonical distance.
#include <algorithm>
#include <cmath>
#include <type_traits>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "dist.hpp"
#include "i8rows.hpp"
#include "ranklist.hpp"

namespace tsdg {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef _Float16 half8 __attribute__((ext_vector_type(8)));

constexpr int kTile = 128;        // queries and candidates per workgroup tile
constexpr float kInf = __builtin_inff();

__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load4(const uint8_t* p)
{
    const uint32_t w = *reinterpret_cast<const uint32_t*>(p);
    return make_float4((float)(w & 0xFFu), (float)((w >> 8) & 0xFFu), (float)((w >> 16) & 0xFFu), (float)(w >> 24));
}

// ---------------------------------------------------------------- row norms, integer test
// info[0] = 1 if some element is not an integer in [0,255]; info[1] = max norm (fp32 bits)
constexpr int kNormPasses = 8;   // a workgroup walks through 8 x 32 rows and looks at the shared maximum once per wave

template <typename T>
__global__ __launch_bounds__(256) void norms_kernel(const T* __restrict__ x, int64_t n, int d,
                                                    float* __restrict__ norms, unsigned* info)
{
    // 8 lanes per row, 4 elements per lane and step (128 contiguous bytes per group for fp32)
    const int g = (int)(threadIdx.x & 7);
    bool nonint = false;
    unsigned m = 0u;   // largest norm this lane has seen (norms are not negative: bit patterns order like values)
    for (int pass = 0; pass < kNormPasses; ++pass) {
        const int64_t row = (linear_block() * kNormPasses + pass) * 32 + (threadIdx.x >> 3);
        double acc = 0.0;
        if (row < n) {
            const T* xr = x + row * d;
            for (int j = 4 * g; j < d; j += 32) {
                const float4 v = load4(xr + j);
                acc += (double)v.x * (double)v.x;
                acc += (double)v.y * (double)v.y;
                acc += (double)v.z * (double)v.z;
                acc += (double)v.w * (double)v.w;
                if constexpr (sizeof(T) != 1) {
                    nonint |= !(v.x >= 0.f && v.x <= 255.f && v.x == rintf(v.x));
                    nonint |= !(v.y >= 0.f && v.y <= 255.f && v.y == rintf(v.y));
                    nonint |= !(v.z >= 0.f && v.z <= 255.f && v.z == rintf(v.z));
                    nonint |= !(v.w >= 0.f && v.w <= 255.f && v.w == rintf(v.w));
                }
            }
        }
#pragma unroll
        for (int o = 4; o > 0; o >>= 1) acc += shfl_xor_f64(acc, o);
        const float nf = (float)acc;
        if (row < n && g == 0) norms[row] = nf;
        if (row < n) m = max(m, __float_as_uint(nf));
    }
    // the wave's largest norm, then at most one atomic per wave, and only when the value read
    // first is smaller (the maximum only grows, so a stale read costs a harmless extra atomic)
#pragma unroll
    for (int o = 32; o >= 8; o >>= 1) m = max(m, (unsigned)__shfl_xor((int)m, o, 64));
    const int lane = lane_id();
    if (lane == 0 && m > info[1]) atomicMax(&info[1], m);
    if (ballot64(nonint) && lane == 0 && info[0] == 0u) atomicOr(&info[0], 1u);
}

// what every contraction launch of one row block shares
struct FilterArgs {
    const void* q;        // [nq, d] query rows (type TQ), row 0 = global query q_begin
    const void* x;        // [N, d] base rows (type TB)
    const float* qnorm;   // [nq]
    const float* xnorm;   // [N]
    const float* tau;     // [nq] current thresholds
    unsigned* cnt;        // [nq] entries in each row's buffer
    uint64_t* buf;        // [nq, cap]  (approx distance bits << 32 | id)
    int64_t nq, N;
    int64_t c_begin, c_end;   // column chunk
    int64_t self_offset;      // global id of query row 0 when queries are base rows, else -1
    int d, cap;
};

constexpr int kSplitRows = 64;  // candidate rows per LDS tile of the bf16 split kernel
constexpr int kQueue = 1024;    // survivor queue entries per workgroup

// The survivors of a workgroup's sweep wait in LDS and go to their rows' global buffers in bursts, issued
// by all 256 threads at once instead of one by one from inside the sweep.
template <int CAPQ>
struct SurvivorQueue {
    uint64_t key[CAPQ];
    uint16_t row[CAPQ];   // query row, counted from the workgroup's first
    unsigned count;

    // any lane, any time between two flushes; a full queue sends the entry straight to the global buffer
    __device__ __forceinline__ void push(uint64_t k, int row_in_group, int64_t global_row, unsigned* cnt, uint64_t* buf, int cap)
    {
        const unsigned slot = atomicAdd(&count, 1u);
        if (slot < (unsigned)CAPQ) {
            key[slot] = k;
            row[slot] = (uint16_t)row_in_group;
        } else {
            const unsigned pos = atomicAdd(&cnt[global_row], 1u);
            if (pos < (unsigned)cap) buf[global_row * cap + pos] = k;
        }
    }
    // all THREADS threads of the workgroup, after a barrier that follows the last push; empties the queue once it is half full
    // (or holds anything and `last` is set).  row0 = global row of the workgroup's first query.
    template <int THREADS = 256>
    __device__ __forceinline__ void flush(int64_t row0, unsigned* cnt, uint64_t* buf, int cap, bool last)
    {
        const unsigned queued = count;
        if (queued >= (unsigned)CAPQ / 2 || (last && queued > 0)) {
            const unsigned n = min(queued, (unsigned)CAPQ);
            for (unsigned e = threadIdx.x; e < n; e += THREADS) {
                const int64_t r = row0 + row[e];
                const unsigned pos = atomicAdd(&cnt[r], 1u);
                if (pos < (unsigned)cap) buf[r * cap + pos] = key[e];
            }
            __syncthreads();
            if (threadIdx.x == 0) count = 0u;
            __syncthreads();
        }
    }
};

// ---------------------------------------------------------------- int8 path (integer rows in [0,255], d <= 128)
// The same sweep on the integer matrix cores (v_mfma_i32_32x32x32_i8: twice the rate of bf16 and
// half the bytes per element in LDS).  Rows are rewritten once as x' = x - 128 (int8, padded with
// zeros to 32-element steps); ||q - x||^2 = |q'|^2 + |x'|^2 - 2 q'.x' holds for the centred rows,
// and all of it is exact in int32.  -2q' does not fit a byte, so the accumulators start at
// -(|x'|^2 >> 1) and end as  a = q'.x' - (|x'|^2 >> 1), i.e.  u = |x'|^2 - 2 q'.x' = (|x'|^2 & 1) - 2a.
// The hot test "some a above floor((|q'|^2 - tau) / 2)" lets every survivor through (it ignores
// the parity bit); the rare path then tests u < tau - |q'|^2 exactly.
struct I8Args {
    const uint8_t* qc;    // [nq, DP] centred int8 query rows (row 0 = first query of this sweep)
    const uint8_t* xc;    // [N, DP] centred int8 base rows
    const int* qnorm;     // |q'|^2
    const int* xnorm;     // |x'|^2
    const float* tau;
    unsigned* cnt;
    uint64_t* buf;
    int64_t nq;
    int64_t c_begin, c_end;
    int64_t self_offset;
    int cap, tiles_per_block;
};

constexpr int kI8Rows = 128;  // candidate rows per LDS tile of the int8 kernel (two 64-row halves per barrier)

template <int KS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void filter_i8_kernel(I8Args a)
{
    constexpr int DP = KS * 32;                      // bytes per row
    constexpr int XS = DP + 16;                      // LDS row stride (bytes): 16-B aligned, staggers banks
    constexpr int CHUNKS = kI8Rows * DP / 16;      // 16-byte chunks per tile
    constexpr int PER_THREAD = (CHUNKS + 255) / 256;
    __shared__ __attribute__((aligned(16))) uint8_t Xs[2][kI8Rows * XS];
    __shared__ __attribute__((aligned(16))) int xstart[2][kI8Rows];   // -(|x'|^2 >> 1)
    __shared__ int xpar[2][kI8Rows];                                  // |x'|^2 & 1
    __shared__ SurvivorQueue<kQueue> queue;

    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const int64_t q0 = (int64_t)blockIdx.x * 256 + wave * 64;
    if (threadIdx.x == 0) queue.count = 0u;

    intx4 qf[2][KS];
    int64_t qg[2];
    int qn[2], tq[2], thr[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        qg[j] = q0 + j * 32 + (lane & 31);
        const bool ok = qg[j] < a.nq;
        qn[j] = ok ? a.qnorm[qg[j]] : 0;
        // survivors satisfy u < tau - |q'|^2; tau is an integer-valued float or +inf
        const float tf = ok ? a.tau[qg[j]] : -1.f;
        tq[j] = ok ? (tf < 1.0e9f ? (int)tf - qn[j] : (1 << 30)) : -(1 << 30);
        thr[j] = (-tq[j]) >> 1;                      // floor((|q'|^2 - tau) / 2)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            intx4 w = {0, 0, 0, 0};
            if (ok) w = *reinterpret_cast<const intx4*>(a.qc + qg[j] * DP + ks * 32 + 16 * (lane >> 5));
            qf[j][ks] = w;
        }
    }

    const int64_t span0 = a.c_begin + (int64_t)blockIdx.y * a.tiles_per_block * kI8Rows;
    const int64_t span1 = min(a.c_end, span0 + (int64_t)a.tiles_per_block * kI8Rows);
    if (span0 >= span1) return;
    const int ntiles = (int)((span1 - span0 + kI8Rows - 1) / kI8Rows);

    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // a plain vector: stays in registers
    struct Stage {
        u32x4 x[PER_THREAD];
        int n;
    };
    // A tile is one contiguous block of kI8Rows * DP bytes and this thread's chunks sit at fixed
    // offsets inside it.  No branch: a chunk index past the span's end is clamped to the span's
    // last chunk (rows read twice that way carry ids >= span1 and are dropped by the filter).
    const uint8_t* xspan = a.xc + span0 * DP;
    const int last_chunk = (int)(span1 - span0) * (DP / 16) - 1;
    const int last_row = (int)(span1 - span0) - 1;
    auto fetch = [&](int t, Stage& st) __attribute__((always_inline)) {       // global -> registers
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int ch = min((int)threadIdx.x + i * 256, CHUNKS - 1);
            st.x[i] = *reinterpret_cast<const u32x4*>(xspan + (int64_t)min(t * CHUNKS + ch, last_chunk) * 16);
        }
        st.n = 0;
        if (threadIdx.x < kI8Rows) st.n = a.xnorm[span0 + min(t * kI8Rows + (int)threadIdx.x, last_row)];
    };
    auto commit = [&](int b, const Stage& st) __attribute__((always_inline)) {      // registers -> LDS buffer b
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int ch = (int)threadIdx.x + i * 256;
            const int r = ch / (DP / 16), c16 = ch % (DP / 16);
            if (ch < CHUNKS) *reinterpret_cast<u32x4*>(&Xs[b][r * XS + c16 * 16]) = st.x[i];
        }
        if (threadIdx.x < kI8Rows) {
            xstart[b][threadIdx.x] = -(st.n >> 1);
            xpar[b][threadIdx.x] = st.n & 1;
        }
    };

    // The loads of tile t+1 are in flight while tile t (in LDS buffer t & 1) is multiplied.
    // Fetches past the last tile are clamped re-reads that nobody uses.
    Stage st;
    fetch(0, st);
    commit(0, st);
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const int cur = t & 1;
        fetch(t + 1, st);
        for (int h = 0; h < kI8Rows / 64; ++h) {   // the tile's 64-row halves, one after the other
            // lane l, register r of a 32x32 block holds candidate row 8*(r/4) + 4*(l/32) + r%4
            intx16 acc[2][2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const intx4 v = *reinterpret_cast<const intx4*>(&xstart[cur][h * 64 + i * 32 + 8 * r4 + 4 * (lane >> 5)]);
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        acc[i][j][4 * r4 + 0] = v.x; acc[i][j][4 * r4 + 1] = v.y;
                        acc[i][j][4 * r4 + 2] = v.z; acc[i][j][4 * r4 + 3] = v.w;
                    }
                }
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                intx4 xa[2];
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    xa[i] = *reinterpret_cast<const intx4*>(
                        &Xs[cur][(h * 64 + i * 32 + (lane & 31)) * XS + ks * 32 + 16 * (lane >> 5)]);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xa[i], qf[j][ks], acc[i][j], 0, 0, 0);
            }
            const int64_t c0 = span0 + (int64_t)t * kI8Rows + h * 64;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    int hi = max(acc[i][j][0], acc[i][j][1]);
#pragma unroll
                    for (int r = 2; r < 16; r += 2) hi = max(max(hi, acc[i][j][r]), acc[i][j][r + 1]);
                    if (ballot64(hi > thr[j])) {
                        uint32_t mask = 0;
#pragma unroll
                        for (int r = 0; r < 16; ++r) mask |= (acc[i][j][r] > thr[j]) ? (1u << r) : 0u;
                        // rare: walk the set bits; the accumulator is picked by a select chain so
                        // that the loop needs no indexed register access
#pragma unroll 1
                        while (ballot64(mask != 0u)) {
                            const int rr = mask ? (int)__builtin_ctz(mask) : 16;
                            mask &= mask - 1u;
                            int av = 0;
#pragma unroll
                            for (int r = 0; r < 16; ++r) av = rr == r ? acc[i][j][r] : av;
                            const int m = i * 32 + 8 * (rr >> 2) + 4 * (lane >> 5) + (rr & 3);
                            const int64_t c = c0 + m;
                            const int u = xpar[cur][(h * 64 + m) & (kI8Rows - 1)] - 2 * av;   // |x'|^2 - 2 q'.x', exact
                            if (rr < 16 && u < tq[j] && c < span1 && c != a.self_offset + qg[j]) {
                                const uint64_t key =
                                    ((uint64_t)__float_as_uint((float)max(u + qn[j], 0)) << 32) | (uint64_t)(uint32_t)c;
                                queue.push(key, wave * 64 + j * 32 + (lane & 31), qg[j], a.cnt, a.buf, a.cap);
                            }
                        }
                    }
                }
            }
        }
        if (t + 1 < ntiles) commit(cur ^ 1, st);
        __syncthreads();
        queue.flush((int64_t)blockIdx.x * 256, a.cnt, a.buf, a.cap, t + 1 == ntiles);
    }
}

// ---------------------------------------------------------------- real-valued rows, d <= 128
// A real-valued row is centred (global mean removed: distances do not change, norms shrink).  The
// form tried first writes it as one binary16 part (half_prep_kernel, filter_split_kernel<KS, true>).
// The fallback writes it as x = hi + lo with hi = bf16(x), lo = bf16(x - hi), both round-to-nearest; what is
// left is below 2^-16 |x|.  q.x is taken as hi.hi + hi.lo + lo.hi on the bf16 matrix cores
// (three MFMAs per k-step, products exact in fp32), which is 16/3 times the fp32-MFMA rate at
// nearly the same accuracy: |error of q.x| <= (3*2^-16 + 3d*2^-24) sum|q_j||x_j|; the
// accumulators also carry |x|^2 from the start, which doubles the accumulation term.  The
// result only SELECTS candidates; the acceptance test of the re-scoring pass carries the
// bound.  One wave owns 64 queries (hi and lo fragments in registers: every candidate fragment
// read from LDS feeds six MFMAs), four waves share a 64-row candidate tile (hi and lo) in LDS,
// double buffered.
__device__ __forceinline__ uint16_t bf16_rne(float v)
{
    const uint32_t b = __float_as_uint(v);
    return (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

template <typename T>
__global__ __launch_bounds__(128) void colsum_kernel(const T* __restrict__ x, int64_t n, int d, double* __restrict__ sums)
{
    const int64_t r0 = (int64_t)blockIdx.x * 512;
    for (int c = (int)threadIdx.x; c < d; c += 128) {
        double acc = 0.0;
        for (int64_t r = r0; r < min(n, r0 + 512); ++r) acc += (double)(float)x[r * d + c];
        atomicAdd(&sums[c], acc);
    }
}
__global__ void mean_kernel(const double* sums, int d, int64_t n, float* mean)
{
    const int c = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (c < d) mean[c] = (float)(sums[c] / (double)n);
}

constexpr int kPrepRowsPerWave = 16;   // rows a wave of the two centring kernels walks through: one look at the
                                       // shared maximum per wave instead of one per row

// a wave walks through 16 rows: centred hi / lo rows (padded to dp), centred squared norm, max norm
template <typename T>
__global__ __launch_bounds__(256) void split_prep_kernel(const T* __restrict__ x, int64_t n, int d, int dp,
                                                         const float* __restrict__ mean, uint16_t* __restrict__ xh,
                                                         uint16_t* __restrict__ xl, float* __restrict__ norms,
                                                         unsigned* maxnorm)
{
    const int64_t row0 = (linear_block() * 4 + (threadIdx.x >> 6)) * kPrepRowsPerWave;
    const int lane = lane_id();
    unsigned wmax = 0u;
    for (int64_t row = row0; row < min(n, row0 + kPrepRowsPerWave); ++row) {
        double acc = 0.0;
        for (int j = lane; j < dp; j += 64) {
            float c = 0.f;
            if (j < d) c = (float)x[row * d + j] - mean[j];
            const uint16_t h = bf16_rne(c);
            const uint16_t l = bf16_rne(c - bf16_to_f32(h));
            xh[row * dp + j] = h;
            xl[row * dp + j] = l;
            acc += (double)c * (double)c;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc += shfl_xor_f64(acc, o);
        const float nf = (float)acc;
        if (lane == 0) norms[row] = nf;
        wmax = max(wmax, __float_as_uint(nf));
    }
    if (lane == 0 && wmax > *maxnorm) atomicMax(maxnorm, wmax);
}

// a wave walks through 16 rows: centred rows as ONE binary16 part, scaled by a power of two (scale) that puts the
// largest element near 2^14, well inside binary16's range; centred squared norm (unscaled), max norm
template <typename T>
__global__ __launch_bounds__(256) void half_prep_kernel(const T* __restrict__ x, int64_t n, int d, int dp,
                                                        const float* __restrict__ mean, float scale,
                                                        uint16_t* __restrict__ xh, float* __restrict__ norms,
                                                        unsigned* maxnorm)
{
    const int64_t row0 = (linear_block() * 4 + (threadIdx.x >> 6)) * kPrepRowsPerWave;
    const int lane = lane_id();
    unsigned wmax = 0u;
    for (int64_t row = row0; row < min(n, row0 + kPrepRowsPerWave); ++row) {
        double acc = 0.0;
        for (int j = lane; j < dp; j += 64) {
            float c = 0.f;
            if (j < d) c = (float)x[row * d + j] - mean[j];
            const _Float16 h = (_Float16)(c * scale);   // round to nearest even
            xh[row * dp + j] = __builtin_bit_cast(uint16_t, h);
            acc += (double)c * (double)c;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc += shfl_xor_f64(acc, o);
        const float nf = (float)acc;
        if (lane == 0) norms[row] = nf;
        wmax = max(wmax, __float_as_uint(nf));   // norms are not negative: their bit patterns order like the values
    }
    if (lane == 0 && wmax > *maxnorm) atomicMax(maxnorm, wmax);
}

// rows of integers in [0,255], centred (x - 128, exact in bf16) and zero-padded to dp elements, with
// |x - 128|^2 as an int; 8 lanes per row
template <typename T>
__global__ __launch_bounds__(256) void bf16_rows_kernel(const T* __restrict__ x, int64_t n, int d, int dp,
                                                        uint16_t* __restrict__ xb, int* __restrict__ norms)
{
    const int64_t row = linear_block() * 32 + (threadIdx.x >> 3);
    int acc = 0;
    if (row < n)
        for (int j = (int)(threadIdx.x & 7); j < dp; j += 8) {
            const int c = j < d ? (int)x[row * d + j] - 128 : 0;
            acc += c * c;
            xb[row * dp + j] = (uint16_t)(__float_as_uint((float)c) >> 16);
        }
#pragma unroll
    for (int o = 4; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (row < n && (threadIdx.x & 7) == 0) norms[row] = acc;
}

// two packed bf16 values, each multiplied by -2 (exact; zero stays zero)
__device__ __forceinline__ uint32_t bf16x2_times_minus2(uint32_t w)
{
    const float lo = -2.f * __uint_as_float(w << 16);
    const float hi = -2.f * __uint_as_float(w & 0xFFFF0000u);
    return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xFFFF0000u);
}

struct SplitArgs {
    const uint16_t* qh;   // [nq, DP] hi / lo parts of the centred query rows
    const uint16_t* ql;
    const uint16_t* xh;   // [N, DP] hi / lo parts of the centred base rows
    const uint16_t* xl;
    const float* qnorm;   // centred norms
    const float* xnorm;
    const float* tau;
    unsigned* cnt;
    uint64_t* buf;
    int64_t nq;
    int64_t c_begin, c_end;
    int64_t self_offset;
    int cap, tiles_per_block;
    float scale2, inv_scale2;   // square of the rows' scale and its inverse (powers of two; 1 for the hi + lo rows)
};

constexpr int kSplitQueue = 512;
constexpr int split_tile_rows(int ks, bool single) { return single && ks >= 7 ? 2 * kSplitRows : kSplitRows; }
constexpr int kSplitQB = 2;   // blocks of 32 queries per wave

// SINGLE: the rows are one binary16 part (half_prep_kernel) instead of bf16 hi + lo: one MFMA per k-step
// instead of three, |error of q.x| <= (2^-10 + d*2^-24) sum|q_j||x_j| instead of 3*2^-16: a wider margin in
// the acceptance test of the re-scoring pass, the same answer.  Norms and thresholds stay in the rows'
// own units in memory and are multiplied by scale2 where they meet the accumulators.
template <int KS, bool SINGLE>
__global__ __launch_bounds__(256, (SINGLE && KS <= 6) ? 3 : 2) void filter_split_kernel(SplitArgs a)
{
    constexpr int QB = kSplitQB;
    constexpr int PARTS = SINGLE ? 1 : 2;
    // candidate rows per LDS tile (64-row halves per barrier).  One part, measured at N = 10^6: up to 96 elements
    // three waves per SIMD on 64-row tiles win (0.246 s against 0.261 s at d = 96); beyond, three waves spill
    // and two waves on 128-row tiles win (0.311 s against 0.351 s at d = 128).
    constexpr int ROWS = split_tile_rows(KS, SINGLE);
    using frag_t = std::conditional_t<SINGLE, half8, bf16x8>;
    constexpr int DP = KS * 16;
    constexpr int XS = DP + 8;
    constexpr int CHUNKS = ROWS * DP / 8;       // 16-byte chunks per part of a tile
    constexpr int PER_THREAD = (CHUNKS + 255) / 256;
    __shared__ __attribute__((aligned(16))) uint16_t Xs[2][PARTS][ROWS * XS];   // [buffer][hi|lo]
    __shared__ __attribute__((aligned(16))) float xn[2][ROWS];
    __shared__ SurvivorQueue<kSplitQueue> queue;

    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    if (threadIdx.x == 0) queue.count = 0u;

    // QB blocks of 32 queries per wave
    frag_t qfh[QB][KS], qfl[SINGLE ? 1 : QB][SINGLE ? 1 : KS];
    int64_t qg[QB];
    float qn[QB], tq[QB];   // in the accumulators' units (times scale2)
#pragma unroll
    for (int j = 0; j < QB; ++j) {
        qg[j] = (int64_t)blockIdx.x * (128 * QB) + wave * (32 * QB) + j * 32 + (lane & 31);
        const bool qok = qg[j] < a.nq;
        qn[j] = qok ? a.qnorm[qg[j]] * a.scale2 : 0.f;
        tq[j] = qok ? a.tau[qg[j]] * a.scale2 - qn[j] : -kInf;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint4 wh = make_uint4(0u, 0u, 0u, 0u), wl = wh;
            if (qok) {
                wh = *reinterpret_cast<const uint4*>(a.qh + qg[j] * DP + ks * 16 + 8 * (lane >> 5));
                if constexpr (!SINGLE) wl = *reinterpret_cast<const uint4*>(a.ql + qg[j] * DP + ks * 16 + 8 * (lane >> 5));
            }
            // the query enters as -2q (exact: the scale keeps 2|q_j| inside binary16's range), so that with
            // |x|^2 as the accumulators' start value the contraction itself yields |x|^2 - 2 q.x
            if constexpr (SINGLE) {
                qfh[j][ks] = __builtin_bit_cast(half8, wh) * (_Float16)-2;
            } else {
                wh.x = bf16x2_times_minus2(wh.x); wh.y = bf16x2_times_minus2(wh.y);
                wh.z = bf16x2_times_minus2(wh.z); wh.w = bf16x2_times_minus2(wh.w);
                wl.x = bf16x2_times_minus2(wl.x); wl.y = bf16x2_times_minus2(wl.y);
                wl.z = bf16x2_times_minus2(wl.z); wl.w = bf16x2_times_minus2(wl.w);
                qfh[j][ks] = __builtin_bit_cast(bf16x8, wh);
                qfl[j][ks] = __builtin_bit_cast(bf16x8, wl);
            }
        }
    }

    const int64_t span0 = a.c_begin + (int64_t)blockIdx.y * a.tiles_per_block * ROWS;
    const int64_t span1 = min(a.c_end, span0 + (int64_t)a.tiles_per_block * ROWS);
    if (span0 >= span1) return;
    const int ntiles = (int)((span1 - span0 + ROWS - 1) / ROWS);

    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // a plain vector: stays in registers
    u32x4 stage[PARTS][PER_THREAD];
    float stage_n = 0.f;
    // A tile part is one contiguous block of ROWS * DP elements; a chunk index past the span's
    // end is clamped to the span's last chunk (rows read twice that way carry ids >= span1 and are
    // dropped by the filter), so the loads need no branch.
    const int last_chunk = (int)(span1 - span0) * (DP / 8) - 1;
    const int last_row = (int)(span1 - span0) - 1;
    const uint16_t* xh_span = a.xh + span0 * DP;
    const uint16_t* xl_span = SINGLE ? nullptr : a.xl + span0 * DP;
    auto fetch = [&](int t) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int ch = min((int)threadIdx.x + i * 256, CHUNKS - 1);
            const int64_t off = (int64_t)min(t * CHUNKS + ch, last_chunk) * 8;
            stage[0][i] = *reinterpret_cast<const u32x4*>(xh_span + off);
            if constexpr (!SINGLE) stage[PARTS - 1][i] = *reinterpret_cast<const u32x4*>(xl_span + off);
        }
        if (threadIdx.x < ROWS)
            stage_n = a.xnorm[span0 + min(t * ROWS + (int)threadIdx.x, last_row)] * a.scale2;
    };
    auto commit = [&](int b) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int ch = (int)threadIdx.x + i * 256;
            const int r = ch / (DP / 8), c8 = ch % (DP / 8);
            if (ch < CHUNKS) {
                *reinterpret_cast<u32x4*>(&Xs[b][0][r * XS + c8 * 8]) = stage[0][i];
                if constexpr (!SINGLE) *reinterpret_cast<u32x4*>(&Xs[b][PARTS - 1][r * XS + c8 * 8]) = stage[PARTS - 1][i];
            }
        }
        if (threadIdx.x < ROWS) xn[b][threadIdx.x] = stage_n;
    };

    fetch(0);
    commit(0);
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const int cur = t & 1;
        fetch(t + 1);  // clamped: past the last tile it re-reads the span's end, unused
        for (int h = 0; h < ROWS / 64; ++h) {
        // the accumulators start at |x|^2 of their rows (lane l, register r: row 8*(r/4) + 4*(l/32) + r%4)
        floatx16 acc[2][QB];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const float4 v = *reinterpret_cast<const float4*>(&xn[cur][h * 64 + i * 32 + 8 * r4 + 4 * (lane >> 5)]);
#pragma unroll
                for (int j = 0; j < QB; ++j) {
                    acc[i][j][4 * r4 + 0] = v.x; acc[i][j][4 * r4 + 1] = v.y;
                    acc[i][j][4 * r4 + 2] = v.z; acc[i][j][4 * r4 + 3] = v.w;
                }
            }
        }
        // The half's 2 * KS fragment reads (step s: k-step s / 2, candidate block s % 2) run AHEAD steps before the
        // MFMAs that use them, in a ring of AHEAD register sets, the order pinned: left to itself the compiler keeps
        // one set and waits for every read right after issuing it.  (Two sets: 2 % faster at d = 64..128; three
        // sets spill under the three-waves-per-SIMD register limit and lose it again.)
        constexpr int AHEAD = 2, STEPS = 2 * KS;
        frag_t fh[AHEAD], fl[SINGLE ? 1 : AHEAD];
        auto read_step = [&](int st) __attribute__((always_inline)) {
            const int ks = st >> 1, i = st & 1;
            const int off = (h * 64 + i * 32 + (lane & 31)) * XS + ks * 16 + 8 * (lane >> 5);
            fh[st % AHEAD] = *reinterpret_cast<const frag_t*>(&Xs[cur][0][off]);
            if constexpr (!SINGLE) fl[st % AHEAD] = *reinterpret_cast<const frag_t*>(&Xs[cur][PARTS - 1][off]);
        };
#pragma unroll
        for (int st = 0; st < AHEAD && st < STEPS; ++st) read_step(st);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            const int ks = st >> 1, i = st & 1;
            const frag_t xh = fh[st % AHEAD];
            if constexpr (SINGLE) {
#pragma unroll
                for (int j = 0; j < QB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xh, qfh[j][ks], acc[i][j], 0, 0, 0);
            } else {
                const frag_t xl = fl[st % AHEAD];
#pragma unroll
                for (int j = 0; j < QB; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl, qfh[j][ks], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh, qfl[j][ks], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh, qfh[j][ks], acc[i][j], 0, 0, 0);
                }
            }
            if (st + AHEAD < STEPS) read_step(st + AHEAD);
            __builtin_amdgcn_sched_barrier(0);
        }
        const int64_t c0 = span0 + (int64_t)t * ROWS + h * 64;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int j = 0; j < QB; ++j) {
                float lo = __builtin_fminf(acc[i][j][0], acc[i][j][1]);
#pragma unroll
                for (int r = 2; r < 16; r += 2) lo = __builtin_fminf(__builtin_fminf(lo, acc[i][j][r]), acc[i][j][r + 1]);
                if (ballot64(lo < tq[j])) {
                    uint32_t mask = 0;
#pragma unroll
                    for (int r = 0; r < 16; ++r) mask |= (acc[i][j][r] < tq[j]) ? (1u << r) : 0u;
#pragma unroll 1
                    while (ballot64(mask != 0u)) {
                        const int rr = mask ? (int)__builtin_ctz(mask) : 16;
                        mask &= mask - 1u;
                        float u = 0.f;
#pragma unroll
                        for (int r = 0; r < 16; ++r) u = rr == r ? acc[i][j][r] : u;
                        const int m = i * 32 + 8 * (rr >> 2) + 4 * (lane >> 5) + (rr & 3);
                        const int64_t c = c0 + m;
                        if (rr < 16 && c < span1 && c != a.self_offset + qg[j]) {
                            const uint64_t key =
                                ((uint64_t)__float_as_uint(fmaxf(u + qn[j], 0.f) * a.inv_scale2) << 32) | (uint64_t)(uint32_t)c;
                            queue.push(key, wave * (32 * QB) + j * 32 + (lane & 31), qg[j], a.cnt, a.buf, a.cap);
                        }
                    }
                }
            }
        }
        }
        if (t + 1 < ntiles) commit(cur ^ 1);
        __syncthreads();
        queue.flush((int64_t)blockIdx.x * (128 * QB), a.cnt, a.buf, a.cap, t + 1 == ntiles);
    }
}

// ---------------------------------------------------------------- rows wider than 128 elements
// The same contraction when a query's fragments no longer fit the registers (MODE 1: hi + lo parts; MODE 2:
// one scaled binary16 part; MODE 0: integer rows, which are exact in bf16, one part, one MFMA per k-step): both
// operands go through LDS in slabs of the k dimension, two buffers, the LDS-direct loads of slab g+1 on
// their way during the MFMAs of slab g (one barrier per slab).  The filter runs once per tile, after the last
// slab, so it is amortised over d / 16 k-steps and needs none of the tricks of the register kernels:
// u = |x|^2 - 2 q.x is formed from the finished accumulators.
// Workgroups are numbered so that those resident together form a block of q_group query tiles
// times a few candidate spans: the slabs they stream are then shared through the L2 caches
// instead of each being fetched from memory once per workgroup.
constexpr int kWidePad = 64;   // rows are padded with zeros to a multiple of this many elements (every slab depth divides it)

struct WideArgs {
    SplitArgs s;
    int dp;            // padded row length (a multiple of the slab depth)
    int q_tiles, ny;   // query tiles; candidate spans of tiles_per_block tiles
    int q_group;       // query tiles per group of the block numbering
};

// The shape of a workgroup.  One part per operand (MODE 0, 2): eight waves, four along the queries and two along
// the candidates, each 64 queries x 128 candidates (8 MFMAs per 6 fragment reads), a 256 x 256 tile, slabs 64 deep
// (64 KB, two buffers, one workgroup per compute unit): a third fewer bytes fetched per MFMA than 128 x 256 and half
// the barriers of slabs 32 deep.  hi + lo parts (MODE 1): four waves of 64 x 64, a 128 x 128 tile, slabs 32 deep.
template <int MODE>
struct WideShape {
    static constexpr int WQ = MODE == 1 ? 2 : 4;         // waves along the queries, 64 rows each
    static constexpr int XB = MODE == 1 ? 2 : 4;         // 32-row candidate blocks per wave
    static constexpr int DK = MODE == 1 ? 32 : 64;       // elements of k per slab
    static constexpr int NBUF = 2;                       // slab buffers
    static constexpr int PARTS = MODE == 1 ? 2 : 1;
    static constexpr int QT = 64 * WQ, XT = 64 * XB;     // rows of the tile: queries, candidates
    static constexpr int THREADS = 128 * WQ;
    static constexpr int SLAB = PARTS * (QT + XT) * DK;  // elements
    static constexpr size_t lds_bytes = (size_t)NBUF * SLAB * sizeof(uint16_t);
};
struct WideLaunch { int qt, xt, threads; size_t lds; };
template <int MODE> constexpr WideLaunch wide_launch_of() { using S = WideShape<MODE>; return {S::QT, S::XT, S::THREADS, S::lds_bytes}; }
// candidate rows that one workgroup sweeps
constexpr int wide_span_rows(int mode) { return mode == 1 ? 512 : 2048; }
constexpr WideLaunch wide_launch(int mode) { return mode == 0 ? wide_launch_of<0>() : mode == 1 ? wide_launch_of<1>() : wide_launch_of<2>(); }

// LDS-direct loads: the wave's 64 lanes x 16 (or 4) bytes land contiguously at the LDS address in m0, lane by lane.
// Issued through inline assembly: the compiler would make every later LDS read wait for all of them, which takes
// away the overlap of a slab's loads with the multiplications of the slabs before; the waits are explicit instead.
// The address is a uniform 64-bit base plus a 32-bit unsigned byte offset per lane.  The wait states before the load
// cover m0 and a base that the compiler may have moved into its scalar registers from a vector register just before
// (it does not look into the assembly for what the load needs).
__device__ __forceinline__ uint64_t uniform_address(const void* p)
{
    const uint64_t v = (uint64_t)(uintptr_t)p;   // (the builtin returns a signed int: widened as it is, a low half with
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);   // bit 31 set would flood the high half)
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | (uint64_t)lo;
}
__device__ __forceinline__ void lds_direct_b128(uint32_t lane_offset, const void* base, uint32_t lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %0, %1"
                 ::"v"(lane_offset), "s"(uniform_address(base)), "s"(lds_byte_addr) : "memory", "m0");
}
__device__ __forceinline__ void lds_direct_b32(uint32_t lane_offset, const void* base, uint32_t lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\tglobal_load_lds_dword %0, %1"
                 ::"v"(lane_offset), "s"(uniform_address(base)), "s"(lds_byte_addr) : "memory", "m0");
}
template <typename P> __device__ __forceinline__ uint32_t lds_addr(P* p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(p);
}

// LDS rows are DK elements with no padding; 16-byte chunk c of row r sits at chunk c ^ swizzle(r).  A 16-byte read
// is served 16 lanes (here: 16 consecutive rows, one chunk) per cycle from 64 banks of 4 bytes, so the 16 slots have
// to differ in byte address mod 256: with 64-byte rows four rows already do and the place changes every four rows;
// with 128-byte rows two rows do and the place changes every two.  (Measured: places c ^ (r & 7) on 128-byte rows
// cost one conflict cycle per access cycle; these cost none.)  The period is 16 rows in both.
template <int DK> __device__ __forceinline__ int wide_swizzle(int row) { return DK == 32 ? (row >> 2) & 3 : (row >> 1) & 7; }
template <int DK>
__device__ __forceinline__ int wide_lds_offset(int row, int chunk)
{
    static_assert(DK == 32 || DK == 64, "the swizzles are written for 64- and 128-byte rows");
    return row * DK + ((chunk ^ wide_swizzle<DK>(row)) << 3);
}

// MODE 0: centred integer rows, one bf16 part, exact (filter in int32); 1: real-valued rows as bf16 hi + lo;
// 2: real-valued rows as one scaled binary16 part (see filter_split_kernel's SINGLE).
template <int MODE>
__global__ __launch_bounds__(WideShape<MODE>::THREADS, 2) void filter_wide_kernel(WideArgs w)
{
    using S = WideShape<MODE>;
    constexpr bool LO = MODE == 1;    // lo parts staged and multiplied
    constexpr bool FLT = MODE != 0;   // float arithmetic with a rounding margin downstream
    using frag_t = std::conditional_t<MODE == 2, half8, bf16x8>;
    const SplitArgs& a = w.s;
    constexpr int DK = S::DK;                     // elements of k per slab
    constexpr int XB = S::XB;                     // 32-row candidate blocks per wave
    constexpr int QT = S::QT, XT = S::XT;         // rows of the workgroup's tile
    constexpr int NW = 2 * S::WQ;                 // waves: WQ along the queries x two side by side along the candidates
    constexpr int NBUF = S::NBUF;
    extern __shared__ __attribute__((aligned(16))) uint16_t wide_slabs[];   // [NBUF][q parts: QT * DK | x parts: XT * DK]
    __shared__ __attribute__((aligned(16))) float xn[2][XT];
    __shared__ SurvivorQueue<kSplitQueue> queue;
    constexpr int QPART = QT * DK, XPART = XT * DK;   // elements of one part of a slab, per operand
    constexpr int QPARTS = S::PARTS;
    constexpr int SLAB = S::SLAB;

    // block numbering: groups of q_group query tiles, inside a group the query tile varies fastest
    const int64_t b = linear_block();
    if (b >= (int64_t)w.q_tiles * w.ny) return;
    const int64_t per_group = (int64_t)w.q_group * w.ny;
    const int64_t grp = b / per_group, within = b - grp * per_group;
    const int gq = (int)min((int64_t)w.q_group, (int64_t)w.q_tiles - grp * w.q_group);
    const int64_t q0 = (grp * w.q_group + within % gq) * QT;
    const int64_t y = within / gq;

    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const int wq = wave >> 1, wc = wave & 1;
    if (threadIdx.x == 0) queue.count = 0u;

    // FLT: float arithmetic with a rounding margin downstream.  !FLT: the rows are centred integers, every
    // product and partial sum is an integer below 2^24 in magnitude (d <= 1024), so the accumulators are
    // exact and the norms, thresholds and the filter are taken in int32 (the norm arrays hold ints).
    using V = std::conditional_t<FLT, float, int>;
    int64_t qg[2];
    V qn[2], tq[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        qg[j] = q0 + wq * 64 + j * 32 + (lane & 31);
        const bool ok = qg[j] < a.nq;
        if constexpr (FLT) {   // in the accumulators' units
            qn[j] = ok ? a.qnorm[qg[j]] * a.scale2 : 0.f;
            tq[j] = ok ? a.tau[qg[j]] * a.scale2 - qn[j] : -kInf;
        } else {
            qn[j] = ok ? reinterpret_cast<const int*>(a.qnorm)[qg[j]] : 0;
            const float tf = ok ? a.tau[qg[j]] : -1.f;   // an integer-valued float or +inf
            tq[j] = ok ? (tf < 1.0e9f ? (int)tf - qn[j] : (1 << 30)) : -(1 << 30);
        }
    }

    const int64_t span0 = a.c_begin + y * a.tiles_per_block * XT;
    const int64_t span1 = min(a.c_end, span0 + (int64_t)a.tiles_per_block * XT);
    if (span0 >= span1) return;
    const int ntiles = (int)((span1 - span0 + XT - 1) / XT);
    const int nstage = w.dp / DK;
    const int G = ntiles * nstage;

    // A slab comes in by LDS-direct loads: the 64 lanes of one load fill 1 KB, i.e. GR rows of the slab; lane l fills
    // place l % CPR of row l / CPR of its group and so fetches the chunk that the swizzle keeps there.  No staging
    // registers and no LDS stores, so NBUF - 1 slabs can be on their way while one is multiplied.
    // Addresses are a scalar base (part, tile, slab: all uniform) plus a 32-bit offset per lane that does not change
    // from slab to slab, so that a fetch costs the vector unit nothing but the loads themselves.
    constexpr int CPR = DK / 8, GR = 64 / CPR;               // 16-byte chunks per slab row; rows per load
    constexpr int GQ = QT / GR / NW, GX = XT / GR / NW;      // loads per wave and part: queries, candidates
    static_assert(GQ * GR * NW == QT && GX * GR * NW == XT, "the loads tile the slab");
    static_assert((GR * NW) % 16 == 0, "a wave's groups all start at the same place of the swizzle's 16-row period");
    const int grow = lane / CPR;
    const int gchunk = ((lane % CPR) ^ wide_swizzle<DK>(GR * wave + grow)) << 3;   // element offset inside the slab's DK
    const uint32_t row_bytes = (uint32_t)w.dp * 2u;
    uint32_t qoff[GQ], xoff[GX];   // xoff: for a tile whose XT rows all exist
#pragma unroll
    for (int h = 0; h < GQ; ++h)   // clamped: rows past the end are re-reads whose results are dropped
        qoff[h] = (uint32_t)(min(q0 + GR * (wave + NW * h) + grow, a.nq - 1) - q0) * row_bytes + (uint32_t)gchunk * 2u;
#pragma unroll
    for (int h = 0; h < GX; ++h) xoff[h] = (uint32_t)(GR * (wave + NW * h) + grow) * row_bytes + (uint32_t)gchunk * 2u;
    const int xw = (wave * 64) % XT;   // this wave's share of the tile's norms (shares repeat where the tile has fewer than 256 rows)
    const int last_row = (int)(span1 - span0) - 1;
    const uint32_t slab0 = lds_addr(wide_slabs), xn0 = lds_addr(&xn[0][0]);
    // one slab (and its tile's norms) into buffer buf; every wave waits for its own share with vmcnt(0) before the
    // slab's barrier
    auto fetch = [&](int buf, int t, int sg) __attribute__((always_inline)) {
        const uint32_t base = slab0 + (uint32_t)(buf * SLAB) * 2u;
        const int64_t qfirst = q0 * w.dp + sg * DK, xfirst = (span0 + (int64_t)t * XT) * w.dp + sg * DK;   // elements
        const int lim = last_row - t * XT;   // last row of the tile that exists, counted from the tile's first
#pragma unroll
        for (int h = 0; h < GQ; ++h) {
            const uint32_t at = __builtin_amdgcn_readfirstlane(base + (uint32_t)((wave + NW * h) * GR * DK) * 2u);
            lds_direct_b128(qoff[h], a.qh + qfirst, at);
            if constexpr (LO) lds_direct_b128(qoff[h], a.ql + qfirst, at + (uint32_t)QPART * 2u);
        }
        uint32_t xo[GX], no = (uint32_t)(xw + lane) * 4u;
#pragma unroll
        for (int h = 0; h < GX; ++h) xo[h] = xoff[h];
        if (lim < XT - 1) {   // the span's ragged last tile
#pragma unroll
            for (int h = 0; h < GX; ++h) xo[h] = (uint32_t)min(GR * (wave + NW * h) + grow, lim) * row_bytes + (uint32_t)gchunk * 2u;
            no = (uint32_t)min(xw + lane, lim) * 4u;
        }
#pragma unroll
        for (int h = 0; h < GX; ++h) {
            const uint32_t at = __builtin_amdgcn_readfirstlane(base + (uint32_t)(QPARTS * QPART + (wave + NW * h) * GR * DK) * 2u);
            lds_direct_b128(xo[h], a.xh + xfirst, at);
            if constexpr (LO) lds_direct_b128(xo[h], a.xl + xfirst, at + (uint32_t)XPART * 2u);
        }
        // the tile's norms, again with every slab of it: the same words to the same place
        lds_direct_b32(no, a.xnorm + span0 + (int64_t)t * XT, __builtin_amdgcn_readfirstlane(xn0 + (uint32_t)((t & 1) * XT + xw) * 4u));
    };
    static_assert(NBUF == 2, "the loop below is written for two buffers");
    constexpr int KS = DK / 16;
    static_assert(KS >= 2 && KS % 2 == 0, "query fragments alternate between two register sets, step 0 in set 0");

    // Fragment reads.  The fragments of step k + 1 are asked for while step k multiplies: the queries' into the other
    // of two register sets at the start of the step, each candidate block's in place as soon as its two MFMAs are
    // issued, the order pinned, so that every read has six MFMAs or more between itself and its first use.  (Left to
    // itself the compiler keeps four fragments' worth of registers and waits for most reads right after issuing them.)
    frag_t qh[2][2], ql[2][2], xh[XB], xl[XB];
    auto read_q = [&](const uint16_t* slab, int k16, int b) __attribute__((always_inline)) {
        const int chunk = k16 * 2 + (lane >> 5);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int qo = wide_lds_offset<DK>(wq * 64 + j * 32 + (lane & 31), chunk);
            qh[b][j] = *reinterpret_cast<const frag_t*>(slab + qo);
            if constexpr (LO) ql[b][j] = *reinterpret_cast<const frag_t*>(slab + QPART + qo);
        }
    };
    auto read_x = [&](const uint16_t* slab, int k16, int i) __attribute__((always_inline)) {
        const int chunk = k16 * 2 + (lane >> 5);
        const int xo = wide_lds_offset<DK>(wc * (32 * XB) + i * 32 + (lane & 31), chunk);
        xh[i] = *reinterpret_cast<const frag_t*>(slab + QPARTS * QPART + xo);
        if constexpr (LO) xl[i] = *reinterpret_cast<const frag_t*>(slab + QPARTS * QPART + XPART + xo);
    };
    floatx16 acc[XB][2];
    int t = 0, sg = 0;       // tile and slab being multiplied
    // step k16 of the current slab; `from`, k_next: where the reads issued during it come from.
    // A tile's first step takes zero as its third operand instead of accumulators cleared beforehand.
    auto step = [&](int k16, const uint16_t* from, int k_next, auto fresh) __attribute__((always_inline)) {
        const int b = k16 & 1;
        read_q(from, k_next, b ^ 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < XB; ++i) {
            // Float modes: a tile's accumulators start at -|x|^2 / 2 of their rows (lane l, register r: row
            // 8*(r/4) + 4*(l/32) + r%4 of the block) and end as q.x - |x|^2 / 2 = -u / 2, so the filter is a maximum
            // and one compare per block with no arithmetic on the accumulators; the same sums, scaled by -1/2, as in
            // the register kernel, whose error bound is the one in use.  The integer mode starts at zero (half an odd
            // norm is no integer) and forms u in its filter.
            float start[16];
            if constexpr (decltype(fresh)::value && FLT) {
                const float half = -0.5f * a.scale2;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const float4 v = *reinterpret_cast<const float4*>(&xn[t & 1][wc * (32 * XB) + i * 32 + 8 * r4 + 4 * (lane >> 5)]);
                    start[4 * r4 + 0] = v.x * half; start[4 * r4 + 1] = v.y * half;
                    start[4 * r4 + 2] = v.z * half; start[4 * r4 + 3] = v.w * half;
                }
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                floatx16 c = acc[i][j];
                if constexpr (decltype(fresh)::value) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) c[r] = FLT ? start[r] : 0.f;
                }
                if constexpr (MODE == 2) {
                    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(xh[i], qh[b][j], c, 0, 0, 0);
                } else {
                    if constexpr (LO) {
                        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl[i], qh[b][j], c, 0, 0, 0);
                        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh[i], ql[b][j], c, 0, 0, 0);
                    }
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh[i], qh[b][j], c, 0, 0, 0);
                }
                acc[i][j] = c;
            }
            read_x(from, k_next, i);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto first_fragments = [&](const uint16_t* slab) __attribute__((always_inline)) {
        read_q(slab, 0, 0);
#pragma unroll
        for (int i = 0; i < XB; ++i) read_x(slab, 0, i);
    };

    // The slab's one barrier does not stand at the slab's end but right after its last fragment reads, one step
    // before: by then every wave has everything it needs of the slab in registers (the buffer is free for the slab
    // after next) and has waited for its own loads of the next slab (which is then complete), and the MFMAs of the
    // last step run while the barrier is crossed and the next slab's first fragments are on their way.
    int tn = 0, sn = 0;      // slab fetched last
    fetch(0, 0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
    if (1 < G && ++sn == nstage) { sn = 0; ++tn; }
    fetch(1, tn, sn);        // past the last slab a fetch re-reads it, unused
    first_fragments(wide_slabs);
    for (int g = 0; g < G; ++g) {
        const int cur = g & 1;
        const uint16_t* slab = wide_slabs + cur * SLAB;
        const uint16_t* next = wide_slabs + (cur ^ 1) * SLAB;
        const bool tile_done = sg == nstage - 1, more = g + 1 < G;
        if (sg == 0) step(0, slab, 1, std::true_type{});
        else step(0, slab, 1, std::false_type{});
#pragma unroll
        for (int k16 = 1; k16 + 1 < KS; ++k16) step(k16, slab, k16 + 1, std::false_type{});
        __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0), lgkmcnt(0): the slab's last fragments and this wave's share of the next slab are there
        __syncthreads();
        if (g + 2 < G && ++sn == nstage) { sn = 0; ++tn; }
        fetch(cur, tn, sn);
        step(KS - 1, more ? next : slab, 0, std::false_type{});   // (after the last slab: reads of the same slab again, unused)
        if (tile_done) {
            // lane l, register r of block (i, j): candidate row 8*(r/4) + 4*(l/32) + r%4 of block i, query l%32 of block j
            const int64_t c0 = span0 + (int64_t)t * XT + wc * (32 * XB);
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                V xv[16];
                if constexpr (!FLT) {
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {   // the norms' words, read as the ints they are
                        const float4 v = *reinterpret_cast<const float4*>(&xn[t & 1][wc * (32 * XB) + i * 32 + 8 * r4 + 4 * (lane >> 5)]);
                        xv[4 * r4 + 0] = __float_as_int(v.x); xv[4 * r4 + 1] = __float_as_int(v.y);
                        xv[4 * r4 + 2] = __float_as_int(v.z); xv[4 * r4 + 3] = __float_as_int(v.w);
                    }
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    // u = |x|^2 - 2 q.x against tq.  The float modes hold -u / 2 in the accumulators and test the largest
                    // of them against -tq / 2 (exact scalings); w[] is what the test looks at, `below` says which way.
                    V w[16], lim, ext;
                    if constexpr (FLT) {
                        lim = (V)(-0.5f * (float)tq[j]);
#pragma unroll
                        for (int r = 0; r < 16; ++r) w[r] = acc[i][j][r];
                        ext = __builtin_fmaxf(w[0], w[1]);   // (a maximum that skips values that are no numbers: they pass no test below either)
#pragma unroll
                        for (int r = 2; r < 16; r += 2) ext = __builtin_fmaxf(__builtin_fmaxf(ext, w[r]), w[r + 1]);
                    } else {
                        lim = tq[j];
#pragma unroll
                        for (int r = 0; r < 16; ++r) w[r] = xv[r] - 2 * (int)acc[i][j][r];
                        ext = min(w[0], w[1]);
#pragma unroll
                        for (int r = 2; r < 16; r += 2) ext = min(ext, min(w[r], w[r + 1]));
                    }
                    auto passes = [&](V v) __attribute__((always_inline)) { return FLT ? v > lim : v < lim; };
                    if (ballot64(passes(ext))) {
                        uint32_t mask = 0;
#pragma unroll
                        for (int r = 0; r < 16; ++r) mask |= passes(w[r]) ? (1u << r) : 0u;
#pragma unroll 1
                        while (ballot64(mask != 0u)) {
                            const int rr = mask ? (int)__builtin_ctz(mask) : 16;
                            mask &= mask - 1u;
                            V uv = 0;
#pragma unroll
                            for (int r = 0; r < 16; ++r) uv = rr == r ? w[r] : uv;
                            const int m = i * 32 + 8 * (rr >> 2) + 4 * (lane >> 5) + (rr & 3);
                            const int64_t c = c0 + m;
                            if (rr < 16 && c < span1 && c != a.self_offset + qg[j]) {
                                const float sf = FLT ? fmaxf((float)qn[j] - 2.f * (float)uv, 0.f) * a.inv_scale2 : (float)max((int)(uv + qn[j]), 0);
                                const uint64_t key = ((uint64_t)__float_as_uint(sf) << 32) | (uint64_t)(uint32_t)c;
                                queue.push(key, wq * 64 + j * 32 + (lane & 31), qg[j], a.cnt, a.buf, a.cap);
                            }
                        }
                    }
                }
            }
        }
        if (tile_done) {
            __syncthreads();   // the tile's last push
            queue.template flush<S::THREADS>(q0, a.cnt, a.buf, a.cap, g + 1 == G);
            sg = 0;
            ++t;
        } else {
            ++sg;
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // the unused loads of the last rounds land before the workgroup's LDS is given back
}

// ---------------------------------------------------------------- per-row compaction
// Keeps the kprime entries of the row's buffer with the smallest approximate distances (in any
// order) and sets tau to the kprime-th smallest.  cnt > cap means entries were lost: the row is flagged.
struct CompactArgs {
    unsigned* cnt;
    unsigned* kept;    // entries left by the previous pass
    uint64_t* buf;
    float* tau;
    unsigned* overflow;
    int64_t nq;
    int cap, kprime;
};

// One wavefront cuts a row's unsorted candidate buffer (more than kprime entries, R = capacity / 64 per
// lane, already loaded into e[], unused slots holding the empty key) down to kprime entries with
// the smallest distances and returns
// the kprime-th smallest distance D, the row's new threshold.  D is found by bisection on the
// distance's bit pattern (non-negative floats order like unsigned integers) with wave-wide counts;
// entries below D all stay and of those equal to D as many as still fit (the dropped ones are not
// below the new threshold, which is all the filter's invariant asks for).  No sorting, no LDS.
// The bisection stops early at any value that kprime .. kprime + kCompactSlack entries do not exceed: those all
// stay (`kept` says how many) and that value is the threshold -- a few entries more in the buffer and a threshold a
// few ranks looser, for a handful of bisection steps instead of one per bit of the interval.  Rows with many equal
// distances never meet such a value and end at the exact one.
constexpr int kCompactSlack = 2;   // (1M x 128: 153.5 ms with none, 151.0 with 2, 151.7 with 4, 152.4 with 8: more survivors later)
template <int R>
__device__ __forceinline__ float keep_smallest(uint64_t* __restrict__ g, const uint64_t (&e)[R], int n, int kprime, int lane, int* kept)
{
    uint32_t dist[R];
#pragma unroll
    for (int r = 0; r < R; ++r) dist[r] = (uint32_t)(e[r] >> 32);
    // The kprime-th smallest lies between the smallest and the largest distance present (n >= kprime entries, all
    // finite), which for a row's candidates is a far narrower interval of bit patterns than [0, +inf): fewer
    // bisection steps.  Register slots past the row's n entries (wave-uniform) are skipped in every count.
    uint32_t lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (r * 64 >= n) continue;
        lo = min(lo, dist[r]);
        if (dist[r] != 0xFFFFFFFFu) hi = max(hi, dist[r]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        lo = min(lo, (uint32_t)__shfl_xor((int)lo, o, 64));
        hi = max(hi, (uint32_t)__shfl_xor((int)hi, o, 64));
    }
    while (lo < hi) {   // invariant: count(dist <= hi) >= kprime
        const uint32_t mid = lo + (hi - lo) / 2u;
        int c = 0;
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (r * 64 < n) c += popc64(ballot64(dist[r] <= mid));
        if (c >= kprime) {
            hi = mid;
            if (c <= kprime + kCompactSlack) {   // everything up to mid stays
                // the largest distance that stays is the threshold: a value that occurs (the integer paths take the
                // threshold's integer part) and the tightest that keeps them all
                int base = 0;
                uint32_t top = 0u;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if (r * 64 >= n) continue;
                    const bool keep = dist[r] <= mid;
                    const uint64_t mk = ballot64(keep);
                    if (keep) {
                        g[base + popc64(mk & lanes_below(lane))] = e[r];
                        top = max(top, dist[r]);
                    }
                    base += popc64(mk);
                }
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) top = max(top, (uint32_t)__shfl_xor((int)top, o, 64));
                *kept = c;
                return __uint_as_float(top);
            }
        } else {
            lo = mid + 1u;
        }
    }
    *kept = kprime;
    const uint32_t D = lo;
    int below = 0;
#pragma unroll
    for (int r = 0; r < R; ++r)
        if (r * 64 < n) below += popc64(ballot64(dist[r] < D));
    const int need = kprime - below;  // >= 1 entries equal to D are kept
    int base = 0, ties = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (r * 64 >= n) continue;
        const bool lt = dist[r] < D, eq = dist[r] == D;
        const uint64_t meq = ballot64(eq);
        const bool keep = lt || (eq && ties + popc64(meq & lanes_below(lane)) < need);
        const uint64_t mk = ballot64(keep);
        if (keep) g[base + popc64(mk & lanes_below(lane))] = e[r];
        base += popc64(mk);
        ties += popc64(meq);
    }
    return __uint_as_float(D);
}

template <int R>
__global__ __launch_bounds__(256) void compact_kernel(CompactArgs a)
{
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // one wavefront per row
    if (row >= a.nq) return;
    const int lane = lane_id();
    unsigned n = a.cnt[row];
    if (n > (unsigned)a.cap) {
        if (lane == 0) a.overflow[row] = 1u;
        n = (unsigned)a.cap;
    }
    if (n == a.kept[row]) return;  // nothing new since the last pass
    uint64_t* g = a.buf + row * a.cap;
    if ((int)n <= a.kprime) {      // not yet full: everything stays, no threshold
        if (lane == 0) a.kept[row] = n;
        return;
    }
    uint64_t e[R];
#pragma unroll
    for (int r = 0; r < R; ++r) e[r] = lane + 64 * r < (int)n ? g[lane + 64 * r] : kKeyEmpty;
    int kept;
    const float D = keep_smallest<R>(g, e, (int)n, a.kprime, lane, &kept);
    if (lane == 0) {
        a.cnt[row] = (unsigned)kept;
        a.kept[row] = (unsigned)kept;
        a.tau[row] = D;
    }
}

// ---------------------------------------------------------------- re-scoring (B1r)
struct RefineArgs {
    const void* q;
    const void* x;
    const float* qnorm;
    const unsigned* cnt;
    const uint64_t* buf;
    const float* tau;
    const unsigned* overflow;
    int32_t* out_ids;     // [nq_total, k], row offset applied by the caller
    float* out_s;
    unsigned* redo_cnt;
    int32_t* redo_rows;   // local row indices that need the plain scan
    int64_t nq;
    int d, cap, k;
    float err_scale;      // rounding-error bound of the expansion = err_scale * (|q|^2 + max|x|^2) + err_const
    float err_const;
    float xnorm_max;
    int q_is_base;        // query rows are of the base type
};

// One wavefront per query row: canonical distances of the kept candidates, merged 64 at a
// time into a sorted list of k, then the acceptance test.
template <typename TQ, typename TB, int G, int C>
__global__ __launch_bounds__(64) void refine_kernel(RefineArgs a)
{
    using RD = RowDist<TB, G, C>;
    using chunk_t = typename RD::chunk_t;
    constexpr int VP = RD::VP;
    extern __shared__ uint64_t smem[];
    const int Lp = (a.k + 63) & ~63;
    uint64_t* list = smem;       // [Lp]
    uint64_t* ckey = list + Lp;  // [64]
    const int64_t row = blockIdx.x;
    const int lane = lane_id();
    const TB* __restrict__ X = static_cast<const TB*>(a.x);

    for (int i = lane; i < Lp; i += 64) list[i] = kKeyEmpty;
    RD rd;
    rd.init(a.d, lane);
    if constexpr (sizeof(TQ) == sizeof(TB)) {
        if (a.q_is_base) rd.load_query_row(static_cast<const TB*>(a.q), (uint32_t)row);
        else rd.load_query_f32(reinterpret_cast<const float*>(a.q) + row * a.d);
    } else {
        rd.load_query_f32(static_cast<const float*>(a.q) + row * a.d);
    }
    __syncthreads();

    const int n = (int)min(a.cnt[row], (unsigned)a.cap);
    const uint64_t* g = a.buf + row * a.cap;
    auto sync = [] { __syncthreads(); };
    for (int b0 = 0; b0 < n; b0 += 64) {
        const int m = min(64, n - b0);
        for (int p0 = 0; p0 < m; p0 += VP) {
            const int c = p0 + rd.v;
            const bool ok = c < m;
            const uint32_t e = ok ? (uint32_t)(g[b0 + c] & 0xFFFFFFFFull) : 0u;
            chunk_t buf[C];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) {
                buf[cc] = chunk_t{};
                if (ok && rd.has(cc)) buf[cc] = rd.load(X, e, cc);
            }
            const float tot = rd.distance(buf);
            if (ok && rd.g == 0) ckey[c] = make_key(tot, e);
        }
        __syncthreads();
        const uint64_t key = lane < m ? ckey[lane] : kKeyEmpty;
        list_merge(list, a.k, key, lane, sync);
        __syncthreads();
    }

    // acceptance: the k-th canonical distance must lie below tau - error bound
    const uint64_t kth = list[a.k - 1];
    const float tau = a.tau[row];
    const float err = a.err_scale * (a.qnorm[row] + a.xnorm_max) + a.err_const;
    bool accept = !a.overflow[row];
    if (tau != kInf) accept = accept && kth != kKeyEmpty && key_dist(kth) < tau - err;
    if (!accept && lane == 0) a.redo_rows[atomicAdd(a.redo_cnt, 1u)] = (int32_t)row;
    for (int t = lane; t < a.k; t += 64) {
        const uint64_t key = list[t];
        a.out_ids[row * a.k + t] = key != kKeyEmpty ? (int32_t)key_id(key) : -1;
        a.out_s[row * a.k + t] = key != kKeyEmpty ? key_dist(key) : kInf;
    }
}

// ---------------------------------------------------------------- plain scan for rejected rows
template <typename TQ, typename TB, int G, int C>
__global__ __launch_bounds__(64) void scan_kernel(RefineArgs a, int64_t N, int64_t self_offset)
{
    using RD = RowDist<TB, G, C>;
    using chunk_t = typename RD::chunk_t;
    constexpr int VP = RD::VP;
    constexpr int U = (C >= 3) ? 2 : 4;
    extern __shared__ uint64_t smem[];
    const int Lp = (a.k + 63) & ~63;
    uint64_t* list = smem;
    uint64_t* ckey = list + Lp;
    const int64_t row = a.redo_rows[blockIdx.x];
    const int lane = lane_id();
    const TB* __restrict__ X = static_cast<const TB*>(a.x);
    for (int i = lane; i < Lp; i += 64) list[i] = kKeyEmpty;
    RD rd;
    rd.init(a.d, lane);
    if constexpr (sizeof(TQ) == sizeof(TB)) {
        if (a.q_is_base) rd.load_query_row(static_cast<const TB*>(a.q), (uint32_t)row);
        else rd.load_query_f32(reinterpret_cast<const float*>(a.q) + row * a.d);
    } else {
        rd.load_query_f32(static_cast<const float*>(a.q) + row * a.d);
    }
    __syncthreads();
    auto sync = [] { __syncthreads(); };
    const int64_t self = self_offset >= 0 ? self_offset + row : -1;
    for (int64_t b0 = 0; b0 < N; b0 += 64) {
        const int m = (int)min((int64_t)64, N - b0);
        for (int p0 = 0; p0 < m; p0 += U * VP) {
            chunk_t buf[U][C];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = p0 + u * VP + rd.v;
                ok[u] = c < m;
#pragma unroll
                for (int cc = 0; cc < C; ++cc) {
                    buf[u][cc] = chunk_t{};
                    if (ok[u] && rd.has(cc)) buf[u][cc] = rd.load(X, (uint32_t)(b0 + c), cc);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = p0 + u * VP + rd.v;
                const float tot = rd.distance(buf[u]);
                if (ok[u] && rd.g == 0)
                    ckey[c] = (b0 + c == self) ? kKeyEmpty : make_key(tot, (uint32_t)(b0 + c));
            }
        }
        __syncthreads();
        const uint64_t key = lane < m ? ckey[lane] : kKeyEmpty;
        list_merge(list, a.k, key, lane, sync);
        __syncthreads();
    }
    for (int t = lane; t < a.k; t += 64) {
        const uint64_t key = list[t];
        a.out_ids[row * a.k + t] = key != kKeyEmpty ? (int32_t)key_id(key) : -1;
        a.out_s[row * a.k + t] = key != kKeyEmpty ? key_dist(key) : kInf;
    }
}

__global__ void fill_f32(float* p, int64_t n, float v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// ---------------------------------------------------------------- host driver
namespace {

struct DevBuf {
    void* p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 16); }
    template <typename T> T* as() { return static_cast<T*>(p); }
};

template <typename TQ, typename TB> struct RefineLaunch {
    RefineArgs a;
    int64_t N, self_offset;
    unsigned redo;
    hipStream_t stream;
    bool scan;
    template <typename T, int G, int C> void operator()()
    {
        const int Lp = (a.k + 63) & ~63;
        const size_t lds = (size_t)Lp * 8 + 64 * 8;
        if (!scan)
            TSDG_LAUNCH((refine_kernel<TQ, TB, G, C>), dim3((unsigned)a.nq), dim3(64), lds, stream, a);
        else
            TSDG_LAUNCH((scan_kernel<TQ, TB, G, C>), dim3(redo), dim3(64), lds, stream, a, N, self_offset);
    }
};

template <typename TQ, typename TB>
ann_status knn_typed(const TB* base, int64_t N, int d, ann_dtype dtype, const TQ* queries, int64_t nq, int k,
                     bool self, hipStream_t stream, int32_t* out_ids, float* out_s, bool allow_single, bool* retry,
                     const BuildCtx& ctx)
{
    *retry = false;   // set when the one-part filter left too many rows to the plain scan: run again without it
    int kprime = std::min(2 * k, k + 64);
    int cap = kprime + 192 <= 256 ? 256 : 512;
    // query rows per sweep (bounds the candidate buffers: 4-8 GB at the default)
    const int64_t row_block = ctx.knn_row_block > 0 ? ctx.knn_row_block : 1ll << 21;
    unsigned plain_scan_rows = 0;

    DevBuf xnorm, qnorm, info, tau, cnt, kept, ovf, buf, redo_cnt, redo_rows;
    TSDG_HIP(xnorm.alloc((size_t)N * 4));
    TSDG_HIP(info.alloc(4 * sizeof(unsigned)));
    TSDG_HIP(hipMemsetAsync(info.p, 0, 4 * sizeof(unsigned), stream));
    TSDG_LAUNCH((norms_kernel<TB>), folded_grid((N + 32 * kNormPasses - 1) / (32 * kNormPasses)), dim3(256), 0, stream, base, N, d,
                       xnorm.as<float>(), info.as<unsigned>());
    TSDG_HIP(launch_error());
    float* qn = xnorm.as<float>();
    if (!self) {
        TSDG_HIP(qnorm.alloc((size_t)nq * 4));
        TSDG_LAUNCH((norms_kernel<TQ>), folded_grid((nq + 32 * kNormPasses - 1) / (32 * kNormPasses)), dim3(256), 0, stream, queries, nq, d,
                           qnorm.as<float>(), info.as<unsigned>() + 2);
        TSDG_HIP(launch_error());
        qn = qnorm.as<float>();
    }
    unsigned h_info[4];
    TSDG_HIP(hipMemcpyAsync(h_info, info.p, sizeof(h_info), hipMemcpyDeviceToHost, stream));
    TSDG_HIP(hipStreamSynchronize(stream));
    const bool integer_data = h_info[0] == 0 && (self || h_info[2] == 0);
    float xnorm_max, qnorm_max;
    std::memcpy(&xnorm_max, &h_info[1], 4);
    std::memcpy(&qnorm_max, &h_info[self ? 1 : 3], 4);
    // Integer rows are centred to x - 128; their products and partial sums are then integers of at most
    // d * 2^14 in magnitude: exact in int32 (int8 path) and, up to d = 1024, in the fp32 accumulators
    // of the bf16 path as well.  Wider integer rows are treated like real-valued ones.
    const bool exact = integer_data && d <= 1024;
    const float err_scale = 0.f;  // of the exact paths; the split paths carry split_err
    // With an exact filter the threshold needs no margin for rounding, only for ties: a row is
    // accepted when its k-th distance lies strictly below the kprime-th, so a few extra entries
    // suffice, and every chunk then passes about kprime survivors per row instead of 2k.
    if (exact) kprime = std::min(kprime, k + std::max(8, k / 4));

    // int8 fast path: integer rows with d <= 128 are rewritten once as centred, padded int8
    const bool fast = exact && d <= 128;
    // real-valued rows are centred; up to d = 128 the query fragments stay in registers (k-steps of 16),
    // wider rows are staged through LDS in slabs
    const bool split = !exact;
    const bool wide = split && d > 128;
    // Real-valued rows go through the filter as ONE binary16 part, scaled by a power of
    // two that puts the largest centred element (at most sqrt(max|q|^2) + sqrt(max|x|^2), the mean included)
    // at or below 2^14: a third of the MFMAs of the hi + lo form for a wider, still rigorous, margin.
    bool single = split && allow_single && std::isfinite(xnorm_max) && std::isfinite(qnorm_max);
    float scale = 1.f;
    if (single) {
        const double bound = std::sqrt((double)std::max(xnorm_max, qnorm_max)) + std::sqrt((double)xnorm_max);
        int e = bound > 0.0 ? (int)std::floor(std::log2(16384.0 / bound)) : 0;
        e = std::max(-60, std::min(60, e));
        if (bound * std::ldexp(1.0, e) > 16384.0) single = false;   // rows too large even at the smallest scale
        else scale = std::ldexp(1.f, e);
    }
    const float scale2 = scale * scale;
    const int wdk = kWidePad;   // the staged kernel's rows: whole slabs
    const int ks = (d + 15) / 16;
    const int dp = wide ? (d + wdk - 1) / wdk * wdk : ks * 16;

    const int ks8 = (d + 31) / 32, dp8 = ks8 * 32;
    DevBuf xc8, qc8, xn8, qn8;
    if (fast) {
        TSDG_HIP(xc8.alloc((size_t)N * dp8));
        TSDG_HIP(xn8.alloc((size_t)N * 4));
        TSDG_LAUNCH((i8_prep_kernel<TB>), folded_grid((N + 31) / 32), dim3(256), 0, stream, base, N, d, dp8,
                           xc8.as<uint8_t>(), xn8.as<int>(), static_cast<unsigned*>(nullptr));
        if (!self) {
            TSDG_HIP(qc8.alloc((size_t)nq * dp8));
            TSDG_HIP(qn8.alloc((size_t)nq * 4));
            TSDG_LAUNCH((i8_prep_kernel<TQ>), folded_grid((nq + 31) / 32), dim3(256), 0, stream, queries, nq, d,
                               dp8, qc8.as<uint8_t>(), qn8.as<int>(), static_cast<unsigned*>(nullptr));
        }
        TSDG_HIP(launch_error());
    }

    // integer rows of 129..1024 elements: centred, exact in bf16, so the staged kernel runs on one part
    // per row (one MFMA per k-step) and filters in int32
    const bool iwide = exact && !fast;
    const int dpi = (d + kWidePad - 1) / kWidePad * kWidePad;
    DevBuf xb16, qb16, xn16, qn16;
    if (iwide) {
        TSDG_HIP(xb16.alloc((size_t)N * dpi * 2));
        TSDG_HIP(xn16.alloc((size_t)N * 4));
        TSDG_LAUNCH((bf16_rows_kernel<TB>), folded_grid((N + 31) / 32), dim3(256), 0, stream, base, N, d, dpi,
                           xb16.as<uint16_t>(), xn16.as<int>());
        if (!self) {
            TSDG_HIP(qb16.alloc((size_t)nq * dpi * 2));
            TSDG_HIP(qn16.alloc((size_t)nq * 4));
            TSDG_LAUNCH((bf16_rows_kernel<TQ>), folded_grid((nq + 31) / 32), dim3(256), 0, stream, queries, nq, d,
                               dpi, qb16.as<uint16_t>(), qn16.as<int>());
        }
        TSDG_HIP(launch_error());
    }

    DevBuf xh, xl, qh, ql, csum, cmean, cxnorm, cqnorm, cinfo;
    float split_xmax = 0.f;
    if (split) {
        TSDG_HIP(csum.alloc((size_t)d * 8));
        TSDG_HIP(cmean.alloc((size_t)d * 4));
        TSDG_HIP(cinfo.alloc(4));
        TSDG_HIP(xh.alloc((size_t)N * dp * 2));
        if (!single) TSDG_HIP(xl.alloc((size_t)N * dp * 2));
        TSDG_HIP(cxnorm.alloc((size_t)N * 4));
        TSDG_HIP(hipMemsetAsync(csum.p, 0, (size_t)d * 8, stream));
        TSDG_HIP(hipMemsetAsync(cinfo.p, 0, 4, stream));
        TSDG_LAUNCH((colsum_kernel<TB>), dim3((unsigned)((N + 511) / 512)), dim3(128), 0, stream, base, N, d,
                           csum.as<double>());
        TSDG_LAUNCH(mean_kernel, dim3((unsigned)((d + 63) / 64)), dim3(64), 0, stream, csum.as<double>(), d, N,
                           cmean.as<float>());
        if (single)
            TSDG_LAUNCH((half_prep_kernel<TB>), folded_grid((N + 4 * kPrepRowsPerWave - 1) / (4 * kPrepRowsPerWave)), dim3(256), 0, stream, base, N, d, dp,
                               cmean.as<float>(), scale, xh.as<uint16_t>(), cxnorm.as<float>(), cinfo.as<unsigned>());
        else
            TSDG_LAUNCH((split_prep_kernel<TB>), folded_grid((N + 4 * kPrepRowsPerWave - 1) / (4 * kPrepRowsPerWave)), dim3(256), 0, stream, base, N, d, dp,
                               cmean.as<float>(), xh.as<uint16_t>(), xl.as<uint16_t>(), cxnorm.as<float>(),
                               cinfo.as<unsigned>());
        unsigned h_max = 0;
        TSDG_HIP(hipMemcpyAsync(&h_max, cinfo.p, 4, hipMemcpyDeviceToHost, stream));
        if (!self) {
            TSDG_HIP(qh.alloc((size_t)nq * dp * 2));
            if (!single) TSDG_HIP(ql.alloc((size_t)nq * dp * 2));
            TSDG_HIP(cqnorm.alloc((size_t)nq * 4));
            if (single)
                TSDG_LAUNCH((half_prep_kernel<TQ>), folded_grid((nq + 4 * kPrepRowsPerWave - 1) / (4 * kPrepRowsPerWave)), dim3(256), 0, stream, queries, nq,
                                   d, dp, cmean.as<float>(), scale, qh.as<uint16_t>(), cqnorm.as<float>(),
                                   cinfo.as<unsigned>() /* max over queries is not needed; harmless */);
            else
                TSDG_LAUNCH((split_prep_kernel<TQ>), folded_grid((nq + 4 * kPrepRowsPerWave - 1) / (4 * kPrepRowsPerWave)), dim3(256), 0, stream, queries, nq,
                                   d, dp, cmean.as<float>(), qh.as<uint16_t>(), ql.as<uint16_t>(), cqnorm.as<float>(),
                                   cinfo.as<unsigned>() /* max over queries is not needed; harmless */);
        }
        TSDG_HIP(launch_error());
        TSDG_HIP(hipStreamSynchronize(stream));
        std::memcpy(&split_xmax, &h_max, 4);
    }
    // rounding-error bound of the split expansion, as a multiple of (|q|^2 + max|x|^2) of the centred rows:
    // dropped terms 3*2^-16, fp32 accumulation over 3*dp products, norms and centring a few 2^-24
    // (the accumulation term is doubled because the accumulators also carry |x|^2 from the start)
    // One binary16 part: each element carries a relative error of 2^-11 or, below the normal range, an absolute
    // one of delta = 2^-25 in scaled units, so |error of |x|^2 - 2 q.x| <= (2^-10 + 2^-22)(|q|^2 + |x|^2)
    // + delta sqrt(dp) (2 + |q|^2 + |x|^2) + 2 dp delta^2 (scaled), plus the accumulation over dp products.
    const double delta = 2.98023223876953125e-8, sq = std::sqrt((double)dp);
    const float split_err = single ? (float)(1.05 * (1.0 / 1024.0 + 1.0 / 4194304.0 + delta * sq + (2.0 * dp + 64.0) * 5.9604645e-8))
                                   : (float)(1.05 * (3.0 / 65536.0 + (6.0 * dp + 64.0) * 5.9604645e-8));
    const float split_err_const = single ? (float)(1.05 * (2.0 * delta * sq + 2.0 * dp * delta * delta) / (double)scale2) : 0.f;

    // dynamic part, the slabs
    const int wmode = !wide ? 0 : single ? 2 : 1;
    const WideLaunch wl = wide_launch(wmode);
    const size_t kWideLds = wl.lds;
    if (wide || iwide) {
        hipError_t e = hipFuncSetAttribute(!wide ? reinterpret_cast<const void*>(&filter_wide_kernel<0>)
                                           : single ? reinterpret_cast<const void*>(&filter_wide_kernel<2>)
                                                    : reinterpret_cast<const void*>(&filter_wide_kernel<1>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kWideLds);
        if (e != hipSuccess) {
            set_error("hipFuncSetAttribute(%zu bytes of LDS) failed: %s", kWideLds, hipGetErrorString(e));
            return ANN_EDEVICE;
        }
    }

    const bool progress = ctx.progress != nullptr;
    const int64_t rb = std::min(row_block, nq);
    TSDG_HIP(tau.alloc((size_t)rb * 4));
    TSDG_HIP(cnt.alloc((size_t)rb * 4));
    TSDG_HIP(kept.alloc((size_t)rb * 4));
    TSDG_HIP(ovf.alloc((size_t)rb * 4));
    TSDG_HIP(buf.alloc((size_t)rb * cap * 8));
    TSDG_HIP(redo_cnt.alloc(4));
    TSDG_HIP(redo_rows.alloc((size_t)rb * 4));

    for (int64_t r0 = 0; r0 < nq; r0 += rb) {
        const int64_t nr = std::min(rb, nq - r0);
        TSDG_HIP(hipMemsetAsync(cnt.p, 0, (size_t)nr * 4, stream));
        TSDG_HIP(hipMemsetAsync(kept.p, 0, (size_t)nr * 4, stream));
        TSDG_HIP(hipMemsetAsync(ovf.p, 0, (size_t)nr * 4, stream));
        TSDG_HIP(hipMemsetAsync(redo_cnt.p, 0, 4, stream));
        TSDG_LAUNCH(fill_f32, dim3((unsigned)((nr + 255) / 256)), dim3(256), 0, stream, tau.as<float>(), nr, kInf);

        FilterArgs f;
        f.q = queries + r0 * d;
        f.x = base;
        f.qnorm = qn + r0;
        f.xnorm = xnorm.as<float>();
        f.tau = tau.as<float>();
        f.cnt = cnt.as<unsigned>();
        f.buf = buf.as<uint64_t>();
        f.nq = nr;
        f.N = N;
        f.self_offset = self ? r0 : -1 - nq;  // never equal to a column id when not self
        f.d = d;
        f.cap = cap;
        CompactArgs c;
        c.cnt = cnt.as<unsigned>();
        c.kept = kept.as<unsigned>();
        c.buf = buf.as<uint64_t>();
        c.tau = tau.as<float>();
        c.overflow = ovf.as<unsigned>();
        c.nq = nr;
        c.cap = cap;
        c.kprime = kprime;

        // column chunks of doubling size; the first must fit a buffer even with tau = +inf
        int64_t cb = 0, width = cap - kprime >= 128 ? 128 : 64;
        while (cb < N) {
            const int64_t ce = std::min(N, cb + width);
            f.c_begin = cb;
            f.c_end = ce;
            if (fast) {
                I8Args fa;
                fa.qc = (self ? xc8.as<uint8_t>() : qc8.as<uint8_t>()) + r0 * dp8;
                fa.xc = xc8.as<uint8_t>();
                fa.qnorm = (self ? xn8.as<int>() : qn8.as<int>()) + r0;
                fa.xnorm = xn8.as<int>();
                fa.tau = f.tau;
                fa.cnt = f.cnt;
                fa.buf = f.buf;
                fa.nq = nr;
                fa.c_begin = cb;
                fa.c_end = ce;
                fa.self_offset = f.self_offset;
                fa.cap = cap;
                const int64_t ftiles = (ce - cb + kI8Rows - 1) / kI8Rows;
                // long column spans per workgroup once there are enough workgroups to fill the chip
                fa.tiles_per_block = (int)std::min<int64_t>((nr + 255) / 256 >= 2048 ? 64 : 16, ftiles);
                dim3 fgrid((unsigned)((nr + 255) / 256), (unsigned)((ftiles + fa.tiles_per_block - 1) / fa.tiles_per_block));
                switch (ks8) {
#define TSDG_KS(n) case n: TSDG_LAUNCH((filter_i8_kernel<n>), fgrid, dim3(256), 0, stream, fa); break;
                    TSDG_KS(1) TSDG_KS(2) TSDG_KS(3) TSDG_KS(4)
#undef TSDG_KS
                }
            } else if (split) {
                WideArgs wa;
                SplitArgs& sa = wa.s;
                sa.qh = (self ? xh.as<uint16_t>() : qh.as<uint16_t>()) + r0 * dp;
                sa.ql = single ? nullptr : (self ? xl.as<uint16_t>() : ql.as<uint16_t>()) + r0 * dp;
                sa.xh = xh.as<uint16_t>();
                sa.xl = single ? nullptr : xl.as<uint16_t>();
                sa.scale2 = scale2;
                sa.inv_scale2 = 1.f / scale2;
                sa.qnorm = (self ? cxnorm.as<float>() : cqnorm.as<float>()) + r0;
                sa.xnorm = cxnorm.as<float>();
                sa.tau = f.tau;
                sa.cnt = f.cnt;
                sa.buf = f.buf;
                sa.nq = nr;
                sa.c_begin = cb;
                sa.c_end = ce;
                sa.self_offset = f.self_offset;
                sa.cap = cap;
                if (wide) {
                    const int64_t wtiles = (ce - cb + wl.xt - 1) / wl.xt;
                    sa.tiles_per_block = (int)std::min<int64_t>(wide_span_rows(wmode) / wl.xt, wtiles);
                    wa.dp = dp;
                    wa.q_tiles = (int)((nr + wl.qt - 1) / wl.qt);
                    wa.ny = (int)((wtiles + sa.tiles_per_block - 1) / sa.tiles_per_block);
                    wa.q_group = 64;
                    if (single)
                        TSDG_LAUNCH(filter_wide_kernel<2>, folded_grid((int64_t)wa.q_tiles * wa.ny), dim3(wl.threads),
                                           kWideLds, stream, wa);
                    else
                        TSDG_LAUNCH(filter_wide_kernel<1>, folded_grid((int64_t)wa.q_tiles * wa.ny), dim3(wl.threads),
                                           kWideLds, stream, wa);
                } else {
                    const int srows = split_tile_rows(ks, single);
                    const int64_t ftiles = (ce - cb + srows - 1) / srows;
                    sa.tiles_per_block = (int)std::min<int64_t>(32 * kSplitRows / srows, ftiles);
                    constexpr int qpb = 128 * kSplitQB;   // queries per workgroup
                    dim3 sgrid((unsigned)((nr + qpb - 1) / qpb), (unsigned)((ftiles + sa.tiles_per_block - 1) / sa.tiles_per_block));
                    switch (ks) {
#define TSDG_KS(n) case n: \
    if (single) TSDG_LAUNCH((filter_split_kernel<n, true>), sgrid, dim3(256), 0, stream, sa); \
    else TSDG_LAUNCH((filter_split_kernel<n, false>), sgrid, dim3(256), 0, stream, sa); \
    break;
                        TSDG_KS(1) TSDG_KS(2) TSDG_KS(3) TSDG_KS(4) TSDG_KS(5) TSDG_KS(6) TSDG_KS(7) TSDG_KS(8)
#undef TSDG_KS
                    }
                }
            } else {  // integer rows wider than 128 elements
                WideArgs wa;
                SplitArgs& sa = wa.s;
                sa.qh = (self ? xb16.as<uint16_t>() : qb16.as<uint16_t>()) + r0 * dpi;
                sa.ql = nullptr;
                sa.xh = xb16.as<uint16_t>();
                sa.xl = nullptr;
                sa.scale2 = sa.inv_scale2 = 1.f;
                sa.qnorm = reinterpret_cast<const float*>((self ? xn16.as<int>() : qn16.as<int>()) + r0);  // ints
                sa.xnorm = reinterpret_cast<const float*>(xn16.as<int>());
                sa.tau = f.tau;
                sa.cnt = f.cnt;
                sa.buf = f.buf;
                sa.nq = nr;
                sa.c_begin = cb;
                sa.c_end = ce;
                sa.self_offset = f.self_offset;
                sa.cap = cap;
                const int64_t wtiles = (ce - cb + wl.xt - 1) / wl.xt;
                sa.tiles_per_block = (int)std::min<int64_t>(wide_span_rows(wmode) / wl.xt, wtiles);
                wa.dp = dpi;
                wa.q_tiles = (int)((nr + wl.qt - 1) / wl.qt);
                wa.ny = (int)((wtiles + sa.tiles_per_block - 1) / sa.tiles_per_block);
                wa.q_group = 64;
                TSDG_LAUNCH(filter_wide_kernel<0>, folded_grid((int64_t)wa.q_tiles * wa.ny), dim3(wl.threads),
                                   kWideLds, stream, wa);
            }
            TSDG_HIP(launch_error());
            if (cap <= 256) TSDG_LAUNCH(compact_kernel<4>, dim3((unsigned)((nr + 3) / 4)), dim3(256), 0, stream, c);
            else TSDG_LAUNCH(compact_kernel<8>, dim3((unsigned)((nr + 3) / 4)), dim3(256), 0, stream, c);
            TSDG_HIP(launch_error());
            cb = ce;
            // next chunk as wide as everything seen so far, up to 2M columns per launch
            width = std::min<int64_t>(std::max<int64_t>(width, cb), 1ll << 21);
            if (progress) {  // long sweeps report each finished chunk
                TSDG_HIP(hipStreamSynchronize(stream));
                ctx.report("knn-sweep", cb, N);
            }
        }

        RefineLaunch<TQ, TB> rl;
        rl.a.q = queries + r0 * d;
        rl.a.x = base;
        rl.a.qnorm = split ? (self ? cxnorm.as<float>() : cqnorm.as<float>()) + r0 : qn + r0;
        rl.a.cnt = cnt.as<unsigned>();
        rl.a.buf = buf.as<uint64_t>();
        rl.a.tau = tau.as<float>();
        rl.a.overflow = ovf.as<unsigned>();
        rl.a.out_ids = out_ids + r0 * k;
        rl.a.out_s = out_s + r0 * k;
        rl.a.redo_cnt = redo_cnt.as<unsigned>();
        rl.a.redo_rows = redo_rows.as<int32_t>();
        rl.a.nq = nr;
        rl.a.d = d;
        rl.a.cap = cap;
        rl.a.k = k;
        rl.a.err_scale = split ? split_err : err_scale;
        rl.a.err_const = split ? split_err_const : 0.f;
        rl.a.xnorm_max = split ? split_xmax : xnorm_max;
        rl.a.q_is_base = self ? 1 : 0;
        rl.N = N;
        rl.self_offset = self ? r0 : -1;
        rl.stream = stream;
        rl.scan = false;
        rl.redo = 0;
        if (!dispatch_row_shape(dtype, d, rl)) {
            set_error("unsupported row shape d=%d", d);
            return ANN_EUNSUPPORTED;
        }
        TSDG_HIP(launch_error());
        unsigned redo = 0;
        TSDG_HIP(hipMemcpyAsync(&redo, redo_cnt.p, 4, hipMemcpyDeviceToHost, stream));
        TSDG_HIP(hipStreamSynchronize(stream));
        ctx.report("knn-rows", r0 + nr, nq);
        // the plain scan costs N distances per row: past a few rows in a thousand the hi + lo filter is cheaper
        if (single && (int64_t)redo > nr / 256 + 64) {
            *retry = true;
            return ANN_OK;
        }
        plain_scan_rows += redo;
        if (redo > 0) {
            rl.scan = true;
            rl.redo = redo;
            dispatch_row_shape(dtype, d, rl);
            TSDG_HIP(launch_error());
        }
    }
    TSDG_HIP(hipStreamSynchronize(stream));
    if (ctx.stats) {
        ctx.stats->knn_contraction = fast ? 0 : (iwide ? 3 : (single ? 1 : 2));
        ctx.stats->knn_plain_scan_rows = plain_scan_rows;
    }
    return ANN_OK;
}

}  // namespace

namespace {
template <typename TQ, typename TB>
ann_status knn_retrying(const TB* base, int64_t N, int d, ann_dtype dtype, const TQ* queries, int64_t nq, int k, bool self,
                        hipStream_t stream, int32_t* out_ids, float* out_s, const BuildCtx& ctx)
{
    const bool precise = ctx.knn_filter == 1;   // never use the one-part filter
    bool retry = false;
    ann_status rc = knn_typed<TQ, TB>(base, N, d, dtype, queries, nq, k, self, stream, out_ids, out_s, !precise, &retry, ctx);
    if (rc == ANN_OK && retry)
        rc = knn_typed<TQ, TB>(base, N, d, dtype, queries, nq, k, self, stream, out_ids, out_s, false, &retry, ctx);
    return rc;
}
}  // namespace

ann_status knn_exact(const void* base, int64_t N, int d, ann_dtype dtype, const float* queries, int64_t nq, int k,
                     bool exclude_self, hipStream_t stream, int32_t* out_ids, float* out_s, const BuildCtx& ctx)
{
    if (exclude_self) {
        if (dtype == ANN_U8)
            return knn_retrying<uint8_t, uint8_t>(static_cast<const uint8_t*>(base), N, d, dtype,
                                                  static_cast<const uint8_t*>(base), N, k, true, stream, out_ids, out_s, ctx);
        return knn_retrying<float, float>(static_cast<const float*>(base), N, d, dtype, static_cast<const float*>(base),
                                          N, k, true, stream, out_ids, out_s, ctx);
    }
    if (dtype == ANN_U8)
        return knn_retrying<float, uint8_t>(static_cast<const uint8_t*>(base), N, d, dtype, queries, nq, k, false, stream,
                                            out_ids, out_s, ctx);
    return knn_retrying<float, float>(static_cast<const float*>(base), N, d, dtype, queries, nq, k, false, stream,
                                      out_ids, out_s, ctx);
}

}  // namespace tsdg
