// Shared host/device definitions of the HIP library (gfx950, wave64).
// Nothing here is shared with the CPU oracle.
#pragma once
#include <algorithm>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tsdg_ann.h"

namespace tsdg {

// ---- packed adjacency word: bits 0..26 node id, bits 27..31 lambda (0..30); all ones = unused slot
constexpr uint32_t kPackPad = 0xFFFFFFFFu;
constexpr uint32_t kIdBits = 27;
constexpr uint32_t kIdMask = (1u << kIdBits) - 1u;
constexpr int kMaxLambda = 30;
constexpr int kMaxK = 64;
constexpr int kMaxL = 512;

// ---- rank-list key: high word = bit pattern of the fp32 squared distance (non-negative, so the
// unsigned order of the bits is the numeric order), low word = id << 1 | expanded flag.  Ids are
// unique in a list, so the unsigned 64-bit order of keys is the (distance, id) order.
constexpr uint64_t kKeyEmpty = ~0ull;
constexpr uint32_t kHashEmpty = 0xFFFFFFFFu;

struct ann_graph_impl {
    int64_t N;
    int K;
    int d;             // row length of the base set the graph describes
    int max_lambda;    // largest lambda stored
    uint32_t* packed;  // [N,K] device
    int device;
};

// What a build call hands down to its steps: the caller's progress callback and report (both
// optional) and the two switches of the exact contraction.
struct BuildCtx {
    ann_progress_fn progress = nullptr;
    void* progress_user = nullptr;
    ann_build_stats* stats = nullptr;
    int knn_filter = 0;        // 1: hi + lo bf16 parts from the start
    int64_t knn_row_block = 0; // 0: default
    void report(const char* step, int64_t done, int64_t total) const
    {
        if (progress) progress(progress_user, step, done, total);
    }
};

// ---- grids that grow with the number of base rows
// A dispatch counts the work-items of each grid dimension in 32 bits, so a 1-D grid of B
// workgroups of T threads needs B*T < 2^32 -- which 64 threads per base row break beyond 67M
// rows.  Such grids are folded into two dimensions; the kernel takes its linear workgroup index
// from linear_block() and leaves when that is past its work.
constexpr unsigned kGridFold = 1u << 16;  // small enough that sets of a few 10^5 rows already take the folded path
inline dim3 folded_grid(int64_t blocks)
{
    if (blocks <= (int64_t)kGridFold) return dim3((unsigned)std::max<int64_t>(blocks, 1));
    return dim3(kGridFold, (unsigned)((blocks + kGridFold - 1) / kGridFold));
}
#ifdef __HIPCC__
__device__ __forceinline__ int64_t linear_block() { return (int64_t)blockIdx.y * (int64_t)gridDim.x + (int64_t)blockIdx.x; }
#endif

// ---- error plumbing (host)
void set_error(const char* fmt, ...);

// ---- every kernel launch goes through this check
// A dispatch counts the work-items of each grid dimension in 32 bits and takes at most 65,535
// workgroups in y and z.  A launch outside that is refused on the host (it would otherwise run with
// a truncated grid or fault): the launch is skipped, the thread's error message says which kernel,
// and launch_error(), which the launchers ask instead of hipGetLastError(), reports it once.
bool launch_fits(dim3 grid, dim3 block, const char* kernel);
hipError_t launch_error();
#define TSDG_LAUNCH(kern, grid, block, lds, stream, ...)                                      \
    do {                                                                                      \
        const dim3 g_ = (grid), b_ = (block);                                                 \
        if (tsdg::launch_fits(g_, b_, #kern)) hipLaunchKernelGGL(kern, g_, b_, lds, stream, __VA_ARGS__); \
    } while (0)
void hip_failed(const char* call, hipError_t e, const char* file, int line);  // sets the thread's error message
#define TSDG_HIP(call)                                                                     \
    do {                                                                                   \
        hipError_t e_ = (call);                                                            \
        if (e_ != hipSuccess) {                                                            \
            tsdg::hip_failed(#call, e_, __FILE__, __LINE__);                               \
            return e_ == hipErrorOutOfMemory ? ANN_ENOMEM : ANN_EDEVICE;                   \
        }                                                                                  \
    } while (0)

// ---- launchers implemented in the .hip files
struct SearchLaunch {
    const uint32_t* packed;
    int64_t N;
    int K;
    const void* base;
    ann_dtype dtype;
    int d;
    const float* queries;
    int nq;
    int k;
    int L;
    int lambda_visit;  // already resolved (1..32)
    int n_seeds;
    uint64_t seed;
    int max_hops;
    int visited_slots;  // a multiple of 64
    int waves;          // 1 = large-batch kernel
    int64_t qi_offset;
    int32_t* out_ids;
    float* out_dists;
    ann_query_stats* stats;
    hipStream_t stream;
};
ann_status launch_search(const SearchLaunch& a);

struct MultiLaunch {
    const uint32_t* packed;
    int64_t N;
    int K;
    const void* base;
    ann_dtype dtype;
    int d;
    const float* queries;
    int nq, k, t0, lambda_visit, max_hops;
    uint64_t seed;
    int64_t qi_offset;
    uint64_t* scratch;  // [nq, t0, 33]
    int32_t* out_ids;
    float* out_dists;
    ann_query_stats* stats;
    hipStream_t stream;
};
ann_status launch_search_multi(const MultiLaunch& a);
// Device address, on the current device, of the library's own scratch for up to
// kMultiStaticSearches searches of one multi-search call (a file-scope array in multi.hip).
constexpr int kMultiStaticSearches = 2048;
ann_status multi_static_scratch(uint64_t** out);

struct Alg2Launch {
    const uint32_t* packed;
    int64_t N;
    int K;
    const void* base;
    ann_dtype dtype;
    int d;
    const float* queries;
    int nq, k, m_c, m_v, lambda_visit, max_hops;
    int metric;   // 0: the measure is the L2 distance sqrt(s); 1: 1 - cos = s/2
    float delta;  // in units of the measure
    uint64_t seed;
    int64_t qi_offset;
    int32_t* out_ids;
    float* out_dists;
    ann_query_stats* stats;
    hipStream_t stream;
};
ann_status launch_search_alg2(const Alg2Launch& a);

ann_status knn_exact(const void* base, int64_t N, int d, ann_dtype dtype, const float* queries,
                     int64_t nq, int k, bool exclude_self, hipStream_t stream, int32_t* out_ids,
                     float* out_s, const BuildCtx& ctx);

// Approximate k-NN lists by neighbourhood propagation (descent.hip); lists in (s,id) order, -1 / +inf padded.
ann_status knn_descent(const void* base, int64_t N, int d, ann_dtype dtype, int K, int S, int max_iters, float delta,
                       uint64_t seed, const int32_t* init_ids, hipStream_t stream, int32_t* out_ids, float* out_s,
                       int* iters_done, int64_t* last_changed, const BuildCtx& ctx);

ann_status diversify(const void* base, int64_t N, int d, ann_dtype dtype, int K, const int32_t* knn_id,
                     const float* knn_s, float alpha_on_s, int lambda0, int rev_cap, hipStream_t stream,
                     uint32_t* packed, int* max_lambda, const BuildCtx& ctx);

ann_status pack_graph(const int32_t* adj, const uint8_t* lam, int64_t N, int K, hipStream_t stream,
                      uint32_t* packed, int* max_lambda);
ann_status unpack_graph(const uint32_t* packed, int64_t N, int K, hipStream_t stream, int32_t* adj,
                        uint8_t* lam);

// ---- device helpers
#if defined(__HIPCC__)
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63u); }
__device__ __forceinline__ uint64_t ballot64(bool p) { return (uint64_t)__ballot(p ? 1 : 0); }
__device__ __forceinline__ int popc64(uint64_t m) { return __popcll((unsigned long long)m); }
__device__ __forceinline__ int ctz64(uint64_t m) { return __builtin_ctzll((unsigned long long)m); }
__device__ __forceinline__ uint64_t lanes_below(int lane) { return (1ull << lane) - 1ull; }

__device__ __forceinline__ uint32_t bcast32(uint32_t v, int src) { return (uint32_t)__shfl((int)v, src, 64); }
__device__ __forceinline__ uint64_t bcast64(uint64_t v, int src)
{
    uint32_t lo = bcast32((uint32_t)v, src), hi = bcast32((uint32_t)(v >> 32), src);
    return ((uint64_t)hi << 32) | lo;
}
// broadcast from a lane whose index is wave-uniform (v_readlane: no LDS round trip)
__device__ __forceinline__ uint32_t readlane32(uint32_t v, int src)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, src);
}
__device__ __forceinline__ uint64_t readlane64(uint64_t v, int src)
{
    return ((uint64_t)readlane32((uint32_t)(v >> 32), src) << 32) | readlane32((uint32_t)v, src);
}
// value of the lane given by a DPP control word (quad_perm / row_mirror / row_half_mirror)
template <int CTRL> __device__ __forceinline__ double dpp_f64(double v)
{
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xFFFFFFFFll), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xF, 0xF, false);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
__device__ __forceinline__ double shfl_xor_f64(double v, int mask)
{
    long long b = __double_as_longlong(v);
    int lo = __shfl_xor((int)(b & 0xFFFFFFFFll), mask, 64);
    int hi = __shfl_xor((int)(b >> 32), mask, 64);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

__device__ __forceinline__ uint64_t make_key(float s, uint32_t id)
{
    return ((uint64_t)__float_as_uint(s) << 32) | (uint64_t)(id << 1);
}
__device__ __forceinline__ uint32_t key_id(uint64_t key) { return (uint32_t)(key & 0xFFFFFFFFull) >> 1; }
__device__ __forceinline__ float key_dist(uint64_t key) { return __uint_as_float((uint32_t)(key >> 32)); }

// Orders memory operations of the lanes of ONE wavefront (LDS is processed in
// issue order per wave; this only stops the compiler from moving accesses).
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}
#endif

}  // namespace tsdg
