// extern "C" entry points (include/tsdg_ann.h): argument validation, the graph
// object, import/export.  Every step of the path runs in the kernels of
// search.hip, knn.hip and diversify.hip; nothing here computes on the host.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "common.hpp"

namespace tsdg {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

void hip_failed(const char* call, hipError_t e, const char* file, int line)
{
    // a launch refused by launch_fits() has already said which kernel and why
    if (e == hipErrorInvalidConfiguration && std::strncmp(g_err, "launch of ", 10) == 0) return;
    set_error("%s failed: %s (%s:%d)", call, hipGetErrorString(e), file, line);
}

static thread_local bool g_launch_refused = false;

bool launch_fits(dim3 grid, dim3 block, const char* kernel)
{
    const uint64_t lim = 1ull << 32;
    const bool ok = grid.x > 0 && grid.y > 0 && grid.z > 0 && (uint64_t)grid.x * block.x < lim &&
                    (uint64_t)grid.y * block.y < lim && (uint64_t)grid.z * block.z < lim && grid.y <= 65535u &&
                    grid.z <= 65535u && (uint64_t)block.x * block.y * block.z <= 1024u;
    if (!ok) {
        set_error("launch of %s refused: grid %u x %u x %u of %u x %u x %u threads exceeds what one dispatch can count",
                  kernel, grid.x, grid.y, grid.z, block.x, block.y, block.z);
        g_launch_refused = true;
    }
    return ok;
}

hipError_t launch_error()
{
    if (g_launch_refused) {
        g_launch_refused = false;
        (void)hipGetLastError();
        return hipErrorInvalidConfiguration;
    }
    return hipGetLastError();
}

// ---- pack / unpack / validate --------------------------------------------------------------
// flags[0]: first violation code; flags[1]: max lambda seen
__global__ void pack_kernel(const int32_t* __restrict__ adj, const uint8_t* __restrict__ lam, int64_t N,
                            int K, uint32_t* __restrict__ packed, int* __restrict__ flags)
{
    const int64_t row = linear_block() * (blockDim.x / 64) + (threadIdx.x >> 6);
    const int lane = lane_id();
    if (row >= N) return;
    int32_t id = -1;
    int l = 255;
    if (lane < K) {
        id = adj[row * K + lane];
        l = lam[row * K + lane];
    }
    const bool used = lane < K && id >= 0;
    int bad = 0;
    if (used && (id >= N || id == row)) bad = 1;                 // range / self loop
    if (used && l > kMaxLambda) bad = 2;                         // lambda too large
    if (lane < K && id < -1) bad = 1;
    const uint64_t um = ballot64(used);
    if (um & (um + 1)) bad = bad ? bad : 3;                      // used slots must form a prefix
    for (uint64_t m = um; m; m &= m - 1) {                       // repeats in the row
        const int j = ctz64(m);
        const int32_t idj = (int32_t)bcast32((uint32_t)id, j);
        if (used && j < lane && idj == id) bad = bad ? bad : 4;
    }
    if (lane < K) packed[row * K + lane] = used ? ((uint32_t)id | ((uint32_t)l << kIdBits)) : kPackPad;
    if (bad) atomicCAS(&flags[0], 0, bad);
    // the row's largest lambda, then at most one atomic per row, and only when the value read first is smaller
    int lw = used ? l : 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lw = max(lw, __shfl_xor(lw, o, 64));
    if (lane == 0 && lw > flags[1]) atomicMax(&flags[1], lw);
}

__global__ void unpack_kernel(const uint32_t* __restrict__ packed, int64_t total, int32_t* __restrict__ adj,
                              uint8_t* __restrict__ lam)
{
    const int64_t i = linear_block() * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const uint32_t w = packed[i];
    adj[i] = w == kPackPad ? -1 : (int32_t)(w & kIdMask);
    lam[i] = w == kPackPad ? (uint8_t)255 : (uint8_t)(w >> kIdBits);
}

ann_status pack_graph(const int32_t* adj, const uint8_t* lam, int64_t N, int K, hipStream_t stream,
                      uint32_t* packed, int* max_lambda)
{
    int* flags = nullptr;
    TSDG_HIP(hipMalloc(&flags, 2 * sizeof(int)));
    hipError_t e = hipMemsetAsync(flags, 0, 2 * sizeof(int), stream);
    if (e == hipSuccess) {
        const int rows_per_block = 4;
        TSDG_LAUNCH(pack_kernel, folded_grid((N + rows_per_block - 1) / rows_per_block), dim3(64 * rows_per_block), 0, stream, adj, lam, N, K, packed,
                           flags);
        e = launch_error();
    }
    int h[2] = {0, 0};
    if (e == hipSuccess) e = hipMemcpyAsync(h, flags, sizeof(h), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    (void)hipFree(flags);
    if (e != hipSuccess) {
        set_error("graph import failed on the device: %s", hipGetErrorString(e));
        return ANN_EDEVICE;
    }
    if (h[0]) {
        static const char* why[] = {"", "id out of range or self loop", "lambda above 30",
                                    "unused slot before a used one", "repeated id in a row"};
        set_error("graph import: invalid adjacency (%s)", why[h[0]]);
        return ANN_EINVAL;
    }
    *max_lambda = h[1];
    return ANN_OK;
}

ann_status unpack_graph(const uint32_t* packed, int64_t N, int K, hipStream_t stream, int32_t* adj, uint8_t* lam)
{
    const int64_t total = N * K;
    TSDG_LAUNCH(unpack_kernel, folded_grid((total + 255) / 256), dim3(256), 0, stream, packed, total, adj, lam);
    TSDG_HIP(launch_error());
    TSDG_HIP(hipStreamSynchronize(stream));
    return ANN_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// storage_types: the call also takes rows that are only a storage format (binary16)
static ann_status check_rows(const void* base, int64_t N, int d, ann_dtype dtype, const char* what,
                             bool storage_types = false)
{
    if (!base) { set_error("%s: null pointer", what); return ANN_EINVAL; }
    if (dtype == ANN_F16 && !storage_types) {
        set_error("%s: binary16 rows are a storage type of the search calls only", what);
        return ANN_EUNSUPPORTED;
    }
    if (dtype != ANN_F32 && dtype != ANN_U8 && dtype != ANN_F16) { set_error("%s: unknown dtype %d", what, (int)dtype); return ANN_EINVAL; }
    if (N <= 0 || d <= 0) { set_error("%s: N and d must be positive", what); return ANN_EINVAL; }
    if (!aligned16(base)) { set_error("%s: rows must be 16-byte aligned", what); return ANN_EINVAL; }
    const int pc = dtype == ANN_U8 ? 16 : (dtype == ANN_F16 ? 8 : 4);
    const int dmax = dtype == ANN_U8 ? 1024 : 2048;
    if (d % pc != 0 || d > dmax) {
        set_error("%s: d=%d unsupported (must be a multiple of %d and at most %d)", what, d, pc, dmax);
        return ANN_EUNSUPPORTED;
    }
    return ANN_OK;
}

static ann_status check_metric(ann_metric metric, ann_dtype dtype, const char* what)
{
    if (metric != ANN_L2 && metric != ANN_COSINE) { set_error("%s: unknown metric %d", what, (int)metric); return ANN_EINVAL; }
    if (metric == ANN_COSINE && dtype != ANN_F32) {
        set_error("%s: the cosine metric needs unit rows, hence fp32 storage", what);
        return ANN_EUNSUPPORTED;
    }
    return ANN_OK;
}

static ann_status check_descent(int64_t N, int K, int S, int max_iters, float delta, const char* what)
{
    if (K < 1 || K > kMaxK || N <= K || N >= (1ll << kIdBits)) { set_error("%s: need 1 <= K <= 64 and K < N < 2^27", what); return ANN_EINVAL; }
    if (S < 2 || S > 16 || (S & (S - 1)) != 0) { set_error("%s: the sample size S must be 2, 4, 8 or 16 (S=%d)", what, S); return ANN_EINVAL; }
    if (max_iters < 0 || !(delta >= 0.f)) { set_error("%s: negative iteration count or delta", what); return ANN_EINVAL; }
    return ANN_OK;
}

// Distances of a cosine search are reported as m = 1 - cos = s/2 (exact halving; +inf stays +inf).
__global__ __launch_bounds__(256) void halve_kernel(float* __restrict__ v, int64_t n)
{
    const int64_t i = linear_block() * 256 + threadIdx.x;
    if (i < n) v[i] *= 0.5f;
}

static ann_status report_metric(ann_metric metric, float* out_dists, int64_t n, hipStream_t stream)
{
    if (metric != ANN_COSINE || n == 0) return ANN_OK;
    TSDG_LAUNCH(halve_kernel, folded_grid((n + 255) / 256), dim3(256), 0, stream, out_dists, n);
    TSDG_HIP(launch_error());
    return ANN_OK;
}

// One group of 8 lanes per row: sum of squares in fp64, norm rounded to fp32, quotients formed in
// fp64 and rounded once.
__global__ __launch_bounds__(256) void normalize_kernel(const float* __restrict__ src, int64_t n, int d,
                                                        float* __restrict__ dst)
{
    const int64_t row = linear_block() * 32 + (threadIdx.x >> 3);
    const int g = (int)(threadIdx.x & 7);
    double acc = 0.0;
    if (row < n)
        for (int j = 4 * g; j < d; j += 32) {
            const float4 v = *reinterpret_cast<const float4*>(src + row * d + j);
            acc += (double)v.x * (double)v.x;
            acc += (double)v.y * (double)v.y;
            acc += (double)v.z * (double)v.z;
            acc += (double)v.w * (double)v.w;
        }
#pragma unroll
    for (int o = 4; o > 0; o >>= 1) acc += shfl_xor_f64(acc, o);
    const float norm = (float)sqrt(acc);
    if (row < n)
        for (int j = 4 * g; j < d; j += 32) {
            const float4 v = *reinterpret_cast<const float4*>(src + row * d + j);
            float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
            if (norm > 0.f) {
                o.x = (float)((double)v.x / (double)norm);
                o.y = (float)((double)v.y / (double)norm);
                o.z = (float)((double)v.z / (double)norm);
                o.w = (float)((double)v.w / (double)norm);
            }
            *reinterpret_cast<float4*>(dst + row * d + j) = o;
        }
}

// Inner product by its reduction to L2: 8 lanes per row copy the row and append
// sqrt(max(0, M^2 - |x|^2)) (0 for queries) and three zeros; maxbits (optional) collects the
// largest squared norm as fp32 bits (non-negative floats order like unsigned integers).
__global__ __launch_bounds__(256) void ip_augment_kernel(const float* __restrict__ src, int64_t n, int d, float M,
                                                         int is_query, float* __restrict__ dst, unsigned* maxbits)
{
    const int64_t row = linear_block() * 32 + (threadIdx.x >> 3);
    const int g = (int)(threadIdx.x & 7);
    double acc = 0.0;
    if (row < n)
        for (int j = 4 * g; j < d; j += 32) {
            const float4 v = *reinterpret_cast<const float4*>(src + row * d + j);
            acc += (double)v.x * (double)v.x;
            acc += (double)v.y * (double)v.y;
            acc += (double)v.z * (double)v.z;
            acc += (double)v.w * (double)v.w;
            if (dst) *reinterpret_cast<float4*>(dst + row * (d + 4) + j) = v;
        }
#pragma unroll
    for (int o = 4; o > 0; o >>= 1) acc += shfl_xor_f64(acc, o);
    if (row < n && g == 0) {
        if (dst) {
            const double rest = (double)M * (double)M - acc;
            const float extra = is_query ? 0.f : (float)sqrt(rest > 0.0 ? rest : 0.0);
            *reinterpret_cast<float4*>(dst + row * (d + 4) + d) = make_float4(extra, 0.f, 0.f, 0.f);
        }
        if (maxbits) {
            const unsigned b = __float_as_uint((float)sqrt(acc));
            if (b > *maxbits) atomicMax(maxbits, b);
        }
    }
}

// Batch size from which one wavefront per query is the faster kernel (Sec. 4: the division between small and large
// batches depends on the device and on the row length).  Measured on MI355X at K = 32, L = 64, same lambda prefix for
// both kernels, batches of 1..8192 queries: rows of 128 bytes change over between 1,024 and 2,048 queries, rows of
// 384 and 512 bytes at 4,096 (two wavefronts per query still win at 2,048), rows of 3,840 bytes not below 8,192 (four
// wavefronts per query stay 8 % ahead there).  Between the measured row lengths the thresholds are stepped.
static int large_batch_threshold(int row_bytes)
{
    if (row_bytes <= 128) return 1024;
    if (row_bytes <= 512) return 4096;
    if (row_bytes <= 2048) return 16384;
    return 32768;
}

static int pow2_at_least(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

}  // namespace tsdg

using namespace tsdg;

extern "C" {

const char* ann_last_error(void) { return g_err; }

void ann_build_params_default(ann_build_params* p)
{
    if (!p) return;
    p->dtype = ANN_F32;
    p->alpha = 1.2f;
    p->lambda0 = 9;
    p->rev_cap = 0;
    p->stream = nullptr;
    p->metric = ANN_L2;
    p->knn_mode = 0;
    p->descent_S = 0;
    p->descent_iters = 0;
    p->descent_delta = 0.f;
    p->descent_seed = 0;
    p->knn_filter = 0;
    p->knn_row_block = 0;
    p->progress = nullptr;
    p->progress_user = nullptr;
    p->stats = nullptr;
}

void ann_search_params_default(ann_search_params* p)
{
    if (!p) return;
    p->dtype = ANN_F32;
    p->mode = 0;
    p->lambda_visit = 0;
    p->n_seeds = 32;
    p->seed = 0;
    p->max_hops = 0;
    p->visited_slots = 0;
    p->waves_per_query = 0;
    p->qi_offset = 0;
    p->stream = nullptr;
    p->metric = ANN_L2;
}

static void destroy_graph(ann_graph_impl* g)
{
    if (!g) return;
    if (g->packed) (void)hipFree(g->packed);
    delete g;
}

static ann_status new_graph(int64_t N, int K, int d, ann_graph_impl** out)
{
    ann_graph_impl* g = new (std::nothrow) ann_graph_impl();
    if (!g) { set_error("out of host memory"); return ANN_ENOMEM; }
    g->N = N;
    g->K = K;
    g->d = d;
    g->max_lambda = 0;
    g->packed = nullptr;
    g->device = 0;
    (void)hipGetDevice(&g->device);
    hipError_t e = hipMalloc(&g->packed, (size_t)N * (size_t)K * sizeof(uint32_t));
    if (e != hipSuccess) {
        set_error("hipMalloc of the graph (%lld x %d words) failed: %s", (long long)N, K, hipGetErrorString(e));
        delete g;
        return ANN_ENOMEM;
    }
    *out = g;
    return ANN_OK;
}

ann_status ann_graph_import(const int32_t* adj, const uint8_t* lam, int64_t N, int K, int d, void* stream,
                            ann_graph** out)
{
    g_err[0] = 0;
    if (!adj || !lam || !out) { set_error("ann_graph_import: null pointer"); return ANN_EINVAL; }
    if (K < 1 || K > kMaxK) { set_error("ann_graph_import: K=%d outside 1..64", K); return ANN_EINVAL; }
    if (N <= K || N >= (1ll << kIdBits)) { set_error("ann_graph_import: need K < N < 2^27"); return ANN_EINVAL; }
    if (d <= 0) { set_error("ann_graph_import: d must be positive"); return ANN_EINVAL; }
    ann_graph_impl* g = nullptr;
    ann_status rc = new_graph(N, K, d, &g);
    if (rc != ANN_OK) return rc;
    rc = pack_graph(adj, lam, N, K, static_cast<hipStream_t>(stream), g->packed, &g->max_lambda);
    if (rc != ANN_OK) {
        destroy_graph(g);
        return rc;
    }
    *out = reinterpret_cast<ann_graph*>(g);
    return ANN_OK;
}

ann_status ann_graph_export(const ann_graph* graph, int32_t* adj, uint8_t* lam, void* stream)
{
    g_err[0] = 0;
    if (!graph || !adj || !lam) { set_error("ann_graph_export: null pointer"); return ANN_EINVAL; }
    const ann_graph_impl* g = reinterpret_cast<const ann_graph_impl*>(graph);
    return unpack_graph(g->packed, g->N, g->K, static_cast<hipStream_t>(stream), adj, lam);
}

ann_status ann_graph_info(const ann_graph* graph, int64_t* N, int* K, int* d)
{
    if (!graph) { set_error("ann_graph_info: null graph"); return ANN_EINVAL; }
    const ann_graph_impl* g = reinterpret_cast<const ann_graph_impl*>(graph);
    if (N) *N = g->N;
    if (K) *K = g->K;
    if (d) *d = g->d;
    return ANN_OK;
}

void ann_graph_free(ann_graph* graph)
{
    if (!graph) return;
    destroy_graph(reinterpret_cast<ann_graph_impl*>(graph));
}

static ann_status make_ctx(const ann_build_params& p, const char* what, BuildCtx* ctx)
{
    if (p.knn_filter != 0 && p.knn_filter != 1) { set_error("%s: knn_filter must be 0 or 1", what); return ANN_EINVAL; }
    if (p.knn_row_block < 0 || p.knn_row_block % 256 != 0 || p.knn_row_block > (1ll << 21)) {
        set_error("%s: knn_row_block must be 0 or a multiple of 256 up to 2^21", what);
        return ANN_EINVAL;
    }
    ctx->progress = p.progress;
    ctx->progress_user = p.progress_user;
    ctx->stats = p.stats;
    ctx->knn_filter = p.knn_filter;
    ctx->knn_row_block = p.knn_row_block;
    if (p.stats) std::memset(p.stats, 0, sizeof(*p.stats));
    return ANN_OK;
}

// k-NN lists with the device time of the call written to the caller's report
static ann_status timed_knn(const void* base, int64_t N, int d, int K, const ann_build_params& p, const BuildCtx& ctx,
                            int32_t* knn_ids, float* knn_dists)
{
    hipStream_t stream = static_cast<hipStream_t>(p.stream);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (ctx.stats) {
        TSDG_HIP(hipEventCreate(&e0));
        if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); set_error("hipEventCreate failed"); return ANN_EDEVICE; }
        (void)hipEventRecord(e0, stream);
    }
    ann_status rc;
    if (p.knn_mode == 1) {
        int S = p.descent_S;
        if (S == 0) {
            S = 2;
            while (S * 2 <= std::min(16, K / 2)) S *= 2;
        }
        rc = check_descent(N, K, S, p.descent_iters, p.descent_delta, "ann_build_graph");
        if (rc == ANN_OK)
            rc = knn_descent(base, N, d, p.dtype, K, S, p.descent_iters == 0 ? 12 : p.descent_iters,
                             p.descent_delta == 0.f ? 0.001f : p.descent_delta, p.descent_seed, nullptr, stream, knn_ids,
                             knn_dists, nullptr, nullptr, ctx);
        if (rc == ANN_OK && ctx.stats) ctx.stats->knn_contraction = 4;
    } else {
        rc = knn_exact(base, N, d, p.dtype, nullptr, N, K, true, stream, knn_ids, knn_dists, ctx);
    }
    if (ctx.stats) {
        if (rc == ANN_OK) {
            hipError_t e = hipEventRecord(e1, stream);
            if (e == hipSuccess) e = hipEventSynchronize(e1);
            if (e == hipSuccess) e = hipEventElapsedTime(&ctx.stats->knn_ms, e0, e1);
            if (e != hipSuccess) { set_error("timing of the k-NN step failed: %s", hipGetErrorString(e)); rc = ANN_EDEVICE; }
        }
        (void)hipEventDestroy(e0);
        (void)hipEventDestroy(e1);
    }
    return rc;
}

ann_status ann_knn_ex(const void* base, int64_t N, int d, int K, const ann_build_params* params, int32_t* knn_ids,
                      float* knn_dists)
{
    g_err[0] = 0;
    ann_build_params p;
    ann_build_params_default(&p);
    if (params) p = *params;
    ann_status rc = check_rows(base, N, d, p.dtype, "ann_knn");
    if (rc != ANN_OK) return rc;
    if (!knn_ids || !knn_dists) { set_error("ann_knn: null output"); return ANN_EINVAL; }
    if (K < 1 || K > kMaxK || N <= K || N >= (1ll << kIdBits)) {
        set_error("ann_knn: need 1 <= K <= 64 and K < N < 2^27");
        return ANN_EINVAL;
    }
    BuildCtx ctx;
    rc = make_ctx(p, "ann_knn", &ctx);
    if (rc != ANN_OK) return rc;
    p.knn_mode = 0;
    return timed_knn(base, N, d, K, p, ctx, knn_ids, knn_dists);
}

ann_status ann_knn(const void* base, int64_t N, int d, int K, ann_dtype dtype, void* stream, int32_t* knn_ids,
                   float* knn_dists)
{
    ann_build_params p;
    ann_build_params_default(&p);
    p.dtype = dtype;
    p.stream = stream;
    return ann_knn_ex(base, N, d, K, &p, knn_ids, knn_dists);
}

ann_status ann_bruteforce(const void* base, int64_t N, int d, ann_dtype dtype, const float* queries, int nq,
                          int k, void* stream, int32_t* out_ids, float* out_dists)
{
    g_err[0] = 0;
    ann_status rc = check_rows(base, N, d, dtype, "ann_bruteforce");
    if (rc != ANN_OK) return rc;
    if (nq < 0 || (nq > 0 && (!queries || !out_ids || !out_dists))) {
        set_error("ann_bruteforce: null pointer or negative nq");
        return ANN_EINVAL;
    }
    if (!aligned16(queries)) { set_error("ann_bruteforce: query rows must be 16-byte aligned"); return ANN_EINVAL; }
    if (k < 1 || k > 128 || k > N || N >= (1ll << kIdBits)) {
        set_error("ann_bruteforce: need 1 <= k <= min(128, N) and N < 2^27");
        return ANN_EINVAL;
    }
    if (nq == 0) return ANN_OK;
    return knn_exact(base, N, d, dtype, queries, nq, k, false, static_cast<hipStream_t>(stream), out_ids, out_dists,
                     BuildCtx());
}

ann_status ann_build_graph_ex(const void* base, int64_t N, int d, int K, const ann_build_params* params,
                              ann_graph** out)
{
    g_err[0] = 0;
    ann_build_params p;
    ann_build_params_default(&p);
    if (params) p = *params;
    if (!out) { set_error("ann_build_graph: null output"); return ANN_EINVAL; }
    ann_status rc = check_rows(base, N, d, p.dtype, "ann_build_graph");
    if (rc != ANN_OK) return rc;
    if (K < 1 || K > kMaxK || N <= K || N >= (1ll << kIdBits)) {
        set_error("ann_build_graph: need 1 <= K <= 64 and K < N < 2^27");
        return ANN_EINVAL;
    }
    if (!(p.alpha >= 1.0f) || p.alpha > 16.0f) { set_error("ann_build_graph: alpha must be in [1,16]"); return ANN_EINVAL; }
    rc = check_metric(p.metric, p.dtype, "ann_build_graph");
    if (rc != ANN_OK) return rc;
    // Eq. 2 compares alpha*m with m.  m = L2 distance: alpha^2 on the squared distances; m = 1 - cos = s/2: alpha.
    const float alpha_on_s = p.metric == ANN_COSINE ? p.alpha : p.alpha * p.alpha;
    if (p.lambda0 < 0 || p.lambda0 > kMaxLambda) { set_error("ann_build_graph: lambda0 must be in 0..30"); return ANN_EINVAL; }
    if (p.knn_mode != 0 && p.knn_mode != 1) { set_error("ann_build_graph: knn_mode must be 0 or 1"); return ANN_EINVAL; }
    int rev_cap = p.rev_cap == 0 ? 2 * K : p.rev_cap;
    if (rev_cap < K || rev_cap > 2 * kMaxK) { set_error("ann_build_graph: rev_cap must be in K..128"); return ANN_EINVAL; }
    hipStream_t stream = static_cast<hipStream_t>(p.stream);
    BuildCtx ctx;
    rc = make_ctx(p, "ann_build_graph", &ctx);
    if (rc != ANN_OK) return rc;

    int32_t* knn_id = nullptr;
    float* knn_s = nullptr;
    TSDG_HIP(hipMalloc(&knn_id, (size_t)N * K * sizeof(int32_t)));
    hipError_t e = hipMalloc(&knn_s, (size_t)N * K * sizeof(float));
    if (e != hipSuccess) {
        (void)hipFree(knn_id);
        set_error("hipMalloc of the k-NN lists failed: %s", hipGetErrorString(e));
        return ANN_ENOMEM;
    }
    ann_graph_impl* g = nullptr;
    rc = timed_knn(base, N, d, K, p, ctx, knn_id, knn_s);
    if (rc == ANN_OK) rc = new_graph(N, K, d, &g);
    if (rc == ANN_OK)
        rc = diversify(base, N, d, p.dtype, K, knn_id, knn_s, alpha_on_s, p.lambda0, rev_cap, stream, g->packed,
                       &g->max_lambda, ctx);
    (void)hipFree(knn_id);
    (void)hipFree(knn_s);
    if (rc != ANN_OK) {
        destroy_graph(g);
        return rc;
    }
    *out = reinterpret_cast<ann_graph*>(g);
    return ANN_OK;
}

ann_status ann_build_graph(const void* base, int64_t N, int d, int K, ann_graph** out)
{
    return ann_build_graph_ex(base, N, d, K, nullptr, out);
}

ann_status ann_knn_descent(const void* base, int64_t N, int d, int K, ann_dtype dtype, int S, int max_iters,
                           float delta, uint64_t seed, const int32_t* init_ids, void* stream, int32_t* knn_ids,
                           float* knn_dists, int* iters_done, int64_t* last_changed)
{
    g_err[0] = 0;
    ann_status rc = check_rows(base, N, d, dtype, "ann_knn_descent");
    if (rc != ANN_OK) return rc;
    rc = check_descent(N, K, S, max_iters, delta, "ann_knn_descent");
    if (rc != ANN_OK) return rc;
    if (!knn_ids || !knn_dists) { set_error("ann_knn_descent: null output"); return ANN_EINVAL; }
    return knn_descent(base, N, d, dtype, K, S, max_iters, delta, seed, init_ids, static_cast<hipStream_t>(stream),
                       knn_ids, knn_dists, iters_done, last_changed, BuildCtx());
}

ann_status ann_max_row_norm(const float* src, int64_t n, int d, void* stream, float* M)
{
    g_err[0] = 0;
    if (!M) { set_error("ann_max_row_norm: null output"); return ANN_EINVAL; }
    ann_status rc = check_rows(src, n, d, ANN_F32, "ann_max_row_norm");
    if (rc != ANN_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned* bits = nullptr;
    TSDG_HIP(hipMalloc(&bits, sizeof(unsigned)));
    hipError_t e = hipMemsetAsync(bits, 0, sizeof(unsigned), st);
    unsigned h = 0;
    if (e == hipSuccess) {
        TSDG_LAUNCH(ip_augment_kernel, folded_grid((n + 31) / 32), dim3(256), 0, st, src, n, d, 0.f, 1,
                           static_cast<float*>(nullptr), bits);
        e = launch_error();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(&h, bits, sizeof(h), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(bits);
    if (e != hipSuccess) { set_error("ann_max_row_norm failed on the device: %s", hipGetErrorString(e)); return ANN_EDEVICE; }
    std::memcpy(M, &h, sizeof(float));
    return ANN_OK;
}

ann_status ann_ip_augment_rows(const float* src, int64_t n, int d, float M, int is_query, float* dst, void* stream)
{
    g_err[0] = 0;
    if (n == 0) return ANN_OK;
    ann_status rc = check_rows(src, n, d, ANN_F32, "ann_ip_augment_rows");
    if (rc != ANN_OK) return rc;
    if (d + 4 > 2048) { set_error("ann_ip_augment_rows: d + 4 must not exceed 2048"); return ANN_EUNSUPPORTED; }
    if (!dst || !aligned16(dst) || dst == src) { set_error("ann_ip_augment_rows: dst must be another 16-byte aligned device buffer"); return ANN_EINVAL; }
    if (!is_query && !(M > 0.f)) { set_error("ann_ip_augment_rows: base rows need M > 0"); return ANN_EINVAL; }
    TSDG_LAUNCH(ip_augment_kernel, folded_grid((n + 31) / 32), dim3(256), 0, static_cast<hipStream_t>(stream),
                       src, n, d, M, is_query ? 1 : 0, dst, static_cast<unsigned*>(nullptr));
    TSDG_HIP(launch_error());
    return ANN_OK;
}

ann_status ann_normalize_rows(const float* src, int64_t n, int d, float* dst, void* stream)
{
    g_err[0] = 0;
    if (n == 0) return ANN_OK;
    ann_status rc = check_rows(src, n, d, ANN_F32, "ann_normalize_rows");
    if (rc != ANN_OK) return rc;
    if (!dst || !aligned16(dst)) { set_error("ann_normalize_rows: dst must be a 16-byte aligned device pointer"); return ANN_EINVAL; }
    TSDG_LAUNCH(normalize_kernel, folded_grid((n + 31) / 32), dim3(256), 0, static_cast<hipStream_t>(stream),
                       src, n, d, dst);
    TSDG_HIP(launch_error());
    return ANN_OK;
}

ann_status ann_search_ex(const ann_graph* graph, const void* base, const void* queries, int nq, int k, int L,
                         const ann_search_params* params, int32_t* out_ids, float* out_dists,
                         ann_query_stats* stats)
{
    g_err[0] = 0;
    ann_search_params p;
    ann_search_params_default(&p);
    if (params) p = *params;
    if (!graph) { set_error("ann_search: null graph"); return ANN_EINVAL; }
    const ann_graph_impl* g = reinterpret_cast<const ann_graph_impl*>(graph);
    if (nq < 0) { set_error("ann_search: negative nq"); return ANN_EINVAL; }
    if (nq > (1 << 22)) { set_error("ann_search: at most 4,194,304 queries per call (nq=%d)", nq); return ANN_EUNSUPPORTED; }
    if (k < 1 || L < k || L > kMaxL) { set_error("ann_search: need 1 <= k <= L <= 512 (k=%d, L=%d)", k, L); return ANN_EINVAL; }
    if (p.n_seeds < 1) { set_error("ann_search: n_seeds must be positive"); return ANN_EINVAL; }
    if (p.max_hops < 0 || p.mode < 0 || p.mode > 2 || p.lambda_visit < 0) {
        set_error("ann_search: negative max_hops / lambda_visit or unknown mode");
        return ANN_EINVAL;
    }
    if (nq == 0) return ANN_OK;
    if (!queries || !out_ids || !out_dists) { set_error("ann_search: null pointer"); return ANN_EINVAL; }
    ann_status rc = check_rows(base, g->N, g->d, p.dtype, "ann_search", true);
    if (rc != ANN_OK) return rc;
    rc = check_metric(p.metric, p.dtype, "ann_search");
    if (rc != ANN_OK) return rc;
    if (!aligned16(queries)) { set_error("ann_search: query rows must be 16-byte aligned"); return ANN_EINVAL; }

    SearchLaunch s;
    s.packed = g->packed;
    s.N = g->N;
    s.K = g->K;
    s.base = base;
    s.dtype = p.dtype;
    s.d = g->d;
    s.queries = static_cast<const float*>(queries);
    s.nq = nq;
    s.k = k;
    s.L = L;
    s.n_seeds = p.n_seeds;
    s.seed = p.seed;
    s.max_hops = p.max_hops;
    s.qi_offset = p.qi_offset;
    s.out_ids = out_ids;
    s.out_dists = out_dists;
    s.stats = stats;
    s.stream = static_cast<hipStream_t>(p.stream);

    // batch regime (Sec. 4): below the threshold a query gets a whole workgroup
    const int row_bytes = g->d * (p.dtype == ANN_U8 ? 1 : (p.dtype == ANN_F16 ? 2 : 4));
    int mode = p.mode;
    if (mode == 0) mode = nq >= large_batch_threshold(row_bytes) ? 1 : 2;
    int waves = 1;
    if (mode == 2) {
        waves = p.waves_per_query;
        // same measurement: up to 512 queries the gather passes of a hop are best spread over eight wavefronts
        // (four for 128-byte rows, which need fewer passes); beyond, the CUs fill up and two wavefronts per
        // query do best on rows of 384 and 512 bytes, four on shorter and on longer rows
        if (waves == 0) {
            if (nq <= 512) waves = row_bytes <= 128 ? 4 : 8;
            else waves = (row_bytes <= 128 || row_bytes > 512) ? 4 : 2;
        }
        if (waves != 1 && waves != 2 && waves != 4 && waves != 8) {
            set_error("ann_search: waves_per_query must be 0, 1, 2, 4 or 8");
            return ANN_EINVAL;
        }
    }
    s.waves = waves;
    // visited prefix (Sec. 5.4): lambda < 10 for small batches, lambda < 5 for large ones
    int lv = p.lambda_visit;
    if (lv == 0) lv = mode == 2 ? 10 : 5;
    if (lv > 31) lv = 32;
    s.lambda_visit = lv;

    // Visited set: with one wave per query the LDS footprint decides how many queries a CU holds, and a
    // footprint that fills the LDS to the last kilobyte stalls placement; against that, every slot saves rows from
    // being scored twice, which costs more the longer the row.  Measured on 1M x 128 fp32 and uint8 and 4M x 96 fp32
    // (L = 29..512, sizes 384..2,048): while the list is in registers (L <= 128) 1,536 slots are fastest on 384- and
    // 512-byte rows (1,408 within 1 %, 1,792 5 % slower); with the list in LDS, 512-byte rows still take 1,536 (6 %
    // ahead of 1,024 at L = 512), shorter rows 1,024 (at L = 256 on 384-byte rows 1,216 and more are 10 % slower).
    // Byte rows of at most 128 elements run eight waves per SIMD (63 registers), so a CU holds 32 queries when a
    // query's LDS stays near 5 KB, and re-scoring a 128-byte row is cheap: 896 slots with the list in registers
    // (1,024 is 12 % slower), 384 with it in LDS (1,024 is 20 % slower at L = 256).  A workgroup per query has LDS to
    // spare, and a batch that leaves most CUs with one workgroup takes the largest set that still pays.
    int slots = p.visited_slots;
    if (slots == 0) {
        if (mode == 1) {
            slots = (L <= 128 || row_bytes >= 512) ? 1536 : 1024;
            if (p.dtype == ANN_U8 && g->d <= 128) slots = L <= 128 ? 896 : 384;
        } else if (nq <= 512) {
            slots = 8192;
        } else {
            slots = pow2_at_least(16 * L);
            if (slots < 1024) slots = 1024;
            if (slots > 8192) slots = 8192;
        }
    }
    if (slots < 64 || slots > 16384 || slots % 64 != 0) {
        set_error("ann_search: visited_slots must be a multiple of 64 in 64..16384");
        return ANN_EINVAL;
    }
    s.visited_slots = slots;
    rc = launch_search(s);
    if (rc != ANN_OK) return rc;
    return report_metric(p.metric, out_dists, (int64_t)nq * k, s.stream);
}

// Argument checks and launch shared by the two multi-search entry points.  `own_scratch`: the rankings pass
// through the library's file-scope array (no allocation) instead of the caller's workspace.
static ann_status search_multi_common(const ann_graph_impl* g, const void* base, const void* queries, int nq, int k,
                                      int t0, const ann_search_params* params, void* workspace, size_t workspace_bytes,
                                      int32_t* out_ids, float* out_dists, ann_query_stats* stats, bool own_scratch,
                                      const char* what)
{
    g_err[0] = 0;
    ann_search_params p;
    ann_search_params_default(&p);
    if (params) p = *params;
    if (!g) { set_error("%s: null graph", what); return ANN_EINVAL; }
    if (nq < 0) { set_error("%s: negative nq", what); return ANN_EINVAL; }
    if (k < 1 || k > 32) { set_error("%s: need 1 <= k <= 32 (k=%d)", what, k); return ANN_EINVAL; }
    if (t0 < 1 || t0 > 1024) { set_error("%s: need 1 <= t0 <= 1024 (t0=%d)", what, t0); return ANN_EINVAL; }
    if (p.max_hops < 0 || p.lambda_visit < 0) { set_error("%s: negative max_hops / lambda_visit", what); return ANN_EINVAL; }
    if (nq == 0) return ANN_OK;
    if (!queries || !out_ids || !out_dists) { set_error("%s: null pointer", what); return ANN_EINVAL; }
    ann_status rc = check_rows(base, g->N, g->d, p.dtype, what, true);
    if (rc != ANN_OK) return rc;
    rc = check_metric(p.metric, p.dtype, what);
    if (rc != ANN_OK) return rc;
    if (!aligned16(queries)) { set_error("%s: query rows must be 16-byte aligned", what); return ANN_EINVAL; }
    if ((int64_t)nq * t0 > 65535ll * 1024) { set_error("%s: nq * t0 too large", what); return ANN_EUNSUPPORTED; }
    if (nq > 65535) { set_error("%s: at most 65535 queries per call", what); return ANN_EUNSUPPORTED; }
    hipStream_t stream = static_cast<hipStream_t>(p.stream);
    const size_t need = ann_search_multi_workspace_bytes(nq, t0);
    uint64_t* scratch = nullptr;
    void* temporary = nullptr;
    if (own_scratch) {
        if ((int64_t)nq * t0 > kMultiStaticSearches) {
            set_error("%s: nq * t0 = %lld searches exceed the %d the library's own scratch holds", what,
                      (long long)nq * t0, kMultiStaticSearches);
            return ANN_EUNSUPPORTED;
        }
        rc = multi_static_scratch(&scratch);
        if (rc != ANN_OK) return rc;
    } else if (workspace) {
        if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 7u) != 0) {
            set_error("%s: the workspace must be 8-byte aligned and hold %zu bytes (got %zu)", what, need, workspace_bytes);
            return ANN_EINVAL;
        }
        scratch = static_cast<uint64_t*>(workspace);
    } else {
        hipError_t e = hipMalloc(&temporary, need);
        if (e != hipSuccess) { set_error("hipMalloc of the multi-search workspace failed: %s", hipGetErrorString(e)); return ANN_ENOMEM; }
        scratch = static_cast<uint64_t*>(temporary);
    }
    MultiLaunch s;
    s.packed = g->packed;
    s.N = g->N;
    s.K = g->K;
    s.base = base;
    s.dtype = p.dtype;
    s.d = g->d;
    s.queries = static_cast<const float*>(queries);
    s.nq = nq;
    s.k = k;
    s.t0 = t0;
    int lv = p.lambda_visit == 0 ? 10 : p.lambda_visit;   // small-batch prefix (Sec. 5.4)
    if (lv > 31) lv = 32;
    s.lambda_visit = lv;
    s.max_hops = p.max_hops == 0 ? 16 : p.max_hops;
    s.seed = p.seed;
    s.qi_offset = p.qi_offset;
    s.scratch = scratch;
    s.out_ids = out_ids;
    s.out_dists = out_dists;
    s.stats = stats;
    s.stream = stream;
    rc = launch_search_multi(s);
    if (rc == ANN_OK) rc = report_metric(p.metric, out_dists, (int64_t)nq * k, stream);
    if (temporary) {   // the convenience path: wait for the kernels, then give the memory back
        const hipError_t e = hipStreamSynchronize(stream);
        (void)hipFree(temporary);
        if (e != hipSuccess && rc == ANN_OK) { set_error("%s failed on the device: %s", what, hipGetErrorString(e)); rc = ANN_EDEVICE; }
    }
    return rc;
}

size_t ann_search_multi_workspace_bytes(int nq, int t0)
{
    if (nq <= 0 || t0 <= 0) return 0;
    return (size_t)nq * (size_t)t0 * 33 * sizeof(uint64_t);
}

ann_status ann_search_multi(const ann_graph* graph, const void* base, const void* queries, int nq, int k, int t0,
                            const ann_search_params* params, void* workspace, size_t workspace_bytes, int32_t* out_ids,
                            float* out_dists, ann_query_stats* stats)
{
    return search_multi_common(reinterpret_cast<const ann_graph_impl*>(graph), base, queries, nq, k, t0, params, workspace,
                               workspace_bytes, out_ids, out_dists, stats, false, "ann_search_multi");
}

ann_status ann_search_multi_static(const ann_graph* graph, const void* base, const void* queries, int nq, int k,
                                   int t0, const ann_search_params* params, int32_t* out_ids, float* out_dists,
                                   ann_query_stats* stats)
{
    return search_multi_common(reinterpret_cast<const ann_graph_impl*>(graph), base, queries, nq, k, t0, params, nullptr,
                               0, out_ids, out_dists, stats, true, "ann_search_multi_static");
}

ann_status ann_search_alg2(const ann_graph* graph, const void* base, const void* queries, int nq, int k,
                           float delta, int m_c, int m_v, const ann_search_params* params, int32_t* out_ids,
                           float* out_dists, ann_query_stats* stats)
{
    g_err[0] = 0;
    ann_search_params p;
    ann_search_params_default(&p);
    if (params) p = *params;
    if (!graph) { set_error("ann_search_alg2: null graph"); return ANN_EINVAL; }
    const ann_graph_impl* g = reinterpret_cast<const ann_graph_impl*>(graph);
    if (nq < 0) { set_error("ann_search_alg2: negative nq"); return ANN_EINVAL; }
    if (nq > (1 << 22)) { set_error("ann_search_alg2: at most 4,194,304 queries per call (nq=%d)", nq); return ANN_EUNSUPPORTED; }
    if (k < 1 || k > 64) { set_error("ann_search_alg2: need 1 <= k <= 64 (k=%d)", k); return ANN_EINVAL; }
    if (m_c < 1 || m_c > 64 || m_v < 1 || m_v > 64) { set_error("ann_search_alg2: m_c and m_v must be in 1..64"); return ANN_EINVAL; }
    if (!(delta >= 0.0f)) { set_error("ann_search_alg2: delta must be >= 0"); return ANN_EINVAL; }
    if (p.max_hops < 0 || p.lambda_visit < 0) { set_error("ann_search_alg2: negative max_hops / lambda_visit"); return ANN_EINVAL; }
    if (nq == 0) return ANN_OK;
    if (!queries || !out_ids || !out_dists) { set_error("ann_search_alg2: null pointer"); return ANN_EINVAL; }
    ann_status rc = check_rows(base, g->N, g->d, p.dtype, "ann_search_alg2", true);
    if (rc != ANN_OK) return rc;
    rc = check_metric(p.metric, p.dtype, "ann_search_alg2");
    if (rc != ANN_OK) return rc;
    if (!aligned16(queries)) { set_error("ann_search_alg2: query rows must be 16-byte aligned"); return ANN_EINVAL; }
    Alg2Launch s;
    s.packed = g->packed;
    s.N = g->N;
    s.K = g->K;
    s.base = base;
    s.dtype = p.dtype;
    s.d = g->d;
    s.queries = static_cast<const float*>(queries);
    s.nq = nq;
    s.k = k;
    s.m_c = m_c;
    s.m_v = m_v;
    int lv = p.lambda_visit == 0 ? 5 : p.lambda_visit;   // large-batch prefix (Sec. 5.4)
    if (lv > 31) lv = 32;
    s.lambda_visit = lv;
    s.max_hops = p.max_hops;
    s.delta = delta;  // in units of the measure m (Alg. 2 compares m itself)
    s.metric = p.metric == ANN_COSINE ? 1 : 0;
    s.seed = p.seed;
    s.qi_offset = p.qi_offset;
    s.out_ids = out_ids;
    s.out_dists = out_dists;
    s.stats = stats;
    s.stream = static_cast<hipStream_t>(p.stream);
    rc = launch_search_alg2(s);
    if (rc != ANN_OK) return rc;
    return report_metric(p.metric, out_dists, (int64_t)nq * k, s.stream);
}

ann_status ann_search(const ann_graph* graph, const void* base, const void* queries, int nq, int k, int L,
                      int32_t* out_ids, float* out_dists)
{
    return ann_search_ex(graph, base, queries, nq, k, L, nullptr, out_ids, out_dists, nullptr);
}

}  // extern "C"
