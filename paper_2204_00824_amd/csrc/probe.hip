// Measurement probe: how fast can this GPU gather whole rows at random?
//
// The search's step S5 reads rows of d*e bytes at ids nobody can predict; its
// roofline is priced against the published HBM peak, and this kernel shows how
// much of that peak a plain gather of the same shape reaches, with none of the
// search's control flow around it.  G lanes read one row, 16 bytes per lane per
// chunk (the access shape of RowDist), several rows per wave in flight; a row's
// words are xor-folded into one word that is written out, so no load can be dropped.
#include "common.hpp"

namespace tsdg {

template <int G>
__global__ __launch_bounds__(256) void probe_gather_kernel(const uint4* __restrict__ base, uint32_t N, int chunks_per_row,
                                                           const uint32_t* __restrict__ ids, int64_t n,
                                                           uint32_t* __restrict__ out)
{
    constexpr int VP = 64 / G;  // rows per pass of a wave
    constexpr int U = 4;        // passes in flight
    const int lane = lane_id();
    const int g = lane % G, v = lane / G;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t r0 = wave * (U * VP); r0 < n; r0 += nwaves * (U * VP)) {
        uint32_t acc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc[u] = 0u;
            const int64_t r = r0 + u * VP + v;
            if (r < n) {
                const uint32_t id = ids[r] < N ? ids[r] : N - 1u;  // an id past the end cannot fault
                const uint4* row = base + (size_t)id * (size_t)chunks_per_row;
#pragma unroll 4
                for (int c = g; c < chunks_per_row; c += G) {
                    const uint4 x = row[c];
                    acc[u] ^= x.x ^ x.y ^ x.z ^ x.w;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t a = acc[u];
#pragma unroll
            for (int o = 1; o < G; o <<= 1) a ^= (uint32_t)__shfl_xor((int)a, o, 64);
            const int64_t r = r0 + u * VP + v;
            if (r < n && g == 0) out[r] = a;
        }
    }
}

}  // namespace tsdg

extern "C" ann_status ann_probe_gather(const void* base, int64_t N, int row_bytes, const uint32_t* ids, int64_t n,
                                       uint32_t* out, void* stream)
{
    using namespace tsdg;
    if (!base || !ids || !out) { set_error("ann_probe_gather: null pointer"); return ANN_EINVAL; }
    if (N <= 0 || N > 0xFFFFFFFFll || n <= 0) { set_error("ann_probe_gather: need 0 < N < 2^32 and n > 0"); return ANN_EINVAL; }
    if (row_bytes < 16 || row_bytes % 16 != 0 || row_bytes > 8192) {
        set_error("ann_probe_gather: row_bytes must be a multiple of 16 in 16..8192");
        return ANN_EINVAL;
    }
    if (reinterpret_cast<uintptr_t>(base) % 16 != 0) { set_error("ann_probe_gather: base must be 16-byte aligned"); return ANN_EINVAL; }
    const int chunks = row_bytes / 16;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int blocks = 256 * 16;  // 16 workgroups of 4 waves per compute unit
    const uint4* b = static_cast<const uint4*>(base);
    if (chunks <= 32) probe_gather_kernel<8><<<blocks, 256, 0, st>>>(b, (uint32_t)N, chunks, ids, n, out);
    else if (chunks <= 64) probe_gather_kernel<16><<<blocks, 256, 0, st>>>(b, (uint32_t)N, chunks, ids, n, out);
    else if (chunks <= 128) probe_gather_kernel<32><<<blocks, 256, 0, st>>>(b, (uint32_t)N, chunks, ids, n, out);
    else probe_gather_kernel<64><<<blocks, 256, 0, st>>>(b, (uint32_t)N, chunks, ids, n, out);
    TSDG_HIP(hipGetLastError());
    return ANN_OK;
}
