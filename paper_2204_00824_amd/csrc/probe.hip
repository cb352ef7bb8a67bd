// Measurement probes (not steps of the method).
//
// How fast can this GPU gather whole rows at random?
// The search's step S5 reads rows of d*e bytes at ids nobody can predict; its
// roofline is priced against the published HBM peak, and this kernel shows how
// much of that peak a plain gather of the same shape reaches, with none of the
// search's control flow around it.  G lanes read one row, 16 bytes per lane per
// chunk (the access shape of RowDist), several rows per wave in flight; a row's
// words are xor-folded into one word that is written out, so no load can be dropped.
#include "common.hpp"
#include "../../include/tsdg_probe.h"

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

// How fast do the matrix cores run with nothing around them?  Every wave keeps four independent
// 32x32 accumulator blocks in registers and issues MFMAs on constant fragments (all ones, or see RANDOM), no
// memory access in the loop; the k-NN contraction's fraction of the published peak is read
// against what this loop reaches.  KIND 0: v_mfma_i32_32x32x32_i8, 1: v_mfma_f32_32x32x16_bf16.
typedef int probe_i4 __attribute__((ext_vector_type(4)));
typedef int probe_i16 __attribute__((ext_vector_type(16)));
typedef __bf16 probe_bf8 __attribute__((ext_vector_type(8)));
typedef float probe_f16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t probe_mix(uint32_t x)
{
    x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
    return x;
}

// RANDOM: the fragments hold pseudo-random values (int8: any byte; bf16: +-[1, 2) with a random
// mantissa), different in every lane, operand and accumulator block, instead of ones.  The
// instruction stream is the same; what changes is how many wires toggle, that is the power drawn,
// and with it the rate the chip sustains.
template <int KIND, bool RANDOM>
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* __restrict__ out)
{
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    uint4 fa[4], fb[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        uint32_t w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t h = probe_mix((uint32_t)threadIdx.x * 64u + (uint32_t)(b * 8 + i) + 1u);
            const uint32_t one = KIND == 0 ? 0x01010101u : 0x3F803F80u;
            // bf16: keep sign and mantissa bits of both halves, fix the exponent at 127
            w[i] = !RANDOM ? one : KIND == 0 ? h : ((h & 0x807F807Fu) | 0x3F803F80u);
        }
        fa[b] = make_uint4(w[0], w[1], w[2], w[3]);
        fb[b] = make_uint4(w[4], w[5], w[6], w[7]);
    }
    float result = 0.f;
    if constexpr (KIND == 0) {
        probe_i16 acc[4];
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[b][r] = 0;
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(probe_i4, fa[b]),
                                                               __builtin_bit_cast(probe_i4, fb[b]), acc[b], 0, 0, 0);
        result = (float)(acc[0][0] + acc[1][5] + acc[2][10] + acc[3][15]);
    } else {
        probe_f16 acc[4];
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(probe_bf8, fa[b]),
                                                                 __builtin_bit_cast(probe_bf8, fb[b]), acc[b], 0, 0, 0);
        result = acc[0][0] + acc[1][5] + acc[2][10] + acc[3][15];
    }
    if (lane_id() == 0) out[wave] = result;  // ones: 4 * iters * (32 or 16), every MFMA is accounted for
}

}  // namespace tsdg

extern "C" ann_status ann_probe_mfma(int kind, int blocks, int iters, float* out, void* stream)
{
    using namespace tsdg;
    if (!out) { set_error("ann_probe_mfma: null pointer"); return ANN_EINVAL; }
    if (kind < 0 || kind > 3) {
        set_error("ann_probe_mfma: kind must be 0 (int8), 1 (bf16), 2 (int8, random fragments) or 3 (bf16, random fragments)");
        return ANN_EINVAL;
    }
    if (blocks < 1 || blocks > (1 << 20) || iters < 1 || iters > 100000) {
        set_error("ann_probe_mfma: need 1 <= blocks <= 2^20 and 1 <= iters <= 100000");
        return ANN_EINVAL;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (kind == 0) probe_mfma_kernel<0, false><<<blocks, 256, 0, st>>>(iters, out);
    else if (kind == 1) probe_mfma_kernel<1, false><<<blocks, 256, 0, st>>>(iters, out);
    else if (kind == 2) probe_mfma_kernel<0, true><<<blocks, 256, 0, st>>>(iters, out);
    else probe_mfma_kernel<1, true><<<blocks, 256, 0, st>>>(iters, out);
    TSDG_HIP(launch_error());
    return ANN_OK;
}

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
    TSDG_HIP(launch_error());
    return ANN_OK;
}
