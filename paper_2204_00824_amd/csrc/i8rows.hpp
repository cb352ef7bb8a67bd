// Rows that are integers in [0,255] as centred int8 (x' = x - 128), for the integer matrix
// cores: ||a - b||^2 = |a'|^2 + |b'|^2 - 2 a'.b' holds for the centred rows and is exact in int32.
#pragma once
#include "common.hpp"

namespace tsdg {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float4 i8rows_load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 i8rows_load4(const uint8_t* p)
{
    const uint32_t w = *reinterpret_cast<const uint32_t*>(p);
    return make_float4((float)(w & 0xFFu), (float)((w >> 8) & 0xFFu), (float)((w >> 16) & 0xFFu), (float)(w >> 24));
}

// 8 lanes per row: x' = x - 128 as packed bytes (zero beyond d, rows padded to dp, a multiple of
// 32) and |x'|^2.  *not_integer (optional) is set when some element is not an integer in [0,255];
// the outputs are then meaningless.
template <typename T>
__global__ __launch_bounds__(256) void i8_prep_kernel(const T* __restrict__ x, int64_t n, int d, int dp,
                                                      uint8_t* __restrict__ xc, int* __restrict__ norms,
                                                      unsigned* not_integer)
{
    const int64_t row = linear_block() * 32 + (threadIdx.x >> 3);
    const int g = (int)(threadIdx.x & 7);
    int acc = 0;
    bool bad = false;
    if (row < n)
        for (int j = 4 * g; j < dp; j += 32) {
            uint32_t w = 0u;
            if (j < d) {
                const float4 v = i8rows_load4(x + row * d + j);
                bad = bad || !(v.x >= 0.f && v.x <= 255.f && v.x == rintf(v.x)) ||
                      !(v.y >= 0.f && v.y <= 255.f && v.y == rintf(v.y)) ||
                      !(v.z >= 0.f && v.z <= 255.f && v.z == rintf(v.z)) ||
                      !(v.w >= 0.f && v.w <= 255.f && v.w == rintf(v.w));
                const int c0 = (int)v.x - 128, c1 = (int)v.y - 128, c2 = (int)v.z - 128, c3 = (int)v.w - 128;
                acc += c0 * c0 + c1 * c1 + c2 * c2 + c3 * c3;
                w = (uint32_t)(c0 & 0xFF) | ((uint32_t)(c1 & 0xFF) << 8) | ((uint32_t)(c2 & 0xFF) << 16) |
                    ((uint32_t)(c3 & 0xFF) << 24);
            }
            *reinterpret_cast<uint32_t*>(xc + row * dp + j) = w;
        }
#pragma unroll
    for (int o = 4; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (row < n && g == 0) norms[row] = acc;
    if (not_integer && bad && *not_integer == 0u) atomicOr(not_integer, 1u);
}

}  // namespace tsdg
