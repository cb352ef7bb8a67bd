// Wave-cooperative squared-L2 evaluation between one query held in registers and
// rows gathered from the base set (search step S5; also used by the build's
// re-scoring pass).
//
// A row is cut into 16-byte chunks (4 fp32 or 16 uint8 elements).  G lanes form
// a group that owns one row per pass; lane g of the group reads chunks g, g+G,
// ..., so that each load instruction of a group covers G*16 contiguous bytes
// (128 B for G = 8: one cache line per group, 64/G rows per instruction).
// Every lane accumulates the squares of its fp32 differences in fp64, the G
// partial sums are added by an xor butterfly and the total is rounded once to
// fp32: the canonical distance fl32( sum (double)(fl32(a_j - b_j))^2 ).  The
// summation order depends only on (G, C), never on which operand is which, so
// the value is bitwise symmetric and reproducible.
#pragma once
#include "common.hpp"

namespace tsdg {

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kPerChunk = 4;
    using chunk_t = float4;
};
template <> struct Elem<uint8_t> {
    static constexpr int kPerChunk = 16;
    using chunk_t = uint4;
};
template <> struct Elem<_Float16> {  // IEEE binary16 storage; every value converts exactly to fp32
    static constexpr int kPerChunk = 8;
    using chunk_t = uint4;
};

template <typename T, int G, int C> struct RowDist {
    static constexpr int PC = Elem<T>::kPerChunk;
    static constexpr int VP = 64 / G;  // rows per pass
    static constexpr int NC = C;       // chunks per lane
    using chunk_t = typename Elem<T>::chunk_t;

    float q[C * PC];  // this lane's slices of the query
    // uint8 rows with an integer-valued query in [0,255]: the same slices as packed bytes, their
    // sum of squares, and the flag that selects the integer path (wave-uniform)
    uint32_t qbytes[(sizeof(T) == 1) ? C * 4 : 1];
    uint32_t qq;
    bool q_int;
    int g;            // lane within group
    int v;            // group within wave
    int nchunks;      // d / PC
    int d;

    __device__ __forceinline__ void init(int d_, int lane)
    {
        d = d_;
        nchunks = d_ / PC;
        g = lane % G;
        v = lane / G;
    }
    __device__ __forceinline__ bool has(int c) const { return g + G * c < nchunks; }

    // query given as fp32
    __device__ __forceinline__ void load_query_f32(const float* __restrict__ qrow)
    {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const int ci = g + G * c;
#pragma unroll
            for (int e = 0; e < PC; e += 4) {
                float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
                if (ci < nchunks) x = *reinterpret_cast<const float4*>(qrow + (size_t)ci * PC + e);
                q[c * PC + e + 0] = x.x;
                q[c * PC + e + 1] = x.y;
                q[c * PC + e + 2] = x.z;
                q[c * PC + e + 3] = x.w;
            }
        }
        pack_query();
    }
    // query is itself a base row (build passes)
    __device__ __forceinline__ void load_query_row(const T* __restrict__ base, uint32_t row)
    {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            chunk_t x = {};
            if (has(c)) x = load(base, row, c);
            unpack(x, &q[c * PC]);
        }
        pack_query();
    }

    // uint8 rows only: decide whether every query element is an integer in [0,255] (all lanes of
    // the wave vote, so the branch is uniform) and keep the packed bytes and their square sum
    __device__ __forceinline__ void pack_query()
    {
        q_int = false;
        qq = 0u;
        if constexpr (sizeof(T) == 1) {
            bool ok = true;
#pragma unroll
            for (int i = 0; i < C * PC; ++i) ok = ok && q[i] >= 0.f && q[i] <= 255.f && q[i] == rintf(q[i]);
            q_int = ballot64(!ok) == 0ull;
#pragma unroll
            for (int w = 0; w < C * 4; ++w) {
                uint32_t b = 0u;
#pragma unroll
                for (int e = 0; e < 4; ++e) b |= ((uint32_t)q[w * 4 + e] & 0xFFu) << (8 * e);
                qbytes[w] = b;
                qq = __builtin_amdgcn_udot4(b, b, qq, false);
            }
        }
    }

    __device__ __forceinline__ chunk_t load(const T* __restrict__ base, uint32_t row, int c) const
    {
        return *reinterpret_cast<const chunk_t*>(base + (size_t)row * (size_t)d + (size_t)(g + G * c) * PC);
    }

    static __device__ __forceinline__ void unpack(const chunk_t& x, float* out)
    {
        if constexpr (sizeof(T) == 4) {
            out[0] = x.x; out[1] = x.y; out[2] = x.z; out[3] = x.w;
        } else if constexpr (sizeof(T) == 2) {
            const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                out[2 * i + 0] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] & 0xFFFFu));
                out[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] >> 16));
            }
        } else {
            const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                out[4 * i + 0] = (float)(w[i] & 0xFFu);
                out[4 * i + 1] = (float)((w[i] >> 8) & 0xFFu);
                out[4 * i + 2] = (float)((w[i] >> 16) & 0xFFu);
                out[4 * i + 3] = (float)(w[i] >> 24);
            }
        }
    }

    // this lane's share of sum (q_j - x_j)^2 over its chunks
    template <bool FULL = false> __device__ __forceinline__ double partial(const chunk_t (&buf)[C]) const
    {
        double acc = 0.0;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            if (FULL || has(c)) {
                float x[PC];
                unpack(buf[c], x);
#pragma unroll
                for (int e = 0; e < PC; ++e) {
                    const float t = q[c * PC + e] - x[e];
                    acc += (double)t * (double)t;
                }
            }
        }
        return acc;
    }

    // The squared distance between the query and the row whose chunks are in buf, as the fp32
    // canonical value; every lane of the group gets it.  uint8 rows with an integer query take
    // the exact integer route sum q^2 + sum x^2 - 2 sum q x on v_dot4_u32_u8 (8 instructions per
    // 16 elements): the integer total converts to the same fp32 as the fp64 sum of squares.
    // FULL: the row fills all G*C chunks (d = G*C*PC), so no lane has a chunk to skip.
    template <bool FULL = false> __device__ __forceinline__ float distance(const chunk_t (&buf)[C]) const
    {
        if constexpr (sizeof(T) == 1) {
            if (q_int) {
                uint32_t xx = 0u, qx = 0u;
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    if (FULL || has(c)) {
                        const uint32_t w[4] = {buf[c].x, buf[c].y, buf[c].z, buf[c].w};
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            xx = __builtin_amdgcn_udot4(w[i], w[i], xx, false);
                            qx = __builtin_amdgcn_udot4(qbytes[c * 4 + i], w[i], qx, false);
                        }
                    }
                }
                // this lane's share of sum (q-x)^2 (non-negative).  qq is the lane's sum of q^2 kept since
                // pack_query: slices of chunks the lane does not own are zero there, as they are in xx and qx
                const uint32_t part = xx - 2u * qx + qq;
                return (float)group_sum_u32(part);
            }
        }
        return (float)group_sum(partial<FULL>(buf));
    }

    // uint8 rows, q_int set: the integer route alone.  A kernel that calls this and distance_from
    // (never distance) keeps no fp32 copy of the query in registers.
    template <bool FULL = false> __device__ __forceinline__ float distance_int(const chunk_t (&buf)[C]) const
    {
        static_assert(sizeof(T) == 1, "integer route: uint8 rows only");
        uint32_t xx = 0u, qx = 0u;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            if (FULL || has(c)) {
                const uint32_t w[4] = {buf[c].x, buf[c].y, buf[c].z, buf[c].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    xx = __builtin_amdgcn_udot4(w[i], w[i], xx, false);
                    qx = __builtin_amdgcn_udot4(qbytes[c * 4 + i], w[i], qx, false);
                }
            }
        }
        return (float)group_sum_u32(xx - 2u * qx + qq);
    }
    // uint8 rows, any query: the fp64 route with the query read from LDS at every use (qrow = the whole fp32
    // query row, 16-byte aligned), four elements at a time in the element order of partial(): the same value,
    // and no fp32 copy of the query held in registers.  The empty asm makes the address new at every use, so
    // each read stays where it is written, one group of four in flight: this route is about registers, not speed.
    template <bool FULL = false>
    __device__ __forceinline__ float distance_from(const chunk_t (&buf)[C], const float* qrow) const
    {
        static_assert(sizeof(T) == 1, "uint8 rows only");
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        typedef const f32x4 __attribute__((address_space(3)))* lds_f32x4_ptr;
        double acc = 0.0;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            if (FULL || has(c)) {
                const uint32_t w[4] = {buf[c].x, buf[c].y, buf[c].z, buf[c].w};
                lds_f32x4_ptr qc = (lds_f32x4_ptr)(qrow + (g + G * c) * PC);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    asm volatile("" : "+v"(qc));
                    const f32x4 qv = qc[i];
                    const float t0 = qv.x - (float)(w[i] & 0xFFu);
                    const float t1 = qv.y - (float)((w[i] >> 8) & 0xFFu);
                    const float t2 = qv.z - (float)((w[i] >> 16) & 0xFFu);
                    const float t3 = qv.w - (float)(w[i] >> 24);
                    acc += (double)t0 * (double)t0;
                    acc += (double)t1 * (double)t1;
                    acc += (double)t2 * (double)t2;
                    acc += (double)t3 * (double)t3;
                }
            }
        }
        return (float)group_sum(acc);
    }
    // One call for kernels that keep a copy of the query in LDS (qs): byte rows take the integer route for an
    // integer-valued query and the fp64 route reading qs otherwise, so their fp32 query leaves the registers
    // after pack_query; other rows are scored from the registers as ever.
    template <bool FULL = false>
    __device__ __forceinline__ float distance_lds(const chunk_t (&buf)[C], const float* qs) const
    {
        if constexpr (sizeof(T) == 1)
            return q_int ? distance_int<FULL>(buf) : distance_from<FULL>(buf, qs);
        else
            return distance<FULL>(buf);
    }
    // stores this lane's slices of the query at their places in qrow (call from one group of lanes)
    __device__ __forceinline__ void store_query(float* qrow) const
    {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            if (has(c)) {
#pragma unroll
                for (int e = 0; e < PC; e += 4)
                    *reinterpret_cast<float4*>(qrow + (g + G * c) * PC + e) =
                        make_float4(q[c * PC + e], q[c * PC + e + 1], q[c * PC + e + 2], q[c * PC + e + 3]);
            }
        }
    }

    static __device__ __forceinline__ uint32_t group_sum_u32(uint32_t a)
    {
        a += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0xB1, 0xF, 0xF, false);
        a += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0x4E, 0xF, 0xF, false);
        if constexpr (G >= 8) a += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0x141, 0xF, 0xF, false);
        if constexpr (G >= 16) a += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0x140, 0xF, 0xF, false);
        if constexpr (G >= 32) a += (uint32_t)__shfl_xor((int)a, 16, 64);
        if constexpr (G >= 64) a += (uint32_t)__shfl_xor((int)a, 32, 64);
        return a;
    }

    // sum over the G lanes of a group; every lane of the group gets the total.  Butterfly over
    // lane pairs 1, 2 apart (quad permutes), then the mirrored lane of the 8- and 16-lane row
    // (which already holds the other half's total), then xor 16 / 32 through the LDS crossbar.
    static __device__ __forceinline__ double group_sum(double a)
    {
        a += dpp_f64<0xB1>(a);                     // quad_perm [1,0,3,2]
        a += dpp_f64<0x4E>(a);                     // quad_perm [2,3,0,1]
        if constexpr (G >= 8) a += dpp_f64<0x141>(a);   // row_half_mirror
        if constexpr (G >= 16) a += dpp_f64<0x140>(a);  // row_mirror
        if constexpr (G >= 32) a += shfl_xor_f64(a, 16);
        if constexpr (G >= 64) a += shfl_xor_f64(a, 32);
        return a;
    }
};

// (G, C) for a row of `nchunks` 16-byte chunks: the smallest group that covers the
// row with at most 4 chunks per lane (8 for the longest rows).
inline bool pick_group(int nchunks, int* G, int* C)
{
    static const int gs[] = {8, 8, 8, 8, 16, 32, 64, 64};
    static const int cs[] = {1, 2, 3, 4, 4, 4, 4, 8};
    for (int i = 0; i < 8; ++i)
        if (nchunks <= gs[i] * cs[i]) {
            *G = gs[i];
            *C = cs[i];
            return true;
        }
    return false;
}

// Calls f.template operator()<T, G, C>() for the (dtype, d) at hand.
template <typename F> inline bool dispatch_row_shape(ann_dtype dtype, int d, F&& f)
{
    const int pc = dtype == ANN_U8 ? 16 : 4;
    if (d <= 0 || d % pc != 0) return false;
    int G, C;
    if (!pick_group(d / pc, &G, &C)) return false;
#define TSDG_CASE(TT, GG, CC) \
    if (G == GG && C == CC) { f.template operator()<TT, GG, CC>(); return true; }
    if (dtype == ANN_F32) {
        TSDG_CASE(float, 8, 1) TSDG_CASE(float, 8, 2) TSDG_CASE(float, 8, 3) TSDG_CASE(float, 8, 4)
        TSDG_CASE(float, 16, 4) TSDG_CASE(float, 32, 4) TSDG_CASE(float, 64, 4) TSDG_CASE(float, 64, 8)
    } else {
        TSDG_CASE(uint8_t, 8, 1) TSDG_CASE(uint8_t, 8, 2) TSDG_CASE(uint8_t, 8, 3) TSDG_CASE(uint8_t, 8, 4)
        TSDG_CASE(uint8_t, 16, 4)
    }
#undef TSDG_CASE
    return false;
}

// The search entry points also take rows stored as binary16 (8 elements per chunk); the build
// kernels do not, so they keep dispatch_row_shape.
template <typename F> inline bool dispatch_search_row_shape(ann_dtype dtype, int d, F&& f)
{
    if (dtype != ANN_F16) return dispatch_row_shape(dtype, d, f);
    if (d <= 0 || d % 8 != 0) return false;
    int G, C;
    if (!pick_group(d / 8, &G, &C)) return false;
#define TSDG_CASE(GG, CC) \
    if (G == GG && C == CC) { f.template operator()<_Float16, GG, CC>(); return true; }
    TSDG_CASE(8, 1) TSDG_CASE(8, 2) TSDG_CASE(8, 3) TSDG_CASE(8, 4) TSDG_CASE(16, 4) TSDG_CASE(32, 4) TSDG_CASE(64, 4)
#undef TSDG_CASE
    return false;
}

}  // namespace tsdg
