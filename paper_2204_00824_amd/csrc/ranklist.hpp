// The bounded sorted rank-list of the best-first search (steps S2 and S6) and the
// hashed visited set (S4), both in LDS and operated by ONE wavefront.
//
// The list holds L 64-bit keys in ascending order (common.hpp: make_key); unused
// slots hold kKeyEmpty, which sorts last.  Bit 0 of a key is the "expanded" flag;
// comparisons that must ignore it compare (key | 1).
#pragma once
#include "common.hpp"

namespace tsdg {

// S2: index of the first entry not yet expanded, or -1.  All 64 lanes call.
__device__ __forceinline__ int list_first_unexpanded(const uint64_t* list, int L, int lane)
{
    for (int i0 = 0; i0 < L; i0 += 64) {
        const int i = i0 + lane;
        const uint64_t a = i < L ? list[i] : kKeyEmpty;
        const uint64_t m = ballot64(a != kKeyEmpty && (a & 1ull) == 0ull);
        if (m) return i0 + ctz64(m);
        if (ballot64(a == kKeyEmpty)) return -1;  // reached the unused tail
    }
    return -1;
}

// S6: merges up to 64 scored candidates (one per lane, kKeyEmpty = none; ids
// distinct among the lanes) into the list, keeping the L smallest.  A candidate
// whose id is already in the list (same distance, same id) is dropped.
// Positions: with r_j = #{a in list : a < c_j} and t_j = #{c_i < c_j}, candidate
// j lands at r_j + t_j and list entry i at i + #{j : r_j <= i}; together these
// are the positions of the merged sequence, and everything at L or beyond falls
// off.  `sync` must order LDS accesses among the calling lanes.
template <typename Sync>
__device__ __forceinline__ void list_merge(uint64_t* list, int L, uint64_t key, int lane, Sync sync)
{
    const uint64_t worst = list[L - 1] | 1ull;
    bool valid = (key | 1ull) < worst;
    if (!ballot64(valid)) return;

    int r = 0;
    if (valid) {
        int lo = 0, hi = L;
        const uint64_t kk = key | 1ull;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if ((list[mid] | 1ull) < kk) lo = mid + 1; else hi = mid;
        }
        r = lo;
        if (r < L && (list[r] | 1ull) == kk) valid = false;  // already present
    }
    const uint64_t vm = ballot64(valid);
    if (!vm) return;

    int t = 0;
    for (uint64_t m = vm; m; m &= m - 1) {
        const int j = ctz64(m);
        const uint64_t kj = bcast64(key, j);
        t += (kj < key || (kj == key && j < lane)) ? 1 : 0;
    }

    // move list entries, highest block first (entries only move towards the end)
    for (int i0 = ((L - 1) / 64) * 64; i0 >= 0; i0 -= 64) {
        const int i = i0 + lane;
        const uint64_t a = i < L ? list[i] : kKeyEmpty;
        int u = 0;
        for (uint64_t m = vm; m; m &= m - 1) {
            const int j = ctz64(m);
            const int rj = (int)bcast32((uint32_t)r, j);
            u += (rj <= i) ? 1 : 0;
        }
        sync();
        if (i < L && u > 0 && i + u < L) list[i + u] = a;
        sync();
    }
    if (valid && r + t < L) list[r + t] = key;
    sync();
}

// S4: insert-if-absent into an open-addressed table of `slots` (power of two)
// 32-bit ids.  Returns true when the id was already there.  After kProbes full
// slots the home slot is overwritten: the set then forgets an id (a later visit
// re-scores it, which the merge's duplicate rule makes harmless) but never
// reports an id it has not seen.
constexpr int kProbes = 4;
__device__ __forceinline__ uint32_t hash_id(uint32_t id)
{
    uint32_t h = id * 0x9E3779B1u;
    return h ^ (h >> 15);
}
__device__ __forceinline__ bool visited_test_and_set(uint32_t* table, int slots, uint32_t id)
{
    const uint32_t mask = (uint32_t)slots - 1u;
    const uint32_t h = hash_id(id) & mask;
    for (int p = 0; p < kProbes; ++p) {
        const uint32_t old = atomicCAS(&table[(h + p) & mask], kHashEmpty, id);
        if (old == kHashEmpty) return false;
        if (old == id) return true;
    }
    table[h] = id;
    return false;
}

}  // namespace tsdg
