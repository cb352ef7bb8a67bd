// The bounded sorted rank-list of the best-first search (steps S2 and S6) and the
// hashed visited set (S4), both in LDS and operated by ONE wavefront.
//
// The list holds L 64-bit keys in ascending order (common.hpp: make_key); unused
// slots hold kKeyEmpty, which sorts last.  Bit 0 of a key is the "expanded" flag;
// comparisons that must ignore it compare (key | 1).
#pragma once
#include "common.hpp"

namespace tsdg {

// S2: index of the first entry not yet expanded, or -1; *key_out receives that entry.  All 64
// lanes call.
__device__ __forceinline__ int list_first_unexpanded(const uint64_t* list, int L, int lane, uint64_t* key_out)
{
    if (L <= 64) {  // one entry per lane
        const uint64_t a = lane < L ? list[lane] : kKeyEmpty;
        const uint64_t m = ballot64(a != kKeyEmpty && (a & 1ull) == 0ull);
        if (!m) return -1;
        const int b = ctz64(m);
        *key_out = readlane64(a, b);
        return b;
    }
    for (int i0 = 0; i0 < L; i0 += 64) {
        const int i = i0 + lane;
        const uint64_t a = i < L ? list[i] : kKeyEmpty;
        const uint64_t m = ballot64(a != kKeyEmpty && (a & 1ull) == 0ull);
        if (m) {
            const int b = ctz64(m);
            *key_out = readlane64(a, b);
            return i0 + b;
        }
        if (ballot64(a == kKeyEmpty)) return -1;  // reached the unused tail
    }
    return -1;
}

// S6: merges up to 64 scored candidates (one per lane, kKeyEmpty = none; ids distinct among
// the lanes) into the list, keeping the L smallest.  A candidate whose id is already in the
// list (same distance, same id) is dropped.
// Positions: with r_j = #{a in list : a < c_j} and t_j = #{c_i < c_j}, candidate j lands at
// r_j + t_j and list entry i at i + #{j : r_j <= i}; together these are the positions of the
// merged sequence, and everything at L or beyond falls off.  Lists of up to 128 entries sit in
// registers (one or two entries per lane) while the candidates are broadcast one at a time with
// v_readlane, so that a rank is one ballot + popcount; longer lists are searched in LDS (a
// binary search per candidate, all candidates at once) and moved block by block from the end.
// `sync` must order LDS accesses among the calling lanes.
// DISTINCT = false: the lanes may hold the same candidate more than once; only the first lane's
// copy is merged (costs one more pass over the candidates).
// The single-pass merge of list_merge (see there) for lists of at most 64 * B entries, B entries per
// lane; returns false (list untouched) when some candidate is already in the list.
template <int B, typename Sync>
__device__ __forceinline__ bool merge_single_pass(uint64_t* list, int L, uint64_t key, uint64_t kk, bool valid,
                                                  uint64_t vm, int lane, Sync sync)
{
    uint64_t a[B], am1[B];
    int above[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        const int i = b * 64 + lane;
        a[b] = i < L ? list[i] : kKeyEmpty;
        am1[b] = a[b] | 1ull;
        above[b] = 0;
    }
    int pos = 0, n = 0;
    bool present = false;
    for (uint64_t m = vm; m; m &= m - 1) {
        const int j = ctz64(m);
        const uint64_t kj = readlane64(kk, j);
        int below = popc64(ballot64(valid && kk < kj));
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const bool lt = am1[b] < kj;
            below += popc64(ballot64(lt));
            present = present || ballot64(am1[b] == kj) != 0ull;
            above[b] += lt ? 1 : 0;
        }
        pos = lane == j ? below : pos;
        ++n;
    }
    if (present) return false;
    sync();
#pragma unroll
    for (int b = 0; b < B; ++b) {
        const int i = b * 64 + lane;
        const int u = n - above[b];
        if (i < L && u > 0 && i + u < L) list[i + u] = a[b];
    }
    if (valid && pos < L) list[pos] = key;
    sync();
    return true;
}

template <bool DISTINCT = true, typename Sync>
__device__ __forceinline__ void list_merge(uint64_t* list, int L, uint64_t key, int lane, Sync sync)
{
    const uint64_t worst = list[L - 1] | 1ull;
    const uint64_t kk = key | 1ull;
    bool valid = kk < worst;
    uint64_t vm = ballot64(valid);
    if (!vm) return;
    if constexpr (!DISTINCT) {
        bool again = false;
        for (uint64_t m = vm; m; m &= m - 1) {
            const int j = ctz64(m);
            again = again || (j < lane && readlane64(kk, j) == kk);
        }
        valid = valid && !again;
        vm = ballot64(valid);
    }

    // Short lists: a single pass over the candidates yields everything.  Candidate j is broadcast;
    // the list entries below it give r_j, the candidates below it give t_j (lane j keeps their sum,
    // its position in the merged list), and every lane counts the candidates above each of its own
    // entries (one per block of 64), which leaves u = (candidates) - (that count) places to move up.
    // A candidate already in the list is rare and sends the call down the general path below,
    // which has touched nothing yet.
    if (L <= 64) {
        const uint64_t a = lane < L ? list[lane] : kKeyEmpty;
        const uint64_t am1 = a | 1ull;
        int pos = 0, above = 0, n = 0;
        bool present = false;
        for (uint64_t m = vm; m; m &= m - 1) {
            const int j = ctz64(m);
            const uint64_t kj = readlane64(kk, j);
            const bool lt = am1 < kj;
            const uint64_t lt_m = ballot64(lt);
            present = present || ballot64(am1 == kj) != 0ull;
            const uint64_t tb_m = ballot64(valid && kk < kj);
            above += lt ? 1 : 0;
            pos = lane == j ? popc64(lt_m) + popc64(tb_m) : pos;
            ++n;
        }
        if (!present) {
            const int u = n - above;
            sync();
            if (lane < L && u > 0 && lane + u < L) list[lane + u] = a;
            if (valid && pos < L) list[pos] = key;
            sync();
            return;
        }
    } else if (L <= 128) {  // the same with two entries per lane
        if (merge_single_pass<2>(list, L, key, kk, valid, vm, lane, sync)) return;
    }

    // Longer lists.  r_j by a binary search of the list (one LDS read per step, all candidates at once);
    // a candidate that meets its own key there is already present.
    const int top = ((L - 1) / 64) * 64;
    int r = 0;
    bool dup = false;
    {
        int lo = 0, hi = L;
        const int steps = 32 - __builtin_clz((unsigned)L);  // 2^steps > L
        for (int step = 0; step < steps; ++step) {
            const int mid = (lo + hi) >> 1;
            const bool open = lo < hi;
            const bool below = (list[min(mid, L - 1)] | 1ull) < kk;
            lo = open && below ? mid + 1 : lo;
            hi = open && !below ? mid : hi;
        }
        r = lo;
        dup = r < L && (list[min(r, L - 1)] | 1ull) == kk;
    }
    valid = valid && !dup;  // already present
    vm = ballot64(valid);
    if (!vm) return;

    int t = 0, rmin = L;
    for (uint64_t m = vm; m; m &= m - 1) {
        const int j = ctz64(m);
        const uint64_t kj = readlane64(key, j);
        t += (kj < key || (kj == key && j < lane)) ? 1 : 0;
        rmin = min(rmin, (int)readlane32((uint32_t)r, j));
    }

    // move list entries, highest block first (entries only move towards the end); blocks that
    // lie wholly before the smallest insertion point stay
    for (int i0 = top; i0 >= (rmin & ~63); i0 -= 64) {
        const int i = i0 + lane;
        const uint64_t a = i < L ? list[i] : kKeyEmpty;
        // candidates that land before this block all count; those inside it are compared one by one
        int u = popc64(ballot64(valid && r < i0));
        for (uint64_t m = ballot64(valid && r >= i0 && r < i0 + 64); m; m &= m - 1)
            u += ((int)readlane32((uint32_t)r, ctz64(m)) <= i) ? 1 : 0;
        sync();
        if (i < L && u > 0 && i + u < L) list[i + u] = a;
        sync();
    }
    if (valid && r + t < L) list[r + t] = key;
    sync();
}

// ---- The same list held in registers: lane i of the wave holds entry i (and entry 64 + i when B = 2), so lists of
// up to 64 * B entries never touch LDS: the pick is a ballot, an insertion shifts the tail up by one lane with a
// whole-wave DPP shift.  Lanes at L and beyond hold anything and are masked out of every vote.
__device__ __forceinline__ uint64_t wave_shr1_u64(uint64_t v)
{
    const int lo = __builtin_amdgcn_update_dpp((int)(uint32_t)v, (int)(uint32_t)v, 0x138, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp((int)(uint32_t)(v >> 32), (int)(uint32_t)(v >> 32), 0x138, 0xF, 0xF, false);
    return ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo;   // lane l receives lane l-1's value; lane 0 keeps its own
}

template <int B> struct RegList {
    static_assert(B == 1 || B == 2, "one or two entries per lane");
    uint64_t e[B];    // e[b] of lane l = entry 64 b + l
    uint64_t top;     // lanes of the last register that hold entries
    int L;

    __device__ __forceinline__ void init(int L_)
    {
        L = L_;
        const int n = L_ - 64 * (B - 1);               // entries in the last register: 1..64
        top = n >= 64 ? ~0ull : (1ull << n) - 1ull;
#pragma unroll
        for (int b = 0; b < B; ++b) e[b] = kKeyEmpty;
    }
    __device__ __forceinline__ uint64_t valid(int b) const { return b == B - 1 ? top : ~0ull; }

    // S2: index of the first entry not yet expanded, or -1; *key_out receives it.
    __device__ __forceinline__ int first_unexpanded(uint64_t* key_out) const
    {
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const uint64_t m = ballot64(e[b] != kKeyEmpty && (e[b] & 1ull) == 0ull) & valid(b);
            if (m) {
                const int l = ctz64(m);
                *key_out = readlane64(e[b], l);
                return 64 * b + l;
            }
        }
        return -1;
    }
    __device__ __forceinline__ void mark_expanded(int idx, int lane)
    {
#pragma unroll
        for (int b = 0; b < B; ++b) e[b] |= (64 * b + lane == idx) ? 1ull : 0ull;
    }
    // entry t (t = 64 b + lane for the calling lane)
    __device__ __forceinline__ uint64_t entry(int t) const { return B == 2 && t >= 64 ? e[B - 1] : e[0]; }

    // S6: the candidates (one per lane, kKeyEmpty = none, ids distinct among the lanes) go in one after the
    // other, each at p = #{entries below it}; entries from p on move up one place (lane 63 of the first
    // register hands its entry to lane 0 of the second) and the last falls off.  A candidate that is not below
    // the current last entry, or already listed, changes nothing.  The result is the merged list that
    // list_merge produces: the L smallest of the union, in order.
    __device__ __forceinline__ void merge(uint64_t key, int lane)
    {
        const uint64_t kk = key | 1ull;
        const uint64_t worst = readlane64(e[B - 1], L - 64 * (B - 1) - 1) | 1ull;
        for (uint64_t vm = ballot64(kk < worst); vm; vm &= vm - 1) {
            const uint64_t kj = readlane64(kk, ctz64(vm));
            uint64_t same = 0ull;
            int p = 0;                                   // the entries below kj are a prefix: the list is in order
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const uint64_t am1 = e[b] | 1ull;
                p += popc64(ballot64(am1 < kj) & valid(b));
                same |= ballot64(am1 == kj) & valid(b);
            }
            if (same) continue;                          // already listed
            const uint64_t in = kj & ~1ull;
            if constexpr (B == 1) {
                const uint64_t up = wave_shr1_u64(e[0]);
                e[0] = lane > p ? up : (lane == p ? in : e[0]);
            } else {
                const uint64_t up1 = wave_shr1_u64(e[1]);
                if (p < 64) {
                    const uint64_t carry = readlane64(e[0], 63);
                    const uint64_t up0 = wave_shr1_u64(e[0]);
                    e[0] = lane > p ? up0 : (lane == p ? in : e[0]);
                    e[1] = lane == 0 ? carry : up1;
                } else {
                    const int q = p - 64;
                    e[1] = lane > q ? up1 : (lane == q ? in : e[1]);
                }
            }
        }
    }
};

// S4: insert-if-absent into an open-addressed table of `slots` 32-bit ids (any size: the home
// slot is the high half of hash x slots, and probing wraps round).  Returns true when the id was already there.  After kProbes full
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
    const uint32_t h = __umulhi(hash_id(id), (uint32_t)slots);   // any table size, not only powers of two
    for (int p = 0; p < kProbes; ++p) {
        uint32_t j = h + (uint32_t)p;
        j = j >= (uint32_t)slots ? j - (uint32_t)slots : j;
        const uint32_t old = atomicCAS(&table[j], kHashEmpty, id);
        if (old == kHashEmpty) return false;
        if (old == id) return true;
    }
    table[h] = id;
    return false;
}

}  // namespace tsdg
