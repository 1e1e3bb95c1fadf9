// Wavefront-level building blocks (gfx950, wave64): key packing, a register bitonic sort
// over 64*E keys, and the "first R distinct keys" selection that every merge step uses.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned long long u64;
typedef uint32_t u32;

#define KEY_PAD 0xFFFFFFFFFFFFFFFFull   // sorts after every real key

// (dist_bits << 32) | (id << 1) | is_new : ascending key order is ascending (delta, id), and of two
// entries for the same edge the "old" one comes first.
__device__ __forceinline__ u64 make_key(u32 dist_bits, u32 id, u32 is_new)
{
    return ((u64)dist_bits << 32) | ((u64)id << 1) | (u64)is_new;
}
__device__ __forceinline__ u32 key_id(u64 k) { return (u32)(k >> 1) & 0x7FFFFFFFu; }
__device__ __forceinline__ u32 key_dist(u64 k) { return (u32)(k >> 32); }

// Orders LDS traffic between lanes of one wavefront.  A wavefront executes its LDS
// instructions in program order, so only the compiler has to be kept from moving them.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ u64 lanes_below(int lane) { return lane == 0 ? 0ull : (~0ull >> (64 - lane)); }

__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int m)
{
    u32 lo = (u32)v, hi = (u32)(v >> 32);
    lo = __shfl_xor(lo, m);
    hi = __shfl_xor(hi, m);
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 shfl_u64(u64 v, int src)
{
    u32 lo = (u32)v, hi = (u32)(v >> 32);
    lo = __shfl(lo, src);
    hi = __shfl(hi, src);
    return ((u64)hi << 32) | lo;
}
// value of lane l - 1 (lane 0: its own): a wavefront-wide DPP shift, no LDS round trip
__device__ __forceinline__ u64 shfl_up1_u64(u64 v)
{
    u32 lo = (u32)v, hi = (u32)(v >> 32);
    lo = (u32)__builtin_amdgcn_update_dpp((int)lo, (int)lo, 0x138, 0xF, 0xF, false);     // wave_shr:1
    hi = (u32)__builtin_amdgcn_update_dpp((int)hi, (int)hi, 0x138, 0xF, 0xF, false);
    return ((u64)hi << 32) | lo;
}

// Value of lane (l xor S), S a power of two below 64.  Within rows of 16 lanes the exchange is a
// DPP move (no LDS round trip) where the ISA has one: quad permutations for S = 1, 2 and a rotation
// by 8 for S = 8; S = 4 and 16 use the LDS swizzle unit, S = 32 the permute unit.  Every lane of these
// DPP patterns has a source lane, so bound_ctrl changes no value: it only tells the compiler that the
// destination needs no initial value (two moves less per 64-bit exchange).
template <int S>
__device__ __forceinline__ u32 xor_lane_u32(u32 v)
{
    if constexpr (S == 1) return (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);        // quad_perm [1,0,3,2]
    else if constexpr (S == 2) return (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
    else if constexpr (S == 8) return (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x128, 0xF, 0xF, true);  // row_ror:8
    else if constexpr (S == 4) return (u32)__builtin_amdgcn_ds_swizzle((int)v, 0x101F);                     // xor 4, and 0x1F
    else if constexpr (S == 16) return (u32)__builtin_amdgcn_ds_swizzle((int)v, 0x401F);                    // xor 16, and 0x1F
    else return (u32)__shfl_xor((int)v, S);
}

__device__ __forceinline__ u64 xor_lane_u64(u64 v, int stride)
{
    u32 lo = (u32)v, hi = (u32)(v >> 32);
    switch (stride) {   // constant after unrolling
    case 1: lo = xor_lane_u32<1>(lo); hi = xor_lane_u32<1>(hi); break;
    case 2: lo = xor_lane_u32<2>(lo); hi = xor_lane_u32<2>(hi); break;
    case 4: lo = xor_lane_u32<4>(lo); hi = xor_lane_u32<4>(hi); break;
    case 8: lo = xor_lane_u32<8>(lo); hi = xor_lane_u32<8>(hi); break;
    case 16: lo = xor_lane_u32<16>(lo); hi = xor_lane_u32<16>(hi); break;
    default: lo = xor_lane_u32<32>(lo); hi = xor_lane_u32<32>(hi); break;
    }
    return ((u64)hi << 32) | lo;
}

// One compare-exchange of a bitonic network from the point of view of one side: keeps the smaller
// of (mine, other) if take_min, else the larger.
__device__ __forceinline__ u64 keep_of_pair(u64 mine, u64 other, bool take_min)
{
    return ((mine < other) == take_min) ? mine : other;
}

// Ascending bitonic sort of 64*E keys held as k[r] in lane l  <->  element index r*64 + l.
template <int E>
__device__ __forceinline__ void wave_sort(u64 (&k)[E], int lane)
{
#pragma unroll
    for (int size = 2; size <= 64 * E; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            if (stride >= 64) {
                const int rs = stride / 64;
#pragma unroll
                for (int r = 0; r < E; ++r) {
                    if ((r & rs) == 0) {
                        const bool up = (((r * 64) & size) == 0);
                        const u64 a = k[r], b = k[r | rs];
                        const bool swap = (b < a) == up;      // up: smaller first
                        k[r] = swap ? b : a;
                        k[r | rs] = swap ? a : b;
                    }
                }
            } else {
#pragma unroll
                for (int r = 0; r < E; ++r) {
                    const bool up = ((((r * 64) + lane) & size) == 0);
                    const bool lower = (lane & stride) == 0;
                    k[r] = keep_of_pair(k[r], xor_lane_u64(k[r], stride), lower == up);
                }
            }
        }
    }
}

// Ascending bitonic sort inside every group of G consecutive lanes (G = 16, 32 or 64), one key per lane.
template <int G>
__device__ __forceinline__ u64 group_sort(u64 k, int lane)
{
    const int sub = lane & (G - 1);
#pragma unroll
    for (int size = 2; size <= G; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            const bool up = (sub & size) == 0;      // for size == G: always ascending
            const bool lower = (lane & stride) == 0;
            k = keep_of_pair(k, xor_lane_u64(k, stride), lower == up);
        }
    }
    return k;
}

// k[] sorted ascending.  Drops KEY_PAD and every key equal (ignoring the flag bit) to its
// predecessor, and writes the first `cap` survivors, in order, to out[0..) (LDS or global).
// Returns how many were written; *any_new is set if one of them has the flag bit.
// *dropped (may be null) grows by the number of survivors beyond `cap`.
template <int E>
__device__ __forceinline__ int wave_unique_prefix(const u64 (&k)[E], int lane, int cap, u64 *out,
                                                 bool *any_new, int *dropped = nullptr)
{
    int base = 0;
    u64 newacc = 0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
        u64 prev = shfl_up1_u64(k[r]);
        if (lane == 0) prev = KEY_PAD;
        if (r > 0) {
            u64 last = shfl_u64(k[r - 1], 63);
            if (lane == 0) prev = last;
        }
        bool keep = (k[r] != KEY_PAD) && ((k[r] >> 1) != (prev >> 1));
        u64 m = __builtin_amdgcn_ballot_w64(keep);
        int pos = base + __popcll(m & lanes_below(lane));
        bool w = keep && pos < cap;
        if (w) out[pos] = k[r];
        newacc |= __builtin_amdgcn_ballot_w64(w && (k[r] & 1ull));
        base += __popcll(m);
    }
    *any_new = newacc != 0;
    if (dropped && base > cap) *dropped += base - cap;
    return base < cap ? base : cap;
}

// Row `row` (nb keys, ascending) merged with c = ca + cb keys in any order (the first ca at binA, the
// rest at binB): the first R distinct keys of the union, ascending, are written back to row[0..);
// returns the new length.  `stage` is 128 keys of LDS private to this wavefront.
// *dropped (may be null) grows by the number of distinct keys that did not fit (in the streaming case an edge that
// arrives in two different chunks after it was dropped counts twice).
__device__ __forceinline__ int wave_merge_row(u64 *row, int nb, const u64 *binA, int ca, const u64 *binB,
                                              int cb, int R, u64 *stage, int lane, bool *any_new, int *dropped = nullptr)
{
    const int c = ca + cb;
    const int total = nb + c;
    auto bin_at = [&](int e) -> u64 { return e < ca ? binA[e] : binB[e - ca]; };
    int n;
    if (total <= 64) {
        u64 k[1];
        k[0] = lane < nb ? row[lane] : (lane < total ? bin_at(lane - nb) : KEY_PAD);
        wave_sort<1>(k, lane);
        n = wave_unique_prefix<1>(k, lane, R, row, any_new, dropped);
    } else if (total <= 128) {
        u64 k[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            int e = r * 64 + lane;
            k[r] = e < nb ? row[e] : (e < total ? bin_at(e - nb) : KEY_PAD);
        }
        wave_sort<2>(k, lane);
        n = wave_unique_prefix<2>(k, lane, R, row, any_new, dropped);
    } else {
        // stream the bin through in chunks of 128 against the best R found so far
        u64 k[4];
        k[0] = lane < nb ? row[lane] : KEY_PAD;
        k[1] = lane + 64 < nb ? row[lane + 64] : KEY_PAD;
        n = nb;
        for (int done = 0; done < c; done += 128) {
            int e0 = done + lane, e1 = done + 64 + lane;
            k[2] = e0 < c ? bin_at(e0) : KEY_PAD;
            k[3] = e1 < c ? bin_at(e1) : KEY_PAD;
            wave_sort<4>(k, lane);
            n = wave_unique_prefix<4>(k, lane, R, stage, any_new, dropped);
            wave_sync();
            k[0] = lane < n ? stage[lane] : KEY_PAD;
            k[1] = lane + 64 < n ? stage[lane + 64] : KEY_PAD;
            wave_sync();
        }
        if (lane < n) row[lane] = k[0];
        if (lane + 64 < n) row[lane + 64] = k[1];
    }
    return n;
}
