// Graph search (Alg. 1) with the out-degree cap K of Eq. 4, one wavefront per query.
//
// The candidate list C (at most L <= 128 points, ascending by (delta, id)) lives in registers, one or
// two keys per lane: key = (delta bits << 32) | (id << 1) | unvisited.  One step of the loop:
//   select     first unvisited member u of C (ballot), marked visited;
//   expand     its first min(deg(u), K) neighbours (rows are nearest-first), 64 per pass;
//   visited?   a neighbour already evaluated for this query is skipped: one bit per vertex in a bitmap
//              that the wavefront owns, tested and set by a single atomic OR;
//   evaluate   delta(q, v) for the rest, 8 vertices at a time (8 lanes per vertex);
//   insert     C <- the L smallest of C and the new points: the new keys are sorted, reversed, and merged
//              into C by a bitonic merge whose upper half is never formed; keys not below C's last one
//              are dropped first when C is full, and the merge is skipped when none is left.
// The loop ends when C holds no unvisited point (the loop's exit).  InitializeCandidates is
// min(L, N) distinct seeded random vertices from the same counter-based generator as RandomGraph,
// keyed by the query index.  Inserting the new points one by one, as the algorithm is written, and
// merging them at once give the same C, because each keeps the L smallest of what has been seen.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dist.h"
#include "wave_prims.h"

#define SEARCH_MAX_L 128

// S distinct ids != u in [0, n) from draw(seed, u, j), j = 0, 1, ...: draws are examined 64 at a time; a
// draw is accepted iff its id differs from every earlier draw's id, which is the same set, in the same
// order, as accepting one by one.  ids[] is LDS private to the wavefront (at least S entries).
__device__ __forceinline__ u64 splitmix_finish(u64 z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

// Does `id` equal the value some rotation R in [FIRST, END) of `src` within rows of 16 lanes brings to this lane,
// counting only rotations R <= limit (rotation R brings lane (l - R) mod 16: with limit = l the earlier lanes of the row)?
template <int R, int END>
__device__ __forceinline__ bool rotations_match(int id, int src, int limit)
{
    if constexpr (R >= END) {
        return false;
    } else {
        int o = src;
        if constexpr (R > 0) o = __builtin_amdgcn_update_dpp(0, src, 0x120 + R, 0xF, 0xF, true);      // row_ror:R
        // no short-circuit: every lane must take part in every rotation
        const bool here = (o == id) & (R <= limit);
        const bool rest = rotations_match<R + 1, END>(id, src, limit);
        return here | rest;
    }
}

__device__ __forceinline__ void wave_random_ids(u64 seed, long long n, long long u, int S, int *ids, int lane)
{
    const u64 G = 0x9E3779B97F4A7C15ull;
    const u64 hu = splitmix_finish(seed + G * (u64)(u + 1));
    const u64 jmax = 64ull * (u64)S + 1024ull;
    int cnt = 0;
    for (u64 j0 = 0; j0 < jmax && cnt < S;) {
        // examine the next W draws (a few more than still needed; any W gives the same result)
        const int W = (S - cnt) + 12 < 64 ? (S - cnt) + 12 : 64;
        const u64 j = j0 + lane;
        const u64 z = splitmix_finish(hu + G * (j + 1));
        const u64 c = ((z >> 32) * (u64)(n - 1)) >> 32;
        const int id = (int)(c + (c >= (u64)u ? 1 : 0));
        bool ok = lane < W && j < jmax;
        for (int k = 0; k < cnt; ++k) ok = ok && (ids[k] != id);
        if (W <= 32) {
            // the draws under examination sit in lanes 0 .. 31: every lane meets the other 15 of its row of 16 through
            // row rotations (rotation r brings the id of lane (l - r) mod 16, an earlier lane iff r <= l), and the
            // second row meets the whole first one through its copy swapped across rows
            const int l16 = lane & 15;
            const int x = __builtin_amdgcn_ds_swizzle(id, 0x401F);                              // lane xor 16
            const bool in_row = rotations_match<1, 16>(id, id, l16), in_other = rotations_match<0, 16>(id, x, 16);
            const bool dupe = in_row | (((lane & 16) != 0) & in_other);
            ok = ok && !dupe;
        } else {
            for (int l = 0; l < W - 1; ++l) {   // l is the same for the whole wavefront: a scalar read of lane l
                const int o = __builtin_amdgcn_readlane(id, l);
                if (l < lane && o == id) ok = false;
            }
        }
        const u64 m = __builtin_amdgcn_ballot_w64(ok);
        const int pos = cnt + __popcll(m & lanes_below(lane));
        if (ok && pos < S) ids[pos] = id;
        cnt += __popcll(m);
        if (cnt > S) cnt = S;
        j0 += W;
        wave_sync();
    }
    if (cnt < S) {   // fallback, practically unreachable: smallest unused ids
        for (long long id = 0; id < n && cnt < S; ++id) {
            if (id == u) continue;
            bool dup = false;
            for (int k = 0; k < cnt; ++k) dup = dup || (ids[k] == (int)id);
            if (!dup) {
                if (lane == 0) ids[cnt] = (int)id;
                ++cnt;
                wave_sync();
            }
        }
    }
}

struct SearchSmem {
    int id[SEARCH_MAX_L];      // vertices to evaluate
    u32 dist[SEARCH_MAX_L];    // their delta(q, .) bits
};

// delta(q, ids[0..cnt)) -> dist[0..cnt), 8 vertices at a time (8 lanes per vertex).  uint8 rows of at
// most 128 bytes that can be read 16 bytes at a time take one load per lane and vertex: the loads of up
// to 32 vertices are issued together, so their latency is paid once.  (Same arithmetic as the general
// routine: three byte dot products per word, xor-tree sum.)
template <int DT>
__device__ __forceinline__ void search_eval(const void *X, const void *qv, int d, int vec_ok, size_t rowbytes,
                                            SearchSmem &sm, int cnt, int lane)
{
    const int sub = lane & 7, grp = lane >> 3;
    if (DT == DT_U8 && vec_ok && d <= 128) {
        const bool mine = 16 * sub < d;     // d is a multiple of 16 here
        uint4 q4 = make_uint4(0u, 0u, 0u, 0u);
        if (mine) q4 = ((const uint4 *)qv)[sub];
        for (int b = 0; b < cnt; b += 32) {
            uint4 x4[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int p = b + 8 * j + grp;
                x4[j] = make_uint4(0u, 0u, 0u, 0u);
                if (p < cnt && mine) x4[j] = ((const uint4 *)((const char *)X + (size_t)sm.id[p] * rowbytes))[sub];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int p = b + 8 * j + grp;
                int acc = 0;
                acc = sqdiff_word_u8(q4.x, x4[j].x, acc);
                acc = sqdiff_word_u8(q4.y, x4[j].y, acc);
                acc = sqdiff_word_u8(q4.z, x4[j].z, acc);
                acc = sqdiff_word_u8(q4.w, x4[j].w, acc);
                acc = group8_sum(acc);
                if (p < cnt && sub == 0) sm.dist[p] = (u32)acc;
            }
        }
        return;
    }
    for (int b = 0; b < cnt; b += 8) {
        const int p = b + grp;
        const int id = sm.id[p < cnt ? p : cnt - 1];
        const u32 db = group8_dist_bits<DT>(qv, (const char *)X + (size_t)id * rowbytes, d, vec_ok, sub);
        if (p < cnt && sub == 0) sm.dist[p] = db;
    }
}

// C (E registers, ascending, KEY_PAD past its end) <- the 64 E smallest of C and the sorted-ascending
// register kn.  Bitonic merge: against the reversed kn, the element-wise minima are exactly the
// smallest keys and form a bitonic sequence, which strides 64 E / 2 ... 1 then sort.
template <int E>
__device__ __forceinline__ void merge_into_candidates(u64 (&C)[E], u64 kn, int lane)
{
    const u64 rev = shfl_u64(kn, 63 - lane);     // descending
    u64 &top = C[E - 1];
    top = top < rev ? top : rev;
    if (E == 2) {
        const u64 a = C[0], b = C[1];
        C[0] = a < b ? a : b;
        C[1] = a < b ? b : a;
    }
#pragma unroll
    for (int stride = 32; stride > 0; stride >>= 1) {
        const bool lower = (lane & stride) == 0;
#pragma unroll
        for (int r = 0; r < E; ++r) C[r] = keep_of_pair(C[r], xor_lane_u64(C[r], stride), lower);
    }
}

template <int DT, int E>
__global__ __launch_bounds__(256) void k_search(const void *X, long long N, int d, int vec_ok,
                                                const int *graph, const int *degree, int W, const void *Q,
                                                long long nq, int L, int K, int k, u64 seed, u32 *bitmaps,
                                                size_t bitmap_words, int *out_ids, u32 *out_dist,
                                                unsigned long long *evals)
{
    __shared__ SearchSmem smem[4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long gw = (long long)blockIdx.x * 4 + wave, nw = (long long)gridDim.x * 4;
    SearchSmem &sm = smem[wave];
    u32 *seen = bitmaps + (size_t)gw * bitmap_words;   // cleared by this wavefront before every query
    const size_t rowbytes = (size_t)d * dt_size(DT);
    const int L0 = (long long)L < N ? L : (int)N;
    // uint8 rows of at most 128 bytes, readable 16 bytes at a time: one load per lane and vertex
    const bool short_rows = DT == DT_U8 && vec_ok && d <= 128;
    unsigned long long ev = 0;
    for (long long q = gw; q < nq; q += nw) {
        const void *qv = (const char *)Q + (size_t)q * rowbytes;
        uint4 q4 = make_uint4(0u, 0u, 0u, 0u);      // short uint8 rows: this lane's 16 bytes of the query
        if (short_rows && 16 * (lane & 7) < d) q4 = ((const uint4 *)qv)[lane & 7];
        // ---- nothing has been evaluated for this query yet (the memory arrives uninitialised)
        for (size_t w4 = (size_t)lane * 4; w4 < bitmap_words; w4 += 256)
            *(uint4 *)(seen + w4) = make_uint4(0u, 0u, 0u, 0u);
        wave_sync();
        // ---- InitializeCandidates
        if ((long long)L0 == N) {
            for (int t = lane; t < L0; t += 64) sm.id[t] = t;
        } else {
            wave_random_ids(seed + 0x9E3779B97F4A7C15ull * (u64)q, N + 1, N, L0, sm.id, lane);
        }
        wave_sync();
        for (int t = lane; t < L0; t += 64) {
            const int v = sm.id[t];
            atomicOr(&seen[v >> 5], 1u << (v & 31));
        }
        search_eval<DT>(X, qv, d, vec_ok, rowbytes, sm, L0, lane);
        wave_sync();
        u64 C[E];
#pragma unroll
        for (int r = 0; r < E; ++r) {
            const int t = 64 * r + lane;
            C[r] = t < L0 ? make_key(sm.dist[t], (u32)sm.id[t], 1u) : KEY_PAD;
        }
        wave_sort<E>(C, lane);
        int m = L0;
        ev += (unsigned long long)L0;
        // ---- the search loop
        for (;;) {
            // select: the first unvisited member of C
            int iu = -1;
#pragma unroll
            for (int r = E - 1; r >= 0; --r) {
                const u64 b = __builtin_amdgcn_ballot_w64(64 * r + lane < m && (C[r] & 1ull));
                if (b) iu = 64 * r + (int)__builtin_ctzll(b);
            }
            if (iu < 0) break;
            const int u = (int)key_id(shfl_u64(C[iu >> 6], iu & 63));
            if (lane == (iu & 63)) C[iu >> 6] &= ~1ull;
            // the first 64 entries of u's row are read without waiting for its degree (rows are W wide)
            int v0 = -1;
            if (lane < W && lane < K) v0 = graph[(size_t)u * W + lane];
            int du = degree[u];
            if (du > K) du = K;     // Eq. 4: rows are nearest-first
            if (du > W) du = W;
            if (du < 0) du = 0;
            for (int t0 = 0; t0 < du; t0 += 64) {
                // expand, skipping what was evaluated before
                const int t = t0 + lane;
                int v = -1;
                if (t < du) v = t0 == 0 ? v0 : graph[(size_t)u * W + t];
                const bool isv = v >= 0 && (long long)v < N;   // anything else is not a vertex: ignored
                u64 kn;
                if (short_rows) {
                    // evaluate every neighbour, while the bitmap answers which of them are new to this
                    // query: short rows cost less to read than a second round trip; lane p keeps candidate p
                    const int sub = lane & 7, grp = lane >> 3;
                    const int np = du - t0 < 64 ? du - t0 : 64;
                    u32 old = 0xFFFFFFFFu;
                    const u32 bit = 1u << (v & 31);
                    if (isv) old = atomicOr(&seen[v >> 5], bit);
                    wave_sync();
                    for (int b = 0; b < np; b += 32) {
                        uint4 x4[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int p = b + 8 * j + grp;
                            const int idp = __shfl(v, p & 63);
                            x4[j] = make_uint4(0u, 0u, 0u, 0u);
                            if (p < np && idp >= 0 && (long long)idp < N && 16 * sub < d)
                                x4[j] = ((const uint4 *)((const char *)X + (size_t)idp * rowbytes))[sub];
                        }
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int p = b + 8 * j + grp;
                            int acc = 0;
                            acc = sqdiff_word_u8(q4.x, x4[j].x, acc);
                            acc = sqdiff_word_u8(q4.y, x4[j].y, acc);
                            acc = sqdiff_word_u8(q4.z, x4[j].z, acc);
                            acc = sqdiff_word_u8(q4.w, x4[j].w, acc);
                            acc += __shfl_xor(acc, 1);
                            acc += __shfl_xor(acc, 2);
                            acc += __shfl_xor(acc, 4);
                            if (p < np && sub == 0) sm.dist[p] = (u32)acc;
                        }
                    }
                    wave_sync();
                    const bool fresh = isv && (old & bit) == 0u;
                    ev += (unsigned long long)__popcll(__builtin_amdgcn_ballot_w64(fresh));
                    kn = fresh ? make_key(sm.dist[lane], (u32)v, 1u) : KEY_PAD;
                } else {
                    bool fresh = false;
                    if (isv) {
                        const u32 bit = 1u << (v & 31);
                        fresh = (atomicOr(&seen[v >> 5], bit) & bit) == 0u;
                    }
                    const u64 fm = __builtin_amdgcn_ballot_w64(fresh);
                    const int nf = __popcll(fm);
                    if (nf == 0) continue;
                    wave_sync();
                    if (fresh) sm.id[__popcll(fm & lanes_below(lane))] = v;
                    wave_sync();
                    // evaluate
                    search_eval<DT>(X, qv, d, vec_ok, rowbytes, sm, nf, lane);
                    ev += (unsigned long long)nf;
                    wave_sync();
                    kn = lane < nf ? make_key(sm.dist[lane], (u32)sm.id[lane], 1u) : KEY_PAD;
                }
                // insert
                if (m == L) {
                    const u64 last = shfl_u64(C[(L - 1) >> 6], (L - 1) & 63);
                    if ((kn >> 1) >= (last >> 1)) kn = KEY_PAD;
                }
                const int na = __popcll(__builtin_amdgcn_ballot_w64(kn != KEY_PAD));
                if (na == 0) continue;
                u64 ks[1] = {kn};
                wave_sort<1>(ks, lane);
                merge_into_candidates<E>(C, ks[0], lane);
                m = m + na < L ? m + na : L;
                // the registers hold 64 E keys; C is its first L
#pragma unroll
                for (int r = 0; r < E; ++r)
                    if (64 * r + lane >= m) C[r] = KEY_PAD;
            }
        }
        // ---- output: the k nearest members of C
#pragma unroll
        for (int r = 0; r < E; ++r) {
            const int t = 64 * r + lane;
            if (t < k) {
                out_ids[(size_t)q * k + t] = t < m ? (int)key_id(C[r]) : -1;
                if (out_dist) out_dist[(size_t)q * k + t] = t < m ? key_dist(C[r]) : 0xFFFFFFFFu;
            }
        }
    }
    if (lane == 0 && evals && ev) atomicAdd(evals, ev);
}
