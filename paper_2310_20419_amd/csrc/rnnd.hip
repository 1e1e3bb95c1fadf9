// librnnd: Relative NN-Descent graph construction (arXiv 2310.20419, Alg. 4-6) on gfx950.
//
// A wavefront, or a group of 16, 32 or 64 of its lanes, owns one vertex in every per-vertex kernel.
// A round is synchronous:
//   scan     every active vertex (one holding a "new" entry) runs the body of Alg. 4's vertex loop on its own list,
//            writes its kept entries back in place and leaves its redirected edges in its slot of `props`
//   scatter  every redirected edge takes an arrival number at its target (the round's only atomic per
//            edge) and moves into the target's inbox (INBOX_CAP slots per vertex); later arrivals wait
//   classify vertices that received edges form the `touched` lists, by the size of the merge they need;
//            those that received more than INBOX_CAP get a bin, which a second scatter pass fills
//   merge    every touched list becomes the first R distinct keys of (kept entries + inbox + bin)
//   compact  touched vertices whose new list holds a "new" entry form the next active lists,
//            one per degree class (see degree_class)
// Between outer rounds AddReverseEdges (Alg. 5) uses the same inboxes and bins (launch_reverse).
// Counters that many wavefronts would hit at one address are aggregated per block first.
// search.h holds the graph search of Alg. 1 (rnnd_search).
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include <mutex>

#include "../../include/rnnd.h"
#include "wave_prims.h"

#define WAVES_PER_BLOCK 4
#define BLOCK (64 * WAVES_PER_BLOCK)
#define GOLDEN64 0x9E3779B97F4A7C15ull
#define RNND_MAX_SLOTS 0x7FFFFF00ull   // N * (slots per row): bin offsets are ints, -1 = no bin
#define RNND_MAX_RUN_SLOTS 131072      // rounds (x runs per pass): one small counter block each
#define NDEG 8   // degree classes of the active lists (see degree_class)
#define NMRG 4   // merge classes of the touched lists: kept + received at most 16, 32, 64, more
#ifndef INBOX_CAP
#define INBOX_CAP 64   // redirected edges a vertex can receive per round without the overflow path
#endif

// Per-round device counters.  Round t reads ctr[t].n_active[] and fills the rest; its compact step
// writes ctr[t+1].n_active[].  Zeroed once per call, never reset, so they double as statistics.
#define STAT_SLOTS 64
struct RoundCtr {
    u32 n_active[NDEG];   // lengths of this round's active lists
    u32 n_touched[NMRG];  // distinct targets of the redirected edges, by size of the merge they need
    u32 bin_cursor;       // space handed out in the bin array
    u32 has_surplus;      // some vertex received more than INBOX_CAP edges this round
    u32 pad[2];
    u32 n_redo[NDEG];     // float scan: vertices the single-precision form left to the double-precision one
    // ticks of the device's constant-rate clock (0 = not taken): the round's first scan launch starts, its scatter
    // starts (= the scan has ended: launches of one stream run back to back), the round's last kernel has ended
    // (taken by k_stamp after the last round before an AddReverseEdges call or the export, only where statistics
    // ask for it; every other round, and an AddReverseEdges call, ends where the next round's scan starts)
    u64 t_scan_start, t_scan_stop, t_round_stop;
    // statistics, spread over STAT_SLOTS addresses so that the adds of many blocks do not queue up
    // on one: [slot][0..4] = algorithmic evals, executed evals, rows gathered, edges redirected, entries a merge
    // dropped because the list was full
    u64 stat[STAT_SLOTS][5];
};

// One add per wavefront into the slot of its block.
__device__ __forceinline__ void add_round_stats(RoundCtr *ctr, u64 algo, u64 exec, u64 rows, u64 props)
{
    u64 *s = ctr->stat[blockIdx.x & (STAT_SLOTS - 1)];
    atomicAdd(&s[0], algo);
    atomicAdd(&s[1], exec);
    atomicAdd(&s[2], rows);
    atomicAdd(&s[3], props);
}

// Statistics take the scan time of a round from the device's own clock instead of events attached to the launches:
// an event costs 4-7 microseconds of idle queue after its kernel, three per round used to add 1 ms to a 27 ms build.
__device__ __forceinline__ void stamp_scan_start(RoundCtr *ctr)
{   // the first scan launch of a round that comes by fills the field
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0 && ctr->t_scan_start == 0ull) ctr->t_scan_start = wall_clock64();
}
__device__ __forceinline__ void stamp_scan_stop(RoundCtr *ctr)
{
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) ctr->t_scan_stop = wall_clock64();
}
__global__ void k_stamp(u64 *dst) { if (threadIdx.x == 0) *dst = wall_clock64(); }

struct Prop {          // one redirected edge (Alg. 4, the edge update): `key` enters `tgt`'s list
    u64 key;
    u32 tgt;
    u32 arrival;       // set by the scatter: arrival number at tgt, for edges past the inbox
};

// The edge update of Alg. 4: (w, v) enters E.  Recorded in the scanning vertex's own slot.
__device__ __forceinline__ void emit_redirect(u64 key, u32 tgt, Prop *slot)
{
    Prop pr;
    pr.key = key;
    pr.tgt = tgt;
    pr.arrival = 0;
    *slot = pr;
}

#include "dist.h"
#include "scan_mfma.h"
#include "scan_mfma_f32.h"
#include "search.h"

// Degree class of a list of m entries: which scan kernel takes it.  use_classes 0: one list for all
// (generic scan).  2 (uint8 matrix-core scan): classes 0, 1, 2 = at most 8, 16, 32 entries (four, two,
// one vertex per wavefront), 3, 4, 5 = at most 64, 96, 128 (two, three, four 32-row blocks).
// 1 (float matrix-core scan, 16-row groups): classes 0..6 = at most 8, 16, 32, 48, 64, 80, 96 entries
// (1, 1, 2, 3, 4, 5, 6 groups), 7 = more (generic scan).
__device__ __forceinline__ int degree_class(int m, int use_classes)
{
    if (!use_classes) return 0;
    if (m <= 16) return m <= 8 ? 0 : 1;
    if (use_classes == 2) return m <= 32 ? 2 : 2 + ((m - 1) >> 5);
    return m <= 96 ? 1 + ((m - 1) >> 4) : 7;
}

// ------------------------------------------------------------------ RandomGraph
// Alg. 6, RandomGraph: S distinct random neighbours (wave_random_ids), their distances, sorted.
template <int DT>
__global__ __launch_bounds__(BLOCK) void k_random_graph(const void *X, long long N, int d, int vec_ok,
                                                        int S, int R, u64 seed, u64 *keys, int *deg,
                                                        int8_t *vcls, int use_classes)
{
    static_assert(SEARCH_MAX_L >= RNND_MAX_R, "the id / distance tables of the search hold a whole list");
    __shared__ SearchSmem s_tab[WAVES_PER_BLOCK];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long u = (long long)blockIdx.x * WAVES_PER_BLOCK + wave;
    if (u >= N) return;
    int *ids = s_tab[wave].id;
    const size_t rowbytes = (size_t)d * dt_size(DT);
    wave_random_ids(seed, N, u, S, ids, lane);
    wave_sync();
    // delta(u, id), 8 lanes per row; short uint8 rows: the loads of up to 32 rows in flight together
    search_eval<DT>(X, (const char *)X + (size_t)u * rowbytes, d, vec_ok, rowbytes, s_tab[wave], S, lane);
    wave_sync();
    u64 *row = keys + (size_t)u * R;
    if (S <= 32) {     // the upper half of the wavefront sorts padding
        u64 k = lane < S ? make_key(s_tab[wave].dist[lane], (u32)ids[lane], 1u) : KEY_PAD;
        k = group_sort<32>(k, lane);
        if (lane < S) row[lane] = k;
    } else if (S <= 64) {
        u64 k[1];
        k[0] = lane < S ? make_key(s_tab[wave].dist[lane], (u32)ids[lane], 1u) : KEY_PAD;
        wave_sort<1>(k, lane);
        if (lane < S) row[lane] = k[0];
    } else {
        u64 k[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            int e = r * 64 + lane;
            k[r] = e < S ? make_key(s_tab[wave].dist[e], (u32)ids[e], 1u) : KEY_PAD;
        }
        wave_sort<2>(k, lane);
        if (lane < S) row[lane] = k[0];
        if (lane + 64 < S) row[lane + 64] = k[1];
    }
    if (lane == 0) {
        deg[u] = S;
        if (vcls) vcls[u] = (int8_t)degree_class(S, use_classes);   // every vertex starts with "new" entries
    }
}

// ------------------------------------------------- UpdateNeighbors: scan (generic kernel)
// The body of Alg. 4's vertex loop for one vertex per wavefront, in the algorithm's own order: v runs over the
// sorted list; the kept set U' so far is a bit mask; the delta(v,w) of up to 8 eligible w (kept,
// not old/old) are evaluated at once by 8-lane groups in ascending w, and the first failing one
// prunes v and redirects it.  Kept entries are written back in place with the flag cleared.
template <int DT>
__global__ __launch_bounds__(BLOCK) void k_update_scan(const void *X, int d, int vec_ok, int R,
                                                       u64 *keys, int *deg, const int *list,
                                                       const u32 *n_list, Prop *props, int *nprop,
                                                       RoundCtr *ctr)
{
    __shared__ u64 s_key[WAVES_PER_BLOCK][RNND_MAX_R];
    __shared__ u64 s_pkey[WAVES_PER_BLOCK][RNND_MAX_R];
    __shared__ u32 s_ptgt[WAVES_PER_BLOCK][RNND_MAX_R];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, sub = lane & 7, grp = lane >> 3;
    const u32 gw = blockIdx.x * WAVES_PER_BLOCK + wave, nw = gridDim.x * WAVES_PER_BLOCK;
    const u32 n_active = *n_list;
    const size_t rowbytes = (size_t)d * dt_size(DT);
    u64 *sk = s_key[wave];
    stamp_scan_start(ctr);
    u64 evals_algo = 0, evals_exec = 0, rows = 0, nprops_total = 0;
    for (u32 it = gw; it < n_active; it += nw) {
        const int u = list[it];
        int m = deg[u];
        if (m > R) m = R;
        u64 *row = keys + (size_t)u * R;
        u64 k0 = lane < m ? row[lane] : KEY_PAD;
        u64 k1 = lane + 64 < m ? row[lane + 64] : KEY_PAD;
        wave_sync();
        sk[lane] = k0;
        sk[lane + 64] = k1;
        const u64 new0 = __builtin_amdgcn_ballot_w64(lane < m && (k0 & 1ull));
        const u64 new1 = __builtin_amdgcn_ballot_w64(lane + 64 < m && (k1 & 1ull));
        wave_sync();
        if ((new0 | new1) == 0) {
            if (lane == 0) nprop[u] = 0;
            continue;
        }
        rows += m;
        u64 K0 = 0, K1 = 0;   // U' as positions in the sorted list
        int np = 0;
        for (int i = 0; i < m; ++i) {
            const u64 ki = sk[i];
            const u32 di = key_dist(ki), idv = key_id(ki);
            const bool newv = ki & 1ull;
            u64 e0 = newv ? K0 : (K0 & new0);   // old/old pairs are skipped
            u64 e1 = newv ? K1 : (K1 & new1);
            bool pruned = false;
            const char *xv = (const char *)X + (size_t)idv * rowbytes;
            while ((e0 | e1) != 0 && !pruned) {
                int mypos = -1, nb = 0;
#pragma unroll
                for (int g = 0; g < 8; ++g) {
                    int p = -1;
                    if (e0) { p = __builtin_ctzll(e0); e0 &= e0 - 1; }
                    else if (e1) { p = 64 + __builtin_ctzll(e1); e1 &= e1 - 1; }
                    if (p >= 0) ++nb;
                    if (grp == g) mypos = p;
                }
                const u32 idw = key_id(sk[mypos >= 0 ? mypos : 0]);
                u32 db = 0;
                if (mypos >= 0)
                    db = group8_dist_bits<DT>(xv, (const char *)X + (size_t)idw * rowbytes, d, vec_ok, sub);
                const bool fail = mypos >= 0 && di >= db;   // the prune test
                const u64 fm = __builtin_amdgcn_ballot_w64(fail && sub == 0);
                if (fm) {
                    const int fl = __builtin_ctzll(fm);     // first failing w in list order
                    const u32 fdb = __shfl(db, fl), fidw = __shfl(idw, fl);
                    if (lane == 0) {                        // the edge update: (u,v) leaves, (w,v) enters
                        s_pkey[wave][np] = make_key(fdb, idv, 1u);
                        s_ptgt[wave][np] = fidw;
                    }
                    ++np;
                    evals_algo += (fl >> 3) + 1;
                    pruned = true;
                } else {
                    evals_algo += nb;
                }
                evals_exec += nb;
            }
            if (!pruned) {
                if (i < 64) K0 |= 1ull << i; else K1 |= 1ull << (i - 64);   // v joins U'
            }
        }
        // kept entries, flag old, compacted back into the row
        const int nk0 = __popcll(K0);
        if ((K0 >> lane) & 1ull) row[__popcll(K0 & lanes_below(lane))] = k0 & ~1ull;
        if ((K1 >> lane) & 1ull) row[nk0 + __popcll(K1 & lanes_below(lane))] = k1 & ~1ull;
        if (lane == 0) {
            deg[u] = nk0 + __popcll(K1);
            nprop[u] = np;
        }
        wave_sync();
        for (int p = lane; p < np; p += 64)
            emit_redirect(s_pkey[wave][p], s_ptgt[wave][p], props + (size_t)u * R + p);
        nprops_total += np;
    }
    if (lane == 0 && rows) add_round_stats(ctr, evals_algo, evals_exec, rows, nprops_total);
}

// ------------------------------------------------------ UpdateNeighbors: merge
// Vertices x with cnt[x] > list_min are appended to `list`; those with cnt[x] > bin_min get a bin of
// cnt[x] - bin_sub keys starting at binoff[x] (others: binoff = -1).  One pair of atomics per 1024
// vertices.  Optionally clears zero_a[] and zero_b[], sets thr[] to "keep all", and marks in cand[]
// the vertices with deg[x] + cnt[x] > cand_R.
__global__ __launch_bounds__(1024) void k_assign_bins(long long N, const int *cnt, int list_min, int bin_min,
                                                      int bin_sub, int *binoff, u32 *bin_cursor, int *list,
                                                      u32 *n_list, int *zero_a, int *zero_b, u64 *thr,
                                                      const int *deg, int cand_R, int8_t *cand)
{
    __shared__ u32 s_sum[16], s_num[16], s_base[2];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long x = (long long)blockIdx.x * 1024 + threadIdx.x;
    int c = 0;
    if (x < N) {
        c = cnt[x];
        if (zero_a) zero_a[x] = 0;
        if (zero_b) zero_b[x] = 0;
        if (thr) thr[x] = KEY_PAD;
        if (cand) cand[x] = (int8_t)(deg[x] + c > cand_R);
    }
    const bool in_list = c > list_min;
    const u32 mine = c > bin_min ? (u32)(c - bin_sub) : 0u;
    u32 incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        u32 v = __shfl_up(incl, o);
        if (lane >= o) incl += v;
    }
    const u64 hb = __builtin_amdgcn_ballot_w64(in_list);
    if (lane == 63) { s_sum[wave] = incl; s_num[wave] = (u32)__popcll(hb); }
    __syncthreads();
    if (threadIdx.x == 0) {
        u32 ts = 0, tn = 0;
        for (int w = 0; w < 16; ++w) { u32 a = s_sum[w], b = s_num[w]; s_sum[w] = ts; s_num[w] = tn; ts += a; tn += b; }
        s_base[0] = ts ? atomicAdd(bin_cursor, ts) : 0u;
        s_base[1] = tn ? atomicAdd(n_list, tn) : 0u;
    }
    __syncthreads();
    if (x < N) {
        binoff[x] = mine ? (int)(s_base[0] + s_sum[wave] + incl - mine) : -1;
        if (in_list) list[s_base[1] + s_num[wave] + __popcll(hb & lanes_below(lane))] = (int)x;
    }
}

// The active lists of a round's first ncl degree classes walked as one: start[k] = entries of the classes before k.
struct ActiveLists {
    const int *lists;
    long long N;
    u32 start[NDEG + 1];
};

__device__ __forceinline__ ActiveLists active_lists(const int *lists, long long N, const RoundCtr *ctr, int ncl)
{
    ActiveLists a;
    a.lists = lists;
    a.N = N;
    u32 sum = 0;
#pragma unroll
    for (int k = 0; k < NDEG; ++k) {
        a.start[k] = sum;
        sum += k < ncl ? ctr->n_active[k] : 0u;
    }
    a.start[NDEG] = sum;
    return a;
}

// entry i of the concatenation, i < start[NDEG]
__device__ __forceinline__ int active_vertex(const ActiveLists &a, u32 i)
{
    u32 c = 0, off = i;
#pragma unroll
    for (int k = 1; k < NDEG; ++k)
        if (i >= a.start[k]) {
            c = (u32)k;
            off = i - a.start[k];
        }
    return a.lists[(size_t)c * (size_t)a.N + off];
}

// Bit j set iff lane j of this lane's row of 16 holds the same value, for the lanes reached by rotations R .. 15.
template <int R>
__device__ __forceinline__ u32 same_target_mask(u32 tgt, int sub)
{
    if constexpr (R >= 16) {
        return 0u;
    } else {
        const u32 t = (u32)__builtin_amdgcn_update_dpp(0, (int)tgt, 0x120 + R, 0xF, 0xF, true);     // row_ror:R
        const u32 here = (t == tgt ? 1u : 0u) << ((sub - R) & 15);
        return here | same_target_mask<R + 1>(tgt, sub);
    }
}

#define SURPLUS_MARK 0x40000000   // set in nprop[u]: some edge redirected by u arrived past its target's inbox

// Every active vertex moves its redirected edges to their targets, 16 lanes per vertex.  Lanes of a
// group that share a target take their arrival numbers with one atomic (a vertex usually redirects
// several entries to the same kept neighbour).  Arrivals below INBOX_CAP go to the target's inbox;
// later ones record their number in the edge and are placed by k_scatter_surplus once bins exist.
__global__ __launch_bounds__(BLOCK) void k_scatter(long long N, int R, const int *lists, int ncl, RoundCtr *ctr,
                                                   Prop *props, int *nprop, int *fill, u64 *inbox)
{
    const int lane = threadIdx.x & 63, sub = lane & 15, gbase = lane & ~15;
    const u32 g = (blockIdx.x * BLOCK + threadIdx.x) >> 4, ng = (gridDim.x * BLOCK) >> 4;
    // the classes' lists as one: the grid is shared by their entries, however they are spread over the classes
    const ActiveLists al = active_lists(lists, N, ctr, ncl);
    const u32 n = al.start[NDEG];
    bool surplus = false;
    stamp_scan_stop(ctr);
    if (g >= n) return;
    // the loads of the next vertex (its count and its first 16 edges) are issued before the atomics
    // of the current one; the list entry of the vertex after that is fetched one trip earlier still
    auto vertex_at = [&](unsigned long long i) -> int { return i < n ? active_vertex(al, (u32)i) : -1; };
    auto first_edges = [&](int u, int &np, Prop &pr) {
        np = 0;
        pr.key = 0; pr.tgt = 0xFFFFFFFFu; pr.arrival = 0;
        if (u >= 0) {
            np = nprop[u];
            if (sub < R) pr = props[(size_t)u * R + sub];   // slots past np exist; masked below
        }
    };
    int u = vertex_at(g), np;
    Prop pr0;
    first_edges(u, np, pr0);
    int u_next = vertex_at((unsigned long long)g + ng);
    for (unsigned long long it = g; it < n; it += ng) {
        int np_next;
        Prop pr_next;
        first_edges(u_next, np_next, pr_next);
        const int u_after = vertex_at(it + 2ull * ng);

        bool mine_surplus = false;
        for (int p0 = 0; p0 < np; p0 += 16) {      // same trip count for the whole group
            const int p = p0 + sub;
            const bool have = p < np;
            Prop pr = pr0;
            if (p0 > 0 && have) pr = props[(size_t)u * R + p];
            if (!have) pr.tgt = 0xFFFFFFFFu;
            // lanes of my group with my target
            // rotation r of the group's row brings the target of lane (sub - r) mod 16
            const u32 same = (1u << sub) | same_target_mask<1>(pr.tgt, sub);
            const int leader = __builtin_ctz(same), rank = __popc(same & ((1u << sub) - 1u));
            int base = 0;
            if (have && sub == leader) base = atomicAdd(&fill[pr.tgt], __popc(same));
            base = __shfl(base, gbase + leader);
            if (have) {
                const int s = base + rank;
                if (s < INBOX_CAP) {
                    inbox[(size_t)pr.tgt * INBOX_CAP + s] = pr.key;
                } else {
                    props[(size_t)u * R + p].arrival = (u32)s;
                    mine_surplus = true;
                }
            }
        }
        // mark u for the second pass (this group is the only one that touches nprop[u])
        const u32 anyb = ((u32)(__builtin_amdgcn_ballot_w64(mine_surplus) >> gbase)) & 0xFFFFu;
        if (anyb) {
            if (sub == 0) nprop[u] = np | SURPLUS_MARK;
            surplus = true;
        }
        u = u_next; np = np_next; pr0 = pr_next;
        u_next = u_after;
    }
    if (surplus) ctr->has_surplus = 1u;
}

// Second pass, only when some vertex received more than INBOX_CAP edges: the late arrivals go to bins.
__global__ __launch_bounds__(BLOCK) void k_scatter_surplus(long long N, int R, const int *lists, int ncl,
                                                           const RoundCtr *ctr, const Prop *props,
                                                           const int *nprop, const int *binoff, u64 *bins)
{
    if (ctr->has_surplus == 0) return;
    const int sub = threadIdx.x & 15;
    const u32 g = (blockIdx.x * BLOCK + threadIdx.x) >> 4, ng = (gridDim.x * BLOCK) >> 4;
    const ActiveLists al = active_lists(lists, N, ctr, ncl);
    const u32 n = al.start[NDEG];
    for (unsigned long long it = g; it < n; it += ng) {
        const int u = active_vertex(al, (u32)it);
        int np = nprop[u];
        if (!(np & SURPLUS_MARK)) continue;
        np &= ~SURPLUS_MARK;
        for (int p = sub; p < np; p += 16) {
            const Prop pr = props[(size_t)u * R + p];
            if (pr.arrival >= (u32)INBOX_CAP)
                bins[(size_t)binoff[pr.tgt] + (pr.arrival - INBOX_CAP)] = pr.key;
        }
    }
}

// Merge class of a vertex that holds nb entries and received c: how wide a sort its merge needs.
__device__ __forceinline__ int merge_class(int nb, int c)
{
    const int total = nb + c;
    return total <= 16 ? 0 : total <= 32 ? 1 : total <= 64 ? 2 : 3;
}

// Every vertex x that received edges (cnt[x] > 0) is appended to the touched list of its merge class;
// if it received more than INBOX_CAP it also gets a bin for the surplus.  A block covers TC_TILES x 1024
// vertices and takes its space with one atomic per class (and one for the bins).  Four tiles per block
// keep the atomics of a 1M-vertex round few; on small inputs two tiles (twice the blocks, a shorter chain in
// each) are faster: 100,000 vertices 4.68 -> 4.55 ms per build, 1M 26.0 -> 26.1 ms.
template <int TC_TILES>
__global__ __launch_bounds__(1024) void k_touch_classify(long long N, const int *cnt, const int *deg,
                                                         int *binoff, RoundCtr *ctr, int *tlists)
{
    __shared__ u32 s_cnt[TC_TILES][16][NMRG], s_sum[TC_TILES][16], s_base[NMRG + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int mc[TC_TILES];
    u32 mine[TC_TILES], incl[TC_TILES], rank[TC_TILES];
#pragma unroll
    for (int k = 0; k < TC_TILES; ++k) {
        const long long x = ((long long)blockIdx.x * TC_TILES + k) * 1024 + threadIdx.x;
        int c = 0;
        mc[k] = -1;
        if (x < N) {
            c = cnt[x];
            if (c > 0) mc[k] = merge_class(deg[x], c);
        }
        mine[k] = c > INBOX_CAP ? (u32)(c - INBOX_CAP) : 0u;
        u32 in = mine[k];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            u32 v = __shfl_up(in, o);
            if (lane >= o) in += v;
        }
        incl[k] = in;
        rank[k] = 0;
#pragma unroll
        for (int q = 0; q < NMRG; ++q) {
            const u64 b = __builtin_amdgcn_ballot_w64(mc[k] == q);
            if (mc[k] == q) rank[k] = (u32)__popcll(b & lanes_below(lane));
            if (lane == 0) s_cnt[k][wave][q] = (u32)__popcll(b);
        }
        if (lane == 63) s_sum[k][wave] = in;
    }
    __syncthreads();
    if (wave == 0) {
        // exclusive prefix over the TC_TILES x 16 wavefront totals, in (tile, wavefront) order: lane = tile * 16 + wavefront
        static_assert(TC_TILES * 16 <= 64, "one lane of the first wavefront per (tile, wavefront)");
        const bool used = lane < TC_TILES * 16;
        const int k = used ? lane >> 4 : 0, w = lane & 15;
#pragma unroll
        for (int q = 0; q <= NMRG; ++q) {
            const u32 a = !used ? 0u : q < NMRG ? s_cnt[k][w][q] : s_sum[k][w];
            u32 in = a;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                u32 v = __shfl_up(in, o);
                if (lane >= o) in += v;
            }
            if (used) {
                if (q < NMRG) s_cnt[k][w][q] = in - a;
                else s_sum[k][w] = in - a;
            }
            if (lane == 63) s_base[q] = in;
        }
        wave_sync();
        if (lane <= NMRG) {     // the block's atomics are in flight together
            const u32 tot = s_base[lane];
            s_base[lane] = tot ? atomicAdd(lane < NMRG ? &ctr->n_touched[lane] : &ctr->bin_cursor, tot) : 0u;
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TC_TILES; ++k) {
        const long long x = ((long long)blockIdx.x * TC_TILES + k) * 1024 + threadIdx.x;
        if (x < N) {
            binoff[x] = mine[k] ? (int)(s_base[NMRG] + s_sum[k][wave] + incl[k] - mine[k]) : -1;
            if (mc[k] >= 0)
                tlists[(size_t)mc[k] * N + s_base[mc[k]] + s_cnt[k][wave][mc[k]] + rank[k]] = (int)x;
        }
    }
}

// Merge of the touched vertices whose kept entries + received edges number at most G: one vertex per
// group of G lanes.  list <- first R distinct keys; tcls[it] <- degree class if a "new" entry survives, else -1.
// Lane `sub` of a group holds list slot `sub` and inbox slot G-1-sub, so what to load depends only on
// the vertex; the loads of the next vertex and the list entry of the one after are issued before the
// current vertex is sorted.
struct MergeItem {
    int x;        // vertex, -1 past the end of the list
    int nb, c;    // kept entries, received entries
    u64 kr, ki;   // list slot `sub`, inbox slot G-1-sub (either may be garbage: masked by nb, c)
};

template <int G>
__device__ __forceinline__ MergeItem merge_item_load(int x, int R, const u64 *keys, const int *deg,
                                                     const int *cnt, const u64 *inbox, int sub)
{
    // past the end of the list (x < 0) vertex 0 is read instead and given no entries: loads without branches
    MergeItem m;
    const size_t xx = (size_t)(x >= 0 ? x : 0);
    const int nb = deg[xx], c = cnt[xx];
    m.x = x;
    m.nb = x >= 0 ? nb : 0;
    m.c = x >= 0 ? c : 0;
    m.kr = keys[xx * R + (sub < R ? sub : R - 1)];
    m.ki = inbox[xx * INBOX_CAP + (G - 1 - sub)];
    return m;
}

template <int G>
__device__ __forceinline__ void merge_group_body(int R, u64 *keys, int *deg, const int *tlist,
                                                 const u32 *n_ptr, int *cnt, const u64 *inbox,
                                                 int8_t *tcls, int use_classes, RoundCtr *ctr)
{
    int dropped = 0;
    static_assert(G <= INBOX_CAP, "a group merge reads the received edges from the inbox only");
    const int lane = threadIdx.x & 63, sub = lane & (G - 1), shift = lane & ~(G - 1);
    const u64 gmask = G == 64 ? ~0ull : ((1ull << (G & 63)) - 1ull);
    const u32 gid = (blockIdx.x * BLOCK + threadIdx.x) / G, ngrp = (gridDim.x * BLOCK) / G;
    const u32 n = *n_ptr;
    if (gid >= n) return;
    // list indices fit 32 bits with room to spare: n <= 2^31 and three strides of the grid are far below 2^31
    auto vertex_at = [&](u32 i) -> int { const int v = tlist[i < n ? i : n - 1u]; return i < n ? v : -1; };
    MergeItem cur = merge_item_load<G>(vertex_at(gid), R, keys, deg, cnt, inbox, sub);
    int x_next = vertex_at(gid + ngrp);
    int x_after = vertex_at(gid + 2u * ngrp);
    for (u32 it = gid; it < n; it += ngrp) {
        const MergeItem nxt = merge_item_load<G>(x_next, R, keys, deg, cnt, inbox, sub);
        x_next = x_after;
        x_after = vertex_at(it + 3u * ngrp);

        const int x = cur.x, nb = cur.nb, c = cur.c;
        u64 *row = keys + (size_t)x * R;
        u64 k = KEY_PAD;
        if (sub < nb) k = cur.kr;
        else if (G - 1 - sub < c) k = cur.ki;
        k = group_sort<G>(k, lane);
        u64 prev = shfl_up1_u64(k);
        if (sub == 0) prev = KEY_PAD;
        const bool keep = (k != KEY_PAD) && ((k >> 1) != (prev >> 1));
        const u64 m = (__builtin_amdgcn_ballot_w64(keep) >> shift) & gmask;
        const int pos = __popcll(m & lanes_below(sub));
        const bool w = keep && pos < R;
        if (w) row[pos] = k;
        const u64 nm = (__builtin_amdgcn_ballot_w64(w && (k & 1ull)) >> shift) & gmask;
        if (sub == 0) {
            int nd = __popcll(m);
            if (nd > R) { dropped += nd - R; nd = R; }
            deg[x] = nd;
            cnt[x] = 0;
            tcls[it] = nm ? (int8_t)degree_class(nd, use_classes) : (int8_t)-1;
        }
        cur = nxt;
    }
    if (dropped) atomicAdd(&ctr->stat[blockIdx.x & (STAT_SLOTS - 1)][4], (u64)dropped);
}

// General merge (any size): one touched vertex per wavefront; kept entries + inbox + surplus bin.
// The common case (at most INBOX_CAP received, at most 128 keys in all) is sorted in registers from
// loads issued one vertex ahead: lane l holds list slots l and l + 64 and inbox slot 63 - l.
struct WideItem {
    int x, nb, c;
    u64 r0, r1, in;
};

__device__ __forceinline__ WideItem wide_item_load(int x, int R, const u64 *keys, const int *deg, const int *cnt,
                                                   const u64 *inbox, int lane)
{
    WideItem m;
    const size_t xx = (size_t)(x >= 0 ? x : 0);      // as in merge_item_load
    const int nb = deg[xx], c = cnt[xx];
    m.x = x;
    m.nb = x >= 0 ? nb : 0;
    m.c = x >= 0 ? c : 0;
    m.r0 = keys[xx * R + (lane < R ? lane : R - 1)];
    m.r1 = keys[xx * R + (lane + 64 < R ? lane + 64 : R - 1)];
    m.in = inbox[xx * INBOX_CAP + (INBOX_CAP - 1 - lane)];
    return m;
}

__device__ __forceinline__ void merge_general_body(int R, u64 *keys, int *deg, const int *tlist,
                                                   const u32 *n_ptr, int *cnt, const u64 *inbox,
                                                   const int *binoff, const u64 *bins, int8_t *tcls,
                                                   int use_classes, u64 (*s_stage)[RNND_MAX_R], RoundCtr *ctr)
{
    int dropped = 0;
    static_assert(INBOX_CAP == 64, "lane l prefetches inbox slot 63 - l");
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const u32 gw = blockIdx.x * WAVES_PER_BLOCK + wave, nw = gridDim.x * WAVES_PER_BLOCK;
    const u32 n = *n_ptr;
    if (gw >= n) return;
    auto vertex_at = [&](u32 i) -> int { const int v = tlist[i < n ? i : n - 1u]; return i < n ? v : -1; };
    WideItem cur = wide_item_load(vertex_at(gw), R, keys, deg, cnt, inbox, lane);
    int x_next = vertex_at(gw + nw);
    int x_after = vertex_at(gw + 2u * nw);
    for (u32 it = gw; it < n; it += nw) {
        const WideItem nxt = wide_item_load(x_next, R, keys, deg, cnt, inbox, lane);
        x_next = x_after;
        x_after = vertex_at(it + 3u * nw);

        const int x = __builtin_amdgcn_readfirstlane(cur.x);
        const int nb = __builtin_amdgcn_readfirstlane(cur.nb), c = __builtin_amdgcn_readfirstlane(cur.c);
        bool any_new = false;
        int nd;
        if (c <= INBOX_CAP && nb + c <= 128) {
            u64 k[2];
            k[0] = lane < nb ? cur.r0 : KEY_PAD;
            k[1] = lane + 64 < nb ? cur.r1 : (63 - lane < c ? cur.in : KEY_PAD);
            wave_sort<2>(k, lane);
            nd = wave_unique_prefix<2>(k, lane, R, keys + (size_t)x * R, &any_new, &dropped);
        } else {
            const int ca = c < INBOX_CAP ? c : INBOX_CAP;
            nd = wave_merge_row(keys + (size_t)x * R, nb, inbox + (size_t)x * INBOX_CAP, ca,
                                bins + (c > ca ? binoff[x] : 0), c - ca, R, s_stage[wave], lane, &any_new, &dropped);
        }
        if (lane == 0) {
            deg[x] = nd;
            cnt[x] = 0;
            tcls[it] = any_new ? (int8_t)degree_class(nd, use_classes) : (int8_t)-1;
        }
        cur = nxt;
    }
    if (lane == 0 && dropped) atomicAdd(&ctr->stat[blockIdx.x & (STAT_SLOTS - 1)][4], (u64)dropped);
}

// All four merge classes in one launch: blockIdx.y = merge class (touched list y, tcls + y*N).
__global__ __launch_bounds__(BLOCK) void k_merge(long long N, int R, u64 *keys, int *deg, const int *tlists,
                                                 const u32 *n_touched, int *cnt, const u64 *inbox,
                                                 const int *binoff, const u64 *bins, int8_t *tcls,
                                                 int use_classes, RoundCtr *ctr)
{
    __shared__ u64 s_stage[WAVES_PER_BLOCK][RNND_MAX_R];
    const int y = blockIdx.y;
    const int *tlist = tlists + (size_t)y * N;
    int8_t *tc = tcls + (size_t)y * N;
    if (y == 0) merge_group_body<16>(R, keys, deg, tlist, n_touched + 0, cnt, inbox, tc, use_classes, ctr);
    else if (y == 1) merge_group_body<32>(R, keys, deg, tlist, n_touched + 1, cnt, inbox, tc, use_classes, ctr);
    else if (y == 2) merge_group_body<64>(R, keys, deg, tlist, n_touched + 2, cnt, inbox, tc, use_classes, ctr);
    else merge_general_body(R, keys, deg, tlist, n_touched + 3, cnt, inbox, binoff, bins, tc, use_classes, s_stage, ctr);
}

// Items i < n with cls[first + i] >= 0 are appended to list cls[first + i]; item i stands for vertex idx[i]
// (or first + i).  blockIdx.y = s selects source list s: n_ptr[s], idx + s*N, cls + s*N.  One atomic per class
// per 1024 items.  With `taken`, the class of every listed item is then cleared there (taken may be cls).
__global__ __launch_bounds__(1024) void k_compact_classes(const u32 *n_ptr, u32 n_fixed, const int *idx,
                                                          const int8_t *cls, int *lists, long long N,
                                                          u32 *n_out, u32 first, int8_t *taken)
{
    __shared__ u32 s_cnt[16][NDEG], s_base[NDEG];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u32 n = n_ptr ? n_ptr[blockIdx.y] : n_fixed;
    if (idx) idx += (size_t)blockIdx.y * N;
    cls += (size_t)blockIdx.y * N;
    for (u32 base = blockIdx.x * 1024u; base < n; base += gridDim.x * 1024u) {
        const u32 i = base + threadIdx.x;
        const int c = i < n ? (int)cls[first + i] : -1;
        u64 b[NDEG];
#pragma unroll
        for (int k = 0; k < NDEG; ++k) b[k] = __builtin_amdgcn_ballot_w64(c == k);
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < NDEG; ++k) s_cnt[wave][k] = (u32)__popcll(b[k]);
        }
        __syncthreads();
        if (threadIdx.x < NDEG) {
            u32 tot = 0;
            for (int w = 0; w < 16; ++w) { u32 a = s_cnt[w][threadIdx.x]; s_cnt[w][threadIdx.x] = tot; tot += a; }
            s_base[threadIdx.x] = tot ? atomicAdd(&n_out[threadIdx.x], tot) : 0u;
        }
        __syncthreads();
        if (c >= 0 && c < NDEG) {
            u64 mine = b[0];
#pragma unroll
            for (int k = 1; k < NDEG; ++k) mine = (c == k) ? b[k] : mine;
            const u32 off = s_base[c] + s_cnt[wave][c] + (u32)__popcll(mine & lanes_below(lane));
            lists[(size_t)c * N + off] = idx ? idx[i] : (int)(first + i);
            if (taken) taken[first + i] = (int8_t)-1;
        }
        __syncthreads();
    }
}

// Block-sequential passes keep the class of every vertex that holds a "new" entry in vcls[] between runs:
// after a run's merge, vcls[x] <- tcls of every touched vertex x (blockIdx.y = merge class).
__global__ __launch_bounds__(256) void k_store_classes(const u32 *n_touched, const int *tlists, const int8_t *tcls,
                                                       long long N, int8_t *vcls)
{
    const u32 n = n_touched[blockIdx.y];
    const int *tl = tlists + (size_t)blockIdx.y * N;
    const int8_t *tc = tcls + (size_t)blockIdx.y * N;
    for (u32 i = blockIdx.x * 256u + threadIdx.x; i < n; i += gridDim.x * 256u) vcls[tl[i]] = tc[i];
}

// ------------------------------------------------------------ AddReverseEdges
// The union and the out-degree cut of Alg. 5 need, for every x, the edges that point to x.  Every edge (u, v) takes an arrival
// number at v (one atomic on fill[v]); the first INBOX_CAP arrivals are written to v's inbox as
// key(delta, u, new).  A later arrival is remembered with its edge (late[] holds its number, over[u]
// one bit per list position of u, mark[u] says that u has any) and k_reverse_surplus places it in
// v's bin once bins exist.
// 16 lanes per vertex (lists are mostly short: a wavefront per vertex would leave most lanes idle and the
// kernel is bound by its three dependent trips to memory: degree, list entry, arrival number).
__global__ __launch_bounds__(BLOCK) void k_reverse_scatter(long long N, int R, const u64 *keys, const int *deg,
                                                           int *fill, u64 *inbox, u32 *late, u64 *over,
                                                           int8_t *mark)
{
    const int lane = threadIdx.x & 63, sub = lane & 15, gsh = lane & ~15;
    const long long u = ((long long)blockIdx.x * BLOCK + threadIdx.x) >> 4;
    const bool valid = u < N;
    const int m = valid ? deg[u] : 0;
    // the same number of trips for the four vertices of a wavefront (the ballot below is the wavefront's)
    int mmax = m;
    mmax = max(mmax, __shfl_xor(mmax, 16));
    mmax = max(mmax, __shfl_xor(mmax, 32));
    u64 ov[2] = {0ull, 0ull};
    for (int e0 = 0; e0 < mmax; e0 += 16) {
        const int e = e0 + sub;
        bool is_late = false;
        if (e < m) {
            const u64 k = keys[(size_t)u * R + e];
            const u32 v = key_id(k);
            const int a = atomicAdd(&fill[v], 1);
            if (a < INBOX_CAP) {
                inbox[(size_t)v * INBOX_CAP + a] = make_key(key_dist(k), (u32)u, 1u);
            } else {
                late[(size_t)u * R + e] = (u32)a;
                is_late = true;
            }
        }
        const u64 bits = (__builtin_amdgcn_ballot_w64(is_late) >> gsh) & 0xFFFFull;     // my vertex's 16 positions
        ov[e0 >> 6] |= bits << (e0 & 63);
    }
    if (valid && sub == 0) {
        const bool any = (ov[0] | ov[1]) != 0;
        mark[u] = (int8_t)any;
        if (any) { over[2 * u] = ov[0]; over[2 * u + 1] = ov[1]; }
    }
}

// The late arrivals of k_reverse_scatter go to their targets' bins (which hold arrivals INBOX_CAP, ...).
__global__ __launch_bounds__(BLOCK) void k_reverse_surplus(long long N, int R, const u64 *keys, const u32 *late,
                                                           const u64 *over, const int8_t *mark,
                                                           const int *binoff, u64 *bins, const u32 *n_binned)
{
    if (*n_binned == 0u) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long u = (long long)blockIdx.x * WAVES_PER_BLOCK + wave;
    if (u >= N || !mark[u]) return;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const u64 ov = over[2 * u + r];
        if ((ov >> lane) & 1ull) {
            const int e = 64 * r + lane;
            const u64 k = keys[(size_t)u * R + e];
            const u32 v = key_id(k);
            bins[(size_t)binoff[v] + (late[(size_t)u * R + e] - INBOX_CAP)] = make_key(key_dist(k), (u32)u, 1u);
        }
    }
}

// ---- the same transposition without one device-scope atomic per edge (large N) -------------------------
// Targets are cut into ranges of RANGE_TARGETS consecutive ids.  Every block of BIN_CHUNK source vertices
// counts its edges per range in LDS (k_bin_count); a column-wise prefix over the blocks turns the counts into
// the place of every (block, range) run in one edge array ordered by range (k_bin_offsets, k_bin_bases: no
// atomics, the layout is a pure function of the graph); the blocks copy their edges there, taking ranks from
// LDS counters (k_bin_partition); then one workgroup per range, which alone owns its targets, counts the edges
// of each target in LDS, hands out the surplus bins, and moves every edge into its target's inbox or bin with
// arrival numbers from the LDS counters (k_bin_place).  What k_reverse_scatter, the first k_assign_bins and
// k_reverse_surplus leave behind -- fill[], inbox, binoff[], bins, cand[], zeroed cnt[] and cnt_in[] -- is
// left in the same form (slot order inside an inbox is arbitrary in both; every consumer sorts).
#define RANGE_BITS 11
#define RANGE_TARGETS (1 << RANGE_BITS)
#define RANGE_MAX 16384       // ranges a block can histogram in LDS (64 KB): N <= RANGE_MAX * RANGE_TARGETS
#define BIN_CHUNK 2048        // source vertices per block of the count and partition kernels
#define BIN_THREADS 1024

// Walks the edges of the block's BIN_CHUNK source vertices: thread t of a pass takes list position t % 16 of
// vertex t / 16 (lists are short on average; longer ones take further trips), four vertices per thread in
// flight.  f(u, key) is called once per edge.
template <typename F>
__device__ __forceinline__ void for_each_edge_of_chunk(long long N, int W, const u64 *__restrict__ keys,
                                                       const int *__restrict__ deg, F f)
{
    const int sub = threadIdx.x & 15, grp = threadIdx.x >> 4;      // 64 groups of 16 lanes
    const long long u0 = (long long)blockIdx.x * BIN_CHUNK;
    constexpr int GROUPS = BIN_THREADS / 16, UNROLL = 4;
    for (int i = grp; i < BIN_CHUNK; i += GROUPS * UNROLL) {
        long long u[UNROLL];
        int m[UNROLL];
        u64 k[UNROLL];
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) {
            u[j] = u0 + i + j * GROUPS;
            m[j] = (i + j * GROUPS < BIN_CHUNK && u[j] < N) ? deg[u[j]] : 0;
        }
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) k[j] = sub < m[j] ? keys[(size_t)u[j] * W + sub] : 0ull;
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) {
            if (sub < m[j]) f(u[j], k[j]);
            for (int e = sub + 16; e < m[j]; e += 16) f(u[j], keys[(size_t)u[j] * W + e]);
        }
    }
}

__global__ __launch_bounds__(BIN_THREADS) void k_bin_count(long long N, int W, const u64 *__restrict__ keys,
                                                           const int *__restrict__ deg, u32 nranges, u32 *__restrict__ blockhist)
{
    __shared__ u32 hist[RANGE_MAX];
    for (u32 r = threadIdx.x; r < nranges; r += BIN_THREADS) hist[r] = 0;
    __syncthreads();
    for_each_edge_of_chunk(N, W, keys, deg, [&](long long, u64 k) { atomicAdd(&hist[key_id(k) >> RANGE_BITS], 1u); });
    __syncthreads();
    u32 *out = blockhist + (size_t)blockIdx.x * nranges;
    for (u32 r = threadIdx.x; r < nranges; r += BIN_THREADS) out[r] = hist[r];
}

// blockhist[b][r] <- edges of range r in the blocks before b; range_tot[r] <- edges of range r in all.
// A workgroup takes 64 ranges; its 16 wavefronts each take a slice of consecutive blocks (a wavefront reads
// 64 consecutive counters of one block at a time), sum it, and after a prefix over the slices walk it again.
__global__ __launch_bounds__(1024) void k_bin_offsets(u32 nblocks, u32 nranges, u32 *__restrict__ blockhist,
                                                      u32 *__restrict__ range_tot)
{
    __shared__ u32 s_sum[16][64];
    const u32 col = threadIdx.x & 63, slice = threadIdx.x >> 6;
    const u32 r = blockIdx.x * 64 + col;
    const bool have = r < nranges;
    const u32 per = (nblocks + 15) / 16;
    const u32 b0 = slice * per < nblocks ? slice * per : nblocks, b1 = b0 + per < nblocks ? b0 + per : nblocks;
    u32 sum = 0;
    if (have) {
        u32 b = b0;
        for (; b + 4 <= b1; b += 4) {
            const u32 c0 = blockhist[(size_t)b * nranges + r], c1 = blockhist[(size_t)(b + 1) * nranges + r];
            const u32 c2 = blockhist[(size_t)(b + 2) * nranges + r], c3 = blockhist[(size_t)(b + 3) * nranges + r];
            sum += c0 + c1 + c2 + c3;
        }
        for (; b < b1; ++b) sum += blockhist[(size_t)b * nranges + r];
    }
    s_sum[slice][col] = sum;
    __syncthreads();
    u32 run = 0, all = 0;
    for (u32 sl = 0; sl < 16; ++sl) {
        const u32 v = s_sum[sl][col];
        run += sl < slice ? v : 0u;
        all += v;
    }
    if (have) {
        if (slice == 0) range_tot[r] = all;
        u32 b = b0;
        for (; b + 4 <= b1; b += 4) {
            const u32 c0 = blockhist[(size_t)b * nranges + r], c1 = blockhist[(size_t)(b + 1) * nranges + r];
            const u32 c2 = blockhist[(size_t)(b + 2) * nranges + r], c3 = blockhist[(size_t)(b + 3) * nranges + r];
            blockhist[(size_t)b * nranges + r] = run;
            blockhist[(size_t)(b + 1) * nranges + r] = run + c0;
            blockhist[(size_t)(b + 2) * nranges + r] = run + c0 + c1;
            blockhist[(size_t)(b + 3) * nranges + r] = run + c0 + c1 + c2;
            run += c0 + c1 + c2 + c3;
        }
        for (; b < b1; ++b) {
            const u32 c = blockhist[(size_t)b * nranges + r];
            blockhist[(size_t)b * nranges + r] = run;
            run += c;
        }
    }
}

// range_base[r] <- edges of the ranges before r (one block; nranges <= RANGE_MAX); range_base[nranges] <- all.
__global__ __launch_bounds__(1024) void k_bin_bases(u32 nranges, const u32 *__restrict__ range_tot, u32 *__restrict__ range_base)
{
    __shared__ u32 s_w[16];
    constexpr int PER = RANGE_MAX / 1024;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    u32 v[PER], mine = 0;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const u32 r = threadIdx.x * PER + k;
        v[k] = r < nranges ? range_tot[r] : 0u;
        mine += v[k];
    }
    u32 incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const u32 t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    if (lane == 63) s_w[wave] = incl;
    __syncthreads();
    u32 before = 0;
    for (int w = 0; w < wave; ++w) before += s_w[w];
    u32 run = before + incl - mine;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const u32 r = threadIdx.x * PER + k;
        if (r < nranges) range_base[r] = run;
        run += v[k];
    }
    if (threadIdx.x == 1023) range_base[nranges] = run;
}

// Edge (u, v) -> part[place of (my block, range of v) + rank inside it] = { key(delta, u, new), v }.
__global__ __launch_bounds__(BIN_THREADS) void k_bin_partition(long long N, int W, const u64 *__restrict__ keys,
                                                               const int *__restrict__ deg, u32 nranges,
                                                               const u32 *__restrict__ blockhist,
                                                               const u32 *__restrict__ range_base, Prop *__restrict__ part)
{
    __shared__ u32 cursor[RANGE_MAX];
    const u32 *mine = blockhist + (size_t)blockIdx.x * nranges;
    for (u32 r = threadIdx.x; r < nranges; r += BIN_THREADS) cursor[r] = range_base[r] + mine[r];
    __syncthreads();
    for_each_edge_of_chunk(N, W, keys, deg, [&](long long u, u64 k) {
        const u32 v = key_id(k);
        const u32 at = atomicAdd(&cursor[v >> RANGE_BITS], 1u);
        Prop pr;
        pr.key = make_key(key_dist(k), (u32)u, 1u);
        pr.tgt = v;
        pr.arrival = 0;
        part[at] = pr;
    });
}

// One workgroup per range of targets.  One sweep over the range's edges numbers the arrivals per target in LDS
// and writes the first INBOX_CAP of each target straight into its inbox; later arrivals (hubs: rare) wait in an
// LDS stash until the sweep has counted every target and the surplus bins are handed out.  A range whose
// stash overflows is swept again with the bins known, rewriting every place.
#define PLACE_THREADS 512
#define PLACE_STASH 2048
__global__ __launch_bounds__(PLACE_THREADS) void k_bin_place(long long N, int R, const Prop *__restrict__ part,
                                                             const u32 *__restrict__ range_base, const int *__restrict__ deg,
                                                             int *__restrict__ fill, u64 *__restrict__ inbox,
                                                             int *__restrict__ binoff, u64 *__restrict__ bins,
                                                             u32 *__restrict__ bin_cursor, int *__restrict__ zero_a,
                                                             int *__restrict__ zero_b, int8_t *__restrict__ cand)
{
    __shared__ u32 arr[RANGE_TARGETS], bin_at[RANGE_TARGETS];
    __shared__ u64 st_key[PLACE_STASH];
    __shared__ u32 st_tgt[PLACE_STASH], st_arr[PLACE_STASH];
    __shared__ u32 s_w[PLACE_THREADS / 64], s_base, s_stash;
    constexpr int PER = RANGE_TARGETS / PLACE_THREADS, NW = PLACE_THREADS / 64, UNROLL = 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u32 first = blockIdx.x << RANGE_BITS;          // first target of my range
    const u32 e0 = range_base[blockIdx.x], e1 = range_base[blockIdx.x + 1];
#pragma unroll
    for (int k = 0; k < PER; ++k) arr[threadIdx.x * PER + k] = 0;
    if (threadIdx.x == 0) s_stash = 0;
    __syncthreads();
    // pass == 0: arrivals below INBOX_CAP to the inbox, later ones to the stash.  pass == 1 (only after a stash
    // overflow): every edge again, surplus straight to the bins.
    auto sweep = [&](const int pass) {
        for (u32 e = e0 + threadIdx.x; e < e1; e += PLACE_THREADS * UNROLL) {
            Prop pr[UNROLL];
#pragma unroll
            for (int j = 0; j < UNROLL; ++j) {
                pr[j].tgt = 0xFFFFFFFFu;
                if (e + j * PLACE_THREADS < e1) pr[j] = part[e + j * PLACE_THREADS];
            }
#pragma unroll
            for (int j = 0; j < UNROLL; ++j) {
                if (pr[j].tgt == 0xFFFFFFFFu) continue;
                const u32 t = pr[j].tgt - first;
                const u32 a = atomicAdd(&arr[t], 1u);
                if (a < (u32)INBOX_CAP) {
                    inbox[(size_t)pr[j].tgt * INBOX_CAP + a] = pr[j].key;
                } else if (pass == 1) {
                    bins[(size_t)bin_at[t] + (a - INBOX_CAP)] = pr[j].key;
                } else {
                    const u32 at = atomicAdd(&s_stash, 1u);
                    if (at < (u32)PLACE_STASH) { st_key[at] = pr[j].key; st_tgt[at] = t; st_arr[at] = a; }
                }
            }
        }
    };
    sweep(0);
    __syncthreads();
    // per target: the count, the candidate mark of the in-degree cut, cleared counters, a bin for the surplus
    u32 c[PER], surplus[PER], mine = 0;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        c[k] = arr[threadIdx.x * PER + k];
        surplus[k] = c[k] > (u32)INBOX_CAP ? c[k] - (u32)INBOX_CAP : 0u;
        mine += surplus[k];
    }
    u32 incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const u32 t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    if (lane == 63) s_w[wave] = incl;
    __syncthreads();
    if (threadIdx.x == 0) {
        u32 tot = 0;
        for (int w = 0; w < NW; ++w) { const u32 a = s_w[w]; s_w[w] = tot; tot += a; }
        s_base = tot ? atomicAdd(bin_cursor, tot) : 0u;
    }
    __syncthreads();
    u32 run = s_base + s_w[wave] + incl - mine;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const long long v = (long long)first + threadIdx.x * PER + k;
        if (v < N) {
            fill[v] = (int)c[k];
            zero_a[v] = 0;
            zero_b[v] = 0;
            cand[v] = (int8_t)(deg[v] + (int)c[k] > R);
            binoff[v] = surplus[k] ? (int)run : -1;
        }
        bin_at[threadIdx.x * PER + k] = run;     // where the target's bin starts (if it has one)
        run += surplus[k];
    }
    __syncthreads();
    const u32 stashed = s_stash;
    if (stashed <= (u32)PLACE_STASH) {
        for (u32 i = threadIdx.x; i < stashed; i += PLACE_THREADS)
            bins[(size_t)bin_at[st_tgt[i]] + (st_arr[i] - INBOX_CAP)] = st_key[i];
    } else {
#pragma unroll
        for (int k = 0; k < PER; ++k) arr[threadIdx.x * PER + k] = 0;
        __syncthreads();
        sweep(1);
    }
}

// For every edge (u, v) of a flagged list whose v owns a bin: bins[v] <- key(delta, u, flag).  The flagged
// vertices come as a list (one wavefront per vertex).  Nothing to do when no bin was handed out (*n_binned == 0).
__global__ __launch_bounds__(BLOCK) void k_fill_bins(int R, const u64 *keys, const int *deg, const int *flagged,
                                                     const u32 *n_flagged, const int *binoff, int *fill,
                                                     u64 *bins, u32 flag, const u32 *n_binned)
{
    if (*n_binned == 0u) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const u32 n = *n_flagged, nw = gridDim.x * WAVES_PER_BLOCK;
    for (u32 it = blockIdx.x * WAVES_PER_BLOCK + wave; it < n; it += nw) {
        const int u = flagged[it];
        const int m = deg[u];
        for (int e = lane; e < m; e += 64) {
            const u64 k = keys[(size_t)u * R + e];
            const u32 v = key_id(k);
            const int off = binoff[v];
            if (off >= 0) bins[(size_t)off + atomicAdd(&fill[v], 1)] = make_key(key_dist(k), (u32)u, flag);
        }
    }
}

// Alg. 5, union and out-degree cut: list(x) <- first R distinct of list(x) + reversed edges into x (flag new).
// Then the edges of the new list are counted at those targets that can end up with more than R
// incoming edges (cand[v]: |list(v)| + |edges into v| > R before the union; for every other vertex
// the union itself bounds the in-degree by R); rowflag[x] = 0 if the list has such an edge, else -1.
// vcls[x] <- degree class if the list holds a "new" entry, else -1.
struct RevItem {       // what a half-wave holds of its vertex before it is that vertex's turn
    int c, nb;         // reversed edges received, entries held
    u64 kr, ki;        // list slot l32, inbox slot 31 - l32 (either may be garbage: masked by nb, c)
};

__device__ __forceinline__ RevItem rev_item_load(long long x, long long N, int W, const u64 *keys, const int *deg,
                                                 const int *fill, const u64 *inbox, int l32)
{
    // past the last vertex, vertex 0 is read instead and given nothing: loads without branches
    RevItem it;
    const size_t xx = x < N ? (size_t)x : 0;
    const int c = fill[xx], nb = deg[xx];
    it.c = x < N ? c : 0;
    it.nb = x < N ? nb : 0;
    it.kr = keys[xx * W + (l32 < W ? l32 : W - 1)];
    it.ki = inbox[xx * INBOX_CAP + (31 - l32)];
    return it;
}

__global__ __launch_bounds__(BLOCK) void k_reverse_merge(long long N, int W, int R, u64 *keys, int *deg, int *fill,
                                                         const u64 *inbox, const int *binoff, const u64 *bins,
                                                         const int8_t *cand, int *cnt_in, int8_t *rowflag,
                                                         int8_t *vcls, int use_classes)
{   // rows are W slots apart (W >= R); lists are cut to R
    __shared__ u64 s_stage[WAVES_PER_BLOCK][RNND_MAX_R];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    // a wavefront takes two vertices at a time, one per half: lists are short on average, and when both unions
    // have at most 32 keys they are formed side by side (32-lane sorts); otherwise one after the other.  The
    // grid is persistent: what the next pair needs in the short case is loaded before the current pair is sorted.
    const long long npairs = (N + 1) / 2;
    const long long gw = (long long)blockIdx.x * WAVES_PER_BLOCK + wave, nw = (long long)gridDim.x * WAVES_PER_BLOCK;
    if (gw >= npairs) return;
    RevItem cur = rev_item_load(2 * gw + half, N, W, keys, deg, fill, inbox, l32);
    for (long long pair = gw; pair < npairs; pair += nw) {
        const RevItem nxt = rev_item_load(2 * (pair + nw) + half, pair + nw < npairs ? N : 0, W, keys, deg, fill, inbox, l32);
        const long long x0 = 2 * pair, xh = x0 + half;
        const bool have = xh < N;
        const int ch = cur.c, nbh = cur.nb;
        const bool small = __builtin_amdgcn_ballot_w64(nbh + ch > 32) == 0;
        if (small) {
            u64 *row = keys + (size_t)xh * W;
            u64 k = KEY_PAD;
            if (have) {
                if (l32 < nbh) k = cur.kr;
                else if (31 - l32 < ch) k = cur.ki;
            }
            k = group_sort<32>(k, lane);
            u64 prev = shfl_up1_u64(k);
            if (l32 == 0) prev = KEY_PAD;
            const bool keep = (k != KEY_PAD) && ((k >> 1) != (prev >> 1));
            const u32 m = (u32)(__builtin_amdgcn_ballot_w64(keep) >> (32 * half));
            const int pos = __popc(m & ((1u << l32) - 1u));
            const bool w = keep && pos < R;
            if (w) row[pos] = k;
            bool cd = false;
            if (w) {
                const u32 v = key_id(k);
                if (cand[v]) {
                    atomicAdd(&cnt_in[v], 1);
                    cd = true;
                }
            }
            const u32 nm = (u32)(__builtin_amdgcn_ballot_w64(w && (k & 1ull)) >> (32 * half));
            const u32 cm = (u32)(__builtin_amdgcn_ballot_w64(cd) >> (32 * half));
            if (have && l32 == 0) {
                int nd = __popc(m);
                if (nd > R) nd = R;
                deg[xh] = nd;
                fill[xh] = 0;
                rowflag[xh] = (int8_t)(cm != 0 ? 0 : -1);      // class 0 of a compaction = the flagged vertices
                vcls[xh] = nm ? (int8_t)degree_class(nd, use_classes) : (int8_t)-1;
            }
        } else {
            for (int h = 0; h < 2; ++h) {
                const long long x = x0 + h;
                if (x >= N) break;
                u64 *row = keys + (size_t)x * W;
                const int c = __shfl(ch, 32 * h);
                int nd = __shfl(nbh, 32 * h);
                if (c == 0 && nd > R) nd = R;   // Alg. 5 cuts every out-list to its R shortest; the row is sorted and distinct
                if (c > 0) {
                    bool any_new;
                    const int ca = c < INBOX_CAP ? c : INBOX_CAP;
                    wave_sync();    // the staging area may still be read by the previous vertex
                    nd = wave_merge_row(row, nd, inbox + (size_t)x * INBOX_CAP, ca, bins + (c > ca ? binoff[x] : 0), c - ca, R,
                                        s_stage[wave], lane, &any_new);
                    wave_sync();    // the list is read back below by other lanes of this wavefront
                }
                bool nw_ = false, cd = false;
                for (int e = lane; e < nd; e += 64) {
                    const u64 k = row[e];
                    nw_ = nw_ || (k & 1ull);
                    const u32 v = key_id(k);
                    if (cand[v]) {
                        atomicAdd(&cnt_in[v], 1);
                        cd = true;
                    }
                }
                const u64 bn = __builtin_amdgcn_ballot_w64(nw_), bc = __builtin_amdgcn_ballot_w64(cd);
                if (lane == 0) {
                    deg[x] = nd;
                    fill[x] = 0;
                    rowflag[x] = (int8_t)(bc != 0 ? 0 : -1);
                    vcls[x] = bn ? (int8_t)degree_class(nd, use_classes) : (int8_t)-1;
                }
            }
        }
        cur = nxt;
    }
}

// Alg. 5, in-degree cut, first half: thr[v] <- the R-th smallest (delta, source) among the edges into v.
__global__ __launch_bounds__(BLOCK) void k_incap_threshold(int R, const int *list, const u32 *n_list,
                                                           const int *cnt, const int *binoff,
                                                           const u64 *bins, u64 *thr)
{
    __shared__ u64 s_stage[WAVES_PER_BLOCK][RNND_MAX_R];
    __shared__ u64 s_row[WAVES_PER_BLOCK][RNND_MAX_R];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const u32 gw = blockIdx.x * WAVES_PER_BLOCK + wave, nw = gridDim.x * WAVES_PER_BLOCK;
    const u32 n = *n_list;
    for (u32 it = gw; it < n; it += nw) {
        const int v = list[it];
        bool any_new;
        wave_sync();
        const int nd = wave_merge_row(s_row[wave], 0, bins + binoff[v], cnt[v], bins, 0, R, s_stage[wave],
                                      lane, &any_new);
        wave_sync();
        if (lane == 0) thr[v] = s_row[wave][nd - 1];
    }
}

// Alg. 5, in-degree cut, second half: edge (u, v) survives iff (delta, u) <= thr[v]; vcls[u] follows the
// new degree.  Only the flagged lists (those with an edge to a candidate) can lose an edge; they come as a list.
// Nothing to do when no vertex has more than R incoming edges (*n_hubs == 0).
__global__ __launch_bounds__(BLOCK) void k_incap_filter(int R, u64 *keys, int *deg, const u64 *thr,
                                                        const int *flagged, const u32 *n_flagged, int8_t *vcls,
                                                        int use_classes, const u32 *n_hubs)
{
    if (*n_hubs == 0u) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const u32 n = *n_flagged, nw = gridDim.x * WAVES_PER_BLOCK;
    for (u32 it = blockIdx.x * WAVES_PER_BLOCK + wave; it < n; it += nw) {
        const int u = flagged[it];
        const int m = deg[u];
        u64 *row = keys + (size_t)u * R;
        u64 k[2];
        bool keep[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            int e = r * 64 + lane;
            k[r] = e < m ? row[e] : KEY_PAD;
            keep[r] = e < m && make_key(key_dist(k[r]), (u32)u, 0u) <= thr[key_id(k[r])];
        }
        const u64 m0 = __builtin_amdgcn_ballot_w64(keep[0]), m1 = __builtin_amdgcn_ballot_w64(keep[1]);
        const u64 n0 = __builtin_amdgcn_ballot_w64(keep[0] && (k[0] & 1ull));
        const u64 n1 = __builtin_amdgcn_ballot_w64(keep[1] && (k[1] & 1ull));
        const int c0 = __popcll(m0);
        if (keep[0]) row[__popcll(m0 & lanes_below(lane))] = k[0];
        if (keep[1]) row[c0 + __popcll(m1 & lanes_below(lane))] = k[1];
        if (lane == 0) {
            const int nd = c0 + __popcll(m1);
            deg[u] = nd;
            vcls[u] = (n0 | n1) ? (int8_t)degree_class(nd, use_classes) : (int8_t)-1;
        }
    }
}

__global__ void k_zero_u32(u32 *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0;
}

// vcls[u] for a snapshot handed in by the caller
__global__ __launch_bounds__(BLOCK) void k_classify(long long N, int R, const u64 *keys, const int *deg,
                                                    int8_t *vcls, int use_classes)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long u = (long long)blockIdx.x * WAVES_PER_BLOCK + wave;
    if (u >= N) return;
    int m = deg[u];
    if (m > R) m = R;
    bool nw = false;
    for (int e = lane; e < m; e += 64) nw = nw || (keys[(size_t)u * R + e] & 1ull);
    const u64 b = __builtin_amdgcn_ballot_w64(nw);
    if (lane == 0) vcls[u] = b ? (int8_t)degree_class(m, use_classes) : (int8_t)-1;
}

__global__ void k_export(long long N, int R, const u64 *keys, const int *deg, int *graph_out,
                         int *degree_out)
{
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N * R) return;
    long long u = i / R;
    int e = (int)(i - u * R);
    int m = deg[u];
    graph_out[i] = e < m ? (int)key_id(keys[i]) : -1;
    if (e == 0) degree_out[u] = m;
}

// The same, four slots per thread (R a multiple of 4, graph_out 16-byte aligned).
__global__ __launch_bounds__(256) void k_export4(long long N, int R4, const u64 *keys, const int *deg, int4 *graph_out,
                                                 int *degree_out)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;      // group of four slots
    if (i >= N * R4) return;
    const long long u = i / R4;
    const int e = 4 * (int)(i - u * R4);
    const int m = deg[u];
    int4 o = make_int4(-1, -1, -1, -1);
    if (e < m) {
        const ulonglong2 a = ((const ulonglong2 *)keys)[2 * i], b = ((const ulonglong2 *)keys)[2 * i + 1];
        o.x = (int)key_id(a.x);
        if (e + 1 < m) o.y = (int)key_id(a.y);
        if (e + 2 < m) o.z = (int)key_id(b.x);
        if (e + 3 < m) o.w = (int)key_id(b.y);
    }
    graph_out[i] = o;
    if (e == 0) degree_out[u] = m;
}

static void launch_export(long long N, int R, const u64 *keys, const int *deg, int *graph_out, int *degree_out,
                          hipStream_t st)
{
    if (R % 4 == 0 && ((uintptr_t)graph_out & 15) == 0 && ((uintptr_t)keys & 15) == 0)
        hipLaunchKernelGGL(k_export4, dim3((unsigned)(((size_t)N * (R / 4) + 255) / 256)), dim3(256), 0, st, N, R / 4, keys,
                           deg, (int4 *)graph_out, degree_out);
    else
        hipLaunchKernelGGL(k_export, dim3((unsigned)(((size_t)N * R + 255) / 256)), dim3(256), 0, st, N, R, keys, deg,
                           graph_out, degree_out);
}

// Measurement aid: random row gathers and nothing else.  Every wavefront draws row numbers from the
// counter generator and reads whole rows, LPR lanes per row with 16 bytes per lane and piece, four
// rows' worth of loads per lane in flight; the values are folded into one word per thread so that
// the loads cannot be dropped.  This is the access pattern of the scan kernels without their work.
template <int LPR>
__global__ __launch_bounds__(256) void k_probe_gather(const uint4 *X, u32 n_rows, u32 pieces, u64 trips, u64 seed, u32 *sink)
{
    constexpr int RPI = 64 / LPR;       // rows per load instruction
    const int lane = threadIdx.x & 63, r = lane / LPR, q = lane % LPR;
    const u64 gw = ((u64)blockIdx.x * 256 + threadIdx.x) >> 6, nw = ((u64)gridDim.x * 256) >> 6;
    u32 acc = 0;
    for (u64 t = gw; t < trips; t += nw) {
        const uint4 *p[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const u64 z = splitmix_finish(seed + 0x9E3779B97F4A7C15ull * (t * (4 * RPI) + (u64)(k * RPI + r) + 1));
            const u32 row = (u32)(((z >> 32) * (u64)n_rows) >> 32);
            p[k] = X + (size_t)row * pieces + q;
        }
        for (u32 c = 0; c < pieces; c += LPR) {
            uint4 v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] = p[k][c];
#pragma unroll
            for (int k = 0; k < 4; ++k) acc ^= v[k].x + v[k].y + v[k].z + v[k].w;
        }
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = acc;
}

// The same with the lane -> address map as the only variable: LPR lanes per row, each reading its PPL pieces
// of the row (16 bytes, LPR pieces apart), 8 / PPL rows per lane: 8 loads of 16 bytes per lane in flight
// whatever the map, all issued before the first is used.
template <int LPR, int PPL>
__global__ __launch_bounds__(256) void k_probe_gather_map(const uint4 *X, u32 n_rows, u64 trips, u64 seed, u32 *sink)
{
    constexpr int RPI = 64 / LPR, ROWS = 8 / PPL;
    const int lane = threadIdx.x & 63, r = lane / LPR, q = lane % LPR;
    const u64 gw = ((u64)blockIdx.x * 256 + threadIdx.x) >> 6, nw = ((u64)gridDim.x * 256) >> 6;
    u32 acc = 0;
    for (u64 t = gw; t < trips; t += nw) {
        uint4 v[ROWS][PPL];
#pragma unroll
        for (int k = 0; k < ROWS; ++k) {
            const u64 z = splitmix_finish(seed + 0x9E3779B97F4A7C15ull * (t * (ROWS * RPI) + (u64)(k * RPI + r) + 1));
            const u32 row = (u32)(((z >> 32) * (u64)n_rows) >> 32);
            const uint4 *p = X + (size_t)row * (LPR * PPL) + q;
#pragma unroll
            for (int j = 0; j < PPL; ++j) v[k][j] = p[j * LPR];
        }
#pragma unroll
        for (int k = 0; k < ROWS; ++k)
#pragma unroll
            for (int j = 0; j < PPL; ++j) acc ^= v[k][j].x + v[k][j].y + v[k][j].z + v[k][j].w;
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = acc;
}

// ===================================================================== host side
#define HIPCHK(x)                                                                  \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            snprintf(g_last_hip_error, sizeof g_last_hip_error, "%s: %s", #x, hipGetErrorString(e_)); \
            rc = (e_ == hipErrorOutOfMemory) ? RNND_ERR_OOM : RNND_ERR_HIP;        \
            (void)hipGetLastError();   /* reported here: must not surface again in a later call */ \
            goto done;                                                             \
        }                                                                          \
    } while (0)

static char g_last_hip_error[512];
static int g_kernel_variant = 0;
static int g_event_timing = 0;    // 1: per-round times of the statistics from HIP events attached to the launches
static int g_transpose_path = 0;   // AddReverseEdges' transposition: 0 by size, 1 atomics, 2 binned
static int g_scan_launches = 0;    // uint8 matrix-core scan: 0 by size, 1 short lists + one launch per longer class, 2 one launch for all, 3 short lists + one launch for all longer classes
#define SMALL_INPUT_MAX_N 524288   // up to here one launch for all classes is the fastest form (measured, whole build against
                                   // launches per class: 0.75 x at 50,000 vertices, 0.78 x at 100,000, 0.90 x at 300,000, 0.955 x
                                   // at 500,000; 1.02 x at 1M, where it wins only in rounds with fewer than 250,000 active lists).
                                   // Above: the short-list launch and one launch for all longer classes (0.99 x at 1M)
#define LONG_SHARED_MAX_N 2097152  // ... up to here (1.00 x at 2M, 1.01 x at 4M, 1.00 x at 8M, 1.01 x at 20M: no start-up left to
                                   // share, and each class alone gets the occupancy that suits it); above: a launch per class
                                   // (bench.py names the round's scan launches by the same rule; include/rnnd.h states it)
#define BIN_MIN_N 262144            // below this the binned transposition's extra launches cost more than its atomics save

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

struct Workspace {
    char *base = nullptr;
    size_t bytes = 0;
    u64 *keys = nullptr;    // [N*R]   (unless the caller supplies a snapshot)
    int *deg = nullptr;     // [N]
    Prop *props = nullptr;  // [N*R]   slot u*R.. holds the edges vertex u redirected this round
    u64 *inbox = nullptr;   // [N*INBOX_CAP] redirected edges received this round, by target
    u64 *bins = nullptr;    // [N*R]   surplus of the inboxes; AddReverseEdges' bins
    u64 *thr = nullptr;     // [N]
    int *cnt = nullptr, *binoff = nullptr, *fill = nullptr, *touched = nullptr, *hubs = nullptr, *nprop = nullptr;
    int8_t *xs = nullptr;     // X - 128 as int8 (uint8 MFMA scan)
    int *lists = nullptr;   // [NDEG*N] active lists by degree class
    int8_t *vcls = nullptr, *tcls = nullptr;   // [N], [NMRG*N]
    RoundCtr *ctr = nullptr;   // [n_ctr]
    u32 *misc = nullptr;       // [16]: small cursors for AddReverseEdges
    u32 *blockhist = nullptr;  // binned transposition: [blocks of BIN_CHUNK vertices][ranges], null when N is out of its range
    u32 *range_tot = nullptr, *range_base = nullptr;   // [RANGE_MAX + 1] each
    int n_ctr = 0;
    // cnt[], fill[] and ctr[] must read zero when a call starts; they lie next to each other so that one
    // fill kernel clears them (ws_clear)
    u32 *zero_begin = nullptr;
    size_t zero_words = 0;
};

static size_t bin_blocks(long long N) { return (size_t)((N + BIN_CHUNK - 1) / BIN_CHUNK); }
static size_t bin_ranges(long long N) { return (size_t)((N + RANGE_TARGETS - 1) >> RANGE_BITS); }

static size_t ws_layout(Workspace &w, long long N, int R, int n_ctr, bool own_graph, size_t xs_bytes)
{
    size_t off = 0;
    auto take = [&](size_t b) { size_t o = off; off += align_up(b); return o; };
    size_t o_keys = own_graph ? take((size_t)N * R * 8) : 0;
    size_t o_deg = own_graph ? take((size_t)N * 4) : 0;
    size_t o_inbox = take((size_t)N * INBOX_CAP * 8);
    size_t o_props = take((size_t)N * R * sizeof(Prop));
    size_t o_bins = take((size_t)N * R * 8);
    size_t o_thr = take((size_t)N * 8);
    size_t o_binoff = take((size_t)N * 4);
    size_t o_touched = take((size_t)N * 4 * NMRG), o_hubs = take((size_t)N * 4), o_nprop = take((size_t)N * 4);
    size_t o_xs = take(xs_bytes);
    size_t o_lists = take((size_t)N * 4 * NDEG);
    size_t o_vcls = take((size_t)N), o_tcls = take((size_t)N * NMRG);
    size_t o_misc = take(16 * 4);
    const bool binnable = N >= 2 && (unsigned long long)N <= (unsigned long long)RANGE_MAX * RANGE_TARGETS;
    size_t o_range = take(binnable ? (size_t)2 * (RANGE_MAX + 1) * 4 : 0);
    size_t o_blockhist = take(binnable ? bin_blocks(N) * bin_ranges(N) * 4 : 0);
    size_t o_cnt = take((size_t)N * 4), o_fill = take((size_t)N * 4);      // the zeroed span: cnt, fill, ctr
    size_t o_ctr = take((size_t)n_ctr * sizeof(RoundCtr));
    if (w.base) {
        if (own_graph) { w.keys = (u64 *)(w.base + o_keys); w.deg = (int *)(w.base + o_deg); }
        w.inbox = (u64 *)(w.base + o_inbox);
        w.props = (Prop *)(w.base + o_props);
        w.nprop = (int *)(w.base + o_nprop);
        w.bins = (u64 *)(w.base + o_bins);
        w.thr = (u64 *)(w.base + o_thr);
        w.cnt = (int *)(w.base + o_cnt);
        w.binoff = (int *)(w.base + o_binoff);
        w.fill = (int *)(w.base + o_fill);
        w.touched = (int *)(w.base + o_touched);
        w.hubs = (int *)(w.base + o_hubs);
        w.xs = (int8_t *)(w.base + o_xs);
        w.lists = (int *)(w.base + o_lists);
        w.vcls = (int8_t *)(w.base + o_vcls);
        w.tcls = (int8_t *)(w.base + o_tcls);
        w.ctr = (RoundCtr *)(w.base + o_ctr);
        w.misc = (u32 *)(w.base + o_misc);
        w.blockhist = binnable ? (u32 *)(w.base + o_blockhist) : nullptr;
        w.range_tot = (u32 *)(w.base + o_range);
        w.range_base = w.range_tot + (RANGE_MAX + 1);
        w.n_ctr = n_ctr;
        w.zero_begin = (u32 *)(w.base + o_cnt);
        w.zero_words = (off - o_cnt) / 4;
    }
    return off;
}

// Every entry point clears the counters of its workspace with this before its first kernel: a fill kernel,
// not a memset node, so that the same sequence stays valid inside a captured graph.
static void ws_clear(const Workspace &w, hipStream_t st)
{
    const size_t n = w.zero_words;
    const unsigned blocks = (unsigned)((n + 1023) / 1024 < 2048 ? (n + 1023) / 1024 : 2048);
    hipLaunchKernelGGL(k_zero_u32, dim3(blocks ? blocks : 1), dim3(256), 0, st, w.zero_begin, n);
}

static int check_data_args(const void *X, long long N, int d, int dtype, int metric, int R)
{
    if (!X) return RNND_ERR_NULL;
    if (dtype != RNND_U8 && dtype != RNND_F32 && dtype != RNND_F16 && dtype != RNND_BF16) return RNND_ERR_UNSUPPORTED;
    if (metric != RNND_L2SQ) return RNND_ERR_UNSUPPORTED;
    if (N < 2 || N > 2147483646LL || d < 1) return RNND_ERR_BAD_SHAPE;
    if (dtype == RNND_U8 && d > 33025) return RNND_ERR_BAD_SHAPE;
    if (R < 1 || R > RNND_MAX_R) return RNND_ERR_BAD_PARAM;
    // list slots are counted in 32-bit device counters, and a bin offset is an int with -1 for "no bin"
    if ((unsigned long long)N * (unsigned long long)R > RNND_MAX_SLOTS) return RNND_ERR_BAD_SHAPE;
    return RNND_OK;
}

static int vec_ok_for(const void *X, int d, int dtype)
{
    size_t rowbytes = (size_t)d * dt_size(dtype);
    return (rowbytes % 16 == 0) && (((uintptr_t)X) % 16 == 0);
}

// How UpdateNeighbors scans for this input: 1 = generic kernel, 2 = int8 MFMA Gram kernel (uint8 rows),
// 3 = matrix-core Gram kernel for float or half rows (fp32 MFMA first, f64 MFMA for what it leaves).
static int scan_variant_for(const void *X, int d, int dtype)
{
    const bool aligned = (((uintptr_t)X) % 16 == 0);
    if (g_kernel_variant == 1 || !aligned) return 1;
    if (dtype == RNND_U8 && (d == 32 || d == 64 || d == 128)) return 2;
    if (dtype == RNND_F32 && d % 16 == 0) return 3;
    if ((dtype == RNND_F16 || dtype == RNND_BF16) && d % 32 == 0) return 3;      // rows of a multiple of 64 bytes
    return 1;
}

static int cu_count()
{
    static int cus = 0;
    if (!cus) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
    }
    return cus;
}

static int persistent_blocks() { return cu_count() * 8; }   // 32 wavefronts per CU

// A grid that walks a list of at most N vertices, one or more per wavefront of a 4-wavefront block, needs no more
// than N / 4 blocks: small inputs get small grids (a launch costs by its workgroups even when they find no work).
static unsigned capped(long long blocks, long long N)
{
    const long long need = (N + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK;
    return (unsigned)(blocks < need ? blocks : (need < 1 ? 1 : need));
}

static inline int vertex_blocks(long long N) { return (int)((N + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK); }

// Blocks of `kernel` (256 threads, static LDS only) that one CU keeps resident; the persistent
// scans launch exactly that many per CU so that every wavefront starts at once.
template <typename K>
static int resident_blocks_per_cu(K kernel, int fallback)
{
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kernel, 256, 0) != hipSuccess || nb < 1) {
        (void)hipGetLastError();
        nb = fallback;
    }
    return nb;
}

// Events tied to kernels of one round (null: not wanted).  They are attached to the launches
// themselves, which costs no extra packet on the stream.
struct RoundEvents {
    hipEvent_t scan_start = nullptr;   // start of the first scan kernel
    hipEvent_t scan_stop = nullptr;    // end of the last scan kernel
    hipEvent_t round_stop = nullptr;   // end of the round's last kernel
};

template <int NG, int KS>
static void launch_mfma_scan(const Workspace &w, int R, u64 *keys, int *deg, long long N, RoundCtr *c,
                             hipStream_t st, hipEvent_t e_stop)
{
    static const int per_cu = resident_blocks_per_cu(k_update_scan_mfma_u8<NG, KS>, NG == 2 ? 3 : 2);
    hipExtLaunchKernelGGL((k_update_scan_mfma_u8<NG, KS>), dim3(capped(cu_count() * per_cu, N)), dim3(256), 0, st, nullptr,
                          e_stop, 0, (const int8_t *)w.xs, R, keys, deg, w.lists + (size_t)(NG + 1) * N,
                          &c->n_active[NG + 1], w.props, w.nprop, c);
}

// Fills w.xs for the uint8 MFMA scan (d = 32, 64 or 128; X is 16-byte aligned).
static void launch_prepare_u8(const Workspace &w, const void *X, long long N, int d, hipStream_t st)
{
    const size_t n = (size_t)N * d;
    hipLaunchKernelGGL(k_prepare_u8, dim3((unsigned)((n / 16 + 255) / 256)), dim3(256), 0, st, (const uint8_t *)X, n,
                       w.xs);
}

// Bytes of the int8 copy of X that the uint8 MFMA scan works on (0 for every other scan).
static size_t xs_bytes_for(long long N, int d, int variant) { return variant == 2 ? (size_t)N * d : 0; }

template <int KS>
static void launch_mfma_scan_classes(const Workspace &w, int R, u64 *keys, int *deg, long long N, RoundCtr *c,
                                     hipStream_t st, const RoundEvents &re)
{
    static const int per_cu = resident_blocks_per_cu(k_update_scan_mfma_u8_small<KS>, 4);
    const int n_big = (R > 32) + (R > 64) + (R > 96);   // launches after the short-list kernel
    // small inputs: every class in one launch (see k_update_scan_mfma_u8_all)
    if (n_big > 0 && (g_scan_launches == 2 || (g_scan_launches == 0 && N <= SMALL_INPUT_MAX_N))) {
        unsigned gx = capped((long long)cu_count() * 2, N);
        if (gx < 8) gx = 8;      // a block at least for every class
        if (n_big == 1)
            hipExtLaunchKernelGGL((k_update_scan_mfma_u8_all<KS, 4>), dim3(gx), dim3(256), 0, st, re.scan_start, re.scan_stop, 0,
                                  (const int8_t *)w.xs, R, keys, deg, w.lists, N, w.props, w.nprop, c);
        else if (n_big == 2)
            hipExtLaunchKernelGGL((k_update_scan_mfma_u8_all<KS, 5>), dim3(gx), dim3(256), 0, st, re.scan_start, re.scan_stop, 0,
                                  (const int8_t *)w.xs, R, keys, deg, w.lists, N, w.props, w.nprop, c);
        else
            hipExtLaunchKernelGGL((k_update_scan_mfma_u8_all<KS, 6>), dim3(gx), dim3(256), 0, st, re.scan_start, re.scan_stop, 0,
                                  (const int8_t *)w.xs, R, keys, deg, w.lists, N, w.props, w.nprop, c);
        return;
    }
    const int ny = 1 + (R > 8) + (R > 16);
    hipExtLaunchKernelGGL((k_update_scan_mfma_u8_small<KS>), dim3(capped(cu_count() * per_cu, N), ny), dim3(256), 0, st,
                          re.scan_start, n_big == 0 ? re.scan_stop : nullptr, 0, (const int8_t *)w.xs, R, keys, deg,
                          w.lists, N, w.props, w.nprop, c);
    // large inputs: the short-list launch above, then the longer classes in one launch
    if (n_big >= 2 && (g_scan_launches == 3 || (g_scan_launches == 0 && N <= LONG_SHARED_MAX_N))) {
        unsigned gx = capped((long long)cu_count() * 2, N);
        if (gx < 8) gx = 8;      // a block at least for every class
        if (n_big == 2)
            hipExtLaunchKernelGGL((k_update_scan_mfma_u8_all<KS, 5, 3>), dim3(gx), dim3(256), 0, st, nullptr, re.scan_stop, 0,
                                  (const int8_t *)w.xs, R, keys, deg, w.lists, N, w.props, w.nprop, c);
        else
            hipExtLaunchKernelGGL((k_update_scan_mfma_u8_all<KS, 6, 3>), dim3(gx), dim3(256), 0, st, nullptr, re.scan_stop, 0,
                                  (const int8_t *)w.xs, R, keys, deg, w.lists, N, w.props, w.nprop, c);
        return;
    }
    if (R > 32) launch_mfma_scan<2, KS>(w, R, keys, deg, N, c, st, n_big == 1 ? re.scan_stop : nullptr);
    if (R > 64) launch_mfma_scan<3, KS>(w, R, keys, deg, N, c, st, n_big == 2 ? re.scan_stop : nullptr);
    if (R > 96) launch_mfma_scan<4, KS>(w, R, keys, deg, N, c, st, n_big == 3 ? re.scan_stop : nullptr);
}

// Float scan of degree class cls: the single-precision form over the class's active list.  Vertices it
// leaves alone (ties in bulk) go to one redo list for all classes, which launch_f32_redo hands to the
// double-precision form.  The redo list lives in the bin array, which nothing else uses until the
// scatter that follows the scans.  Kernel variant 2: the double-precision form on the active list itself.
template <int NG, int CH, int NRC, int DT>
static void launch_f32_scan_dt(const Workspace &w, const void *X, int d, int R, u64 *keys, int *deg, long long N,
                               RoundCtr *c, int cls, hipStream_t st, hipEvent_t e_start, hipEvent_t e_stop)
{
    // wavefronts that fit per SIMD: about 4 for NG = 1, 2 for NG = 2, 1 for NG = 3 (21 accumulator tiles)
    static const int per_cu_fast = resident_blocks_per_cu(k_update_scan_mfma_f32<NG, CH, NRC, true, DT>, NG == 1 ? 4 : 2);
    static const int per_cu = resident_blocks_per_cu(k_update_scan_mfma_f32<NG, CH, NRC, false, DT>, NG == 1 ? 4 : NG == 2 ? 2 : 1);
    if (g_kernel_variant != 2)
        hipExtLaunchKernelGGL((k_update_scan_mfma_f32<NG, CH, NRC, true, DT>), dim3(capped(cu_count() * per_cu_fast, N)), dim3(256), 0,
                              st, e_start, e_stop, 0, (const char *)X, d, R, keys, deg, w.lists + (size_t)cls * N,
                              &c->n_active[cls], w.props, w.nprop, c, (int *)w.bins, &c->n_redo[0]);
    else
        hipExtLaunchKernelGGL((k_update_scan_mfma_f32<NG, CH, NRC, false, DT>), dim3(capped(cu_count() * per_cu, N)), dim3(256), 0,
                              st, e_start, e_stop, 0, (const char *)X, d, R, keys, deg, w.lists + (size_t)cls * N,
                              &c->n_active[cls], w.props, w.nprop, c, (int *)nullptr, (u32 *)nullptr);
}

template <int NG, int CH, int NRC>
static void launch_f32_scan(const Workspace &w, const void *X, int d, int dtype, int R, u64 *keys, int *deg,
                            long long N, RoundCtr *c, int cls, hipStream_t st, hipEvent_t e_start, hipEvent_t e_stop)
{
    // (the three-group shape compiles badly -- with some versions of this code to thousands of spilled
    // registers -- so lists of 33..48 entries take the four-group kernel, which skips the tiles of the empty
    // group; the shape is not instantiated at all)
    constexpr int NRK = NRC == 3 ? 4 : NRC;
    if (dtype == RNND_F16)
        launch_f32_scan_dt<NG, CH, NRK, DT_F16>(w, X, d, R, keys, deg, N, c, cls, st, e_start, e_stop);
    else if (dtype == RNND_BF16)
        launch_f32_scan_dt<NG, CH, NRK, DT_BF16>(w, X, d, R, keys, deg, N, c, cls, st, e_start, e_stop);
    else
        launch_f32_scan_dt<NG, CH, NRK, DT_F32>(w, X, d, R, keys, deg, N, c, cls, st, e_start, e_stop);
}

// The double-precision form (in its widest shape: lists of up to 96 entries) over the round's redo list.
template <int DT>
static void launch_f32_redo_dt(const Workspace &w, const void *X, int d, int R, u64 *keys, int *deg, RoundCtr *c,
                               hipStream_t st, hipEvent_t e_stop)
{
    static const int per_cu = resident_blocks_per_cu(k_update_scan_mfma_f32<3, 1, 6, false, DT>, 1);
    hipExtLaunchKernelGGL((k_update_scan_mfma_f32<3, 1, 6, false, DT>), dim3(cu_count() * per_cu), dim3(256), 0, st,
                          nullptr, e_stop, 0, (const char *)X, d, R, keys, deg, (const int *)w.bins,
                          (const u32 *)&c->n_redo[0], w.props, w.nprop, c, (int *)nullptr, (u32 *)nullptr);
}

static void launch_f32_redo(const Workspace &w, const void *X, int d, int dtype, int R, u64 *keys, int *deg,
                            RoundCtr *c, hipStream_t st, hipEvent_t e_stop)
{
    if (dtype == RNND_F16) launch_f32_redo_dt<DT_F16>(w, X, d, R, keys, deg, c, st, e_stop);
    else if (dtype == RNND_BF16) launch_f32_redo_dt<DT_BF16>(w, X, d, R, keys, deg, c, st, e_stop);
    else launch_f32_redo_dt<DT_F32>(w, X, d, R, keys, deg, c, st, e_stop);
}

// One run of consecutive vertex ids of a block-sequential pass: ids first .. first + count - 1.
struct VertexRun {
    u32 first = 0, count = 0;
};

// One synchronous round over the active lists of counter slot t (run == nullptr), or one run of a
// block-sequential pass: the run's active lists are taken from vcls[] first, and the classes of the
// vertices its merge touched go back to vcls[] instead of into the next slot's lists.
static hipError_t launch_update_round(const Workspace &w, const void *X, long long N, int d, int dtype,
                                      int vec_ok, int variant, int R, u64 *keys, int *deg, int t,
                                      hipStream_t st, const RoundEvents &re = RoundEvents(),
                                      const VertexRun *run = nullptr)
{
    const unsigned pb = capped(persistent_blocks(), N);
    RoundCtr *c = w.ctr + t;
    const int use_classes = variant == 2 ? 2 : variant == 3 ? 1 : 0;
    if (run) {
        const unsigned cb = (run->count + 1023u) / 1024u;
        hipLaunchKernelGGL(k_compact_classes, dim3(cb < 256u ? cb : 256u, 1), dim3(1024), 0, st, (const u32 *)nullptr,
                           run->count, (const int *)nullptr, (const int8_t *)w.vcls, w.lists, N, c->n_active,
                           run->first, w.vcls);
    }
    if (variant == 2) {
        if (d == 32) launch_mfma_scan_classes<1>(w, R, keys, deg, N, c, st, re);
        else if (d == 64) launch_mfma_scan_classes<2>(w, R, keys, deg, N, c, st, re);
        else launch_mfma_scan_classes<4>(w, R, keys, deg, N, c, st, re);
    } else if (variant == 3) {
        // degree classes 0..6: lists of at most 8, 16, 32, 48, 64, 80, 96 entries = 1, 1, 2, 3, 4, 5, 6 groups of 16
        // rows; class 7 (97..128 entries: too many accumulator tiles) goes to the generic kernel
        const int n_more = (R > 8) + (R > 16) + (R > 32) + (R > 48) + (R > 64) + (R > 80) + (R > 96);
        // the round's scan ends with its last launch: the redo pass, or the generic kernel when R > 96
        const bool redo_pass = g_kernel_variant != 2, generic_tail = R > 96;
        int k = 0;
        auto stop_for = [&](void) {
            const bool last = k++ == n_more;
            return (last && (generic_tail || !redo_pass)) ? re.scan_stop : (hipEvent_t) nullptr;
        };
        const bool wide = ((size_t)d * dt_size(dtype)) % 128 == 0;     // two 64-byte chunks per iteration
        if (wide) launch_f32_scan<1, 2, 1>(w, X, d, dtype, R, keys, deg, N, c, 0, st, re.scan_start, stop_for());
        else launch_f32_scan<1, 1, 1>(w, X, d, dtype, R, keys, deg, N, c, 0, st, re.scan_start, stop_for());
        if (R > 8) {
            if (wide) launch_f32_scan<1, 2, 1>(w, X, d, dtype, R, keys, deg, N, c, 1, st, nullptr, stop_for());
            else launch_f32_scan<1, 1, 1>(w, X, d, dtype, R, keys, deg, N, c, 1, st, nullptr, stop_for());
        }
        if (R > 16) {
            if (wide) launch_f32_scan<1, 2, 2>(w, X, d, dtype, R, keys, deg, N, c, 2, st, nullptr, stop_for());
            else launch_f32_scan<1, 1, 2>(w, X, d, dtype, R, keys, deg, N, c, 2, st, nullptr, stop_for());
        }
        if (R > 32) launch_f32_scan<2, 1, 3>(w, X, d, dtype, R, keys, deg, N, c, 3, st, nullptr, stop_for());
        if (R > 48) launch_f32_scan<2, 1, 4>(w, X, d, dtype, R, keys, deg, N, c, 4, st, nullptr, stop_for());
        if (R > 64) launch_f32_scan<3, 1, 5>(w, X, d, dtype, R, keys, deg, N, c, 5, st, nullptr, stop_for());
        if (R > 80) launch_f32_scan<3, 1, 6>(w, X, d, dtype, R, keys, deg, N, c, 6, st, nullptr, stop_for());
        if (redo_pass) launch_f32_redo(w, X, d, dtype, R, keys, deg, c, st, generic_tail ? (hipEvent_t) nullptr : re.scan_stop);
        if (R > 96) {
            if (dtype == RNND_F16)
                hipExtLaunchKernelGGL(k_update_scan<DT_F16>, dim3(pb), dim3(BLOCK), 0, st, nullptr, stop_for(), 0, X, d,
                                      vec_ok, R, keys, deg, w.lists + (size_t)7 * N, &c->n_active[7], w.props, w.nprop, c);
            else if (dtype == RNND_BF16)
                hipExtLaunchKernelGGL(k_update_scan<DT_BF16>, dim3(pb), dim3(BLOCK), 0, st, nullptr, stop_for(), 0, X, d,
                                      vec_ok, R, keys, deg, w.lists + (size_t)7 * N, &c->n_active[7], w.props, w.nprop, c);
            else
                hipExtLaunchKernelGGL(k_update_scan<DT_F32>, dim3(pb), dim3(BLOCK), 0, st, nullptr, stop_for(), 0, X, d,
                                      vec_ok, R, keys, deg, w.lists + (size_t)7 * N, &c->n_active[7], w.props, w.nprop, c);
        }
    } else if (dtype == RNND_U8) {
        hipExtLaunchKernelGGL(k_update_scan<DT_U8>, dim3(pb), dim3(BLOCK), 0, st, re.scan_start, re.scan_stop, 0, X, d,
                              vec_ok, R, keys, deg, w.lists, &c->n_active[0], w.props, w.nprop, c);
    } else if (dtype == RNND_F16) {
        hipExtLaunchKernelGGL(k_update_scan<DT_F16>, dim3(pb), dim3(BLOCK), 0, st, re.scan_start, re.scan_stop, 0, X, d,
                              vec_ok, R, keys, deg, w.lists, &c->n_active[0], w.props, w.nprop, c);
    } else if (dtype == RNND_BF16) {
        hipExtLaunchKernelGGL(k_update_scan<DT_BF16>, dim3(pb), dim3(BLOCK), 0, st, re.scan_start, re.scan_stop, 0, X, d,
                              vec_ok, R, keys, deg, w.lists, &c->n_active[0], w.props, w.nprop, c);
    } else {
        hipExtLaunchKernelGGL(k_update_scan<DT_F32>, dim3(pb), dim3(BLOCK), 0, st, re.scan_start, re.scan_stop, 0, X, d,
                              vec_ok, R, keys, deg, w.lists, &c->n_active[0], w.props, w.nprop, c);
    }
    // from here on `fill` plays the role of the per-target count of this round
    const int ncl = use_classes ? NDEG : 1;
    hipLaunchKernelGGL(k_scatter, dim3(pb), dim3(BLOCK), 0, st, N, R, w.lists, ncl, c, w.props, w.nprop, w.fill,
                       w.inbox);
    if (N <= SMALL_INPUT_MAX_N)
        hipLaunchKernelGGL(k_touch_classify<2>, dim3((unsigned)((N + 2047) / 2048)), dim3(1024), 0, st, N, w.fill, deg, w.binoff, c,
                           w.touched);
    else
        hipLaunchKernelGGL(k_touch_classify<4>, dim3((unsigned)((N + 4095) / 4096)), dim3(1024), 0, st, N, w.fill, deg, w.binoff, c,
                           w.touched);
    hipLaunchKernelGGL(k_scatter_surplus, dim3(pb), dim3(BLOCK), 0, st, N, R, w.lists, ncl, c, w.props, w.nprop,
                       w.binoff, w.bins);
    static const int merge_per_cu = resident_blocks_per_cu(k_merge, 6);
    hipLaunchKernelGGL(k_merge, dim3(capped(cu_count() * merge_per_cu, N), NMRG), dim3(BLOCK), 0, st, N, R, keys, deg, w.touched, c->n_touched,
                       w.fill, w.inbox, w.binoff, w.bins, w.tcls, use_classes, c);
    if (run)
        hipLaunchKernelGGL(k_store_classes, dim3(64, NMRG), dim3(256), 0, st, (const u32 *)c->n_touched,
                           (const int *)w.touched, (const int8_t *)w.tcls, N, w.vcls);
    else
        hipExtLaunchKernelGGL(k_compact_classes, dim3(128, NMRG), dim3(1024), 0, st, nullptr, re.round_stop, 0,
                              (const u32 *)c->n_touched, 0u, (const int *)w.touched, (const int8_t *)w.tcls, w.lists,
                              N, (c + 1)->n_active, 0u, (int8_t *)nullptr);
    return hipGetLastError();
}

// One block-sequential pass: `blocks` runs of ceil(N / blocks) consecutive ids, in id order, counter slots
// t0, t0 + 1, ...  Returns the number of slots used through *used.
static hipError_t launch_update_pass_blocks(const Workspace &w, const void *X, long long N, int d, int dtype,
                                            int vec_ok, int variant, int R, u64 *keys, int *deg, int t0,
                                            long long blocks, hipStream_t st, int *used)
{
    const long long bs = (N + blocks - 1) / blocks;
    int k = 0;
    for (long long lo = 0; lo < N; lo += bs, ++k) {
        VertexRun run;
        run.first = (u32)lo;
        run.count = (u32)(lo + bs < N ? bs : N - lo);
        hipError_t e = launch_update_round(w, X, N, d, dtype, vec_ok, variant, R, keys, deg, t0 + k, st, RoundEvents(),
                                           &run);
        if (e != hipSuccess) return e;
    }
    *used = k;
    return hipSuccess;
}

// slots a pass of `blocks` runs uses
static long long runs_per_pass(long long N, long long blocks)
{
    const long long bs = (N + blocks - 1) / blocks;
    return (N + bs - 1) / bs;
}

// vcls[] (class of every vertex holding a "new" entry) -> active lists of round t_next
static void launch_compact_all(const Workspace &w, long long N, int t_next, hipStream_t st,
                               hipEvent_t e_stop = nullptr)
{
    hipExtLaunchKernelGGL(k_compact_classes, dim3(256, 1), dim3(1024), 0, st, nullptr, e_stop, 0,
                          (const u32 *)nullptr, (u32)N, (const int *)nullptr, (const int8_t *)w.vcls, w.lists, N,
                          w.ctr[t_next].n_active, 0u, (int8_t *)nullptr);
}

// AddReverseEdges; the active lists for round t_next are rebuilt from scratch (t_next < 0: only vcls[], the
// class of every vertex that holds a "new" entry, is written).  Expects fill[] == 0
// and leaves it so.  Between rounds nprop[], tcls[], props[] and touched[] are free: they serve as the
// second in-edge count, the per-vertex marks, the late arrival numbers and their position masks.  misc: [0] bin cursor, [1] vertices with a bin (union and out-degree cut), [4..11] lengths of the compaction of rowflag[] ([4]: the flagged lists),
// [2] bin cursor, [3] vertices with more than R incoming edges (in-degree cut).
static hipError_t launch_reverse(const Workspace &w, long long N, int R, int use_classes, u64 *keys, int *deg,
                                 int t_next, hipStream_t st, hipEvent_t e_stop = nullptr, int W = 0)
{
    if (W == 0) W = R;      // rows are W slots apart; R is Alg. 5's bound on out- and in-degree
    const int vb = vertex_blocks(N), tb = (int)((N + 1023) / 1024);
    int *cnt_in = w.nprop;
    int8_t *cand = w.tcls, *rowflag = w.tcls + N, *mark = w.tcls + 2 * N;
    u32 *late = (u32 *)w.props;          // one word per list slot (props is 16 bytes per slot)
    u64 *over = (u64 *)w.touched;        // two words per vertex (touched is 16 bytes per vertex)
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, st, w.misc, (size_t)16);
    if (t_next >= 0) hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, st, w.ctr[t_next].n_active, (size_t)NDEG);
    // union with reversed edges, out-lists cut to R
    // the transposition: one arrival-number atomic per edge, or (large N, see k_bin_count) binned by target range
    const bool binned = w.blockhist && g_transpose_path != 1 && (g_transpose_path == 2 || N >= BIN_MIN_N);
    if (binned) {
        const unsigned nb = (unsigned)bin_blocks(N), nr = (unsigned)bin_ranges(N);
        hipLaunchKernelGGL(k_bin_count, dim3(nb), dim3(BIN_THREADS), 0, st, N, W, (const u64 *)keys, (const int *)deg, nr, w.blockhist);
        hipLaunchKernelGGL(k_bin_offsets, dim3((nr + 63) / 64), dim3(1024), 0, st, nb, nr, w.blockhist, w.range_tot);
        hipLaunchKernelGGL(k_bin_bases, dim3(1), dim3(1024), 0, st, nr, (const u32 *)w.range_tot, w.range_base);
        hipLaunchKernelGGL(k_bin_partition, dim3(nb), dim3(BIN_THREADS), 0, st, N, W, (const u64 *)keys, (const int *)deg, nr,
                           (const u32 *)w.blockhist, (const u32 *)w.range_base, w.props);
        hipLaunchKernelGGL(k_bin_place, dim3(nr), dim3(PLACE_THREADS), 0, st, N, R, (const Prop *)w.props, (const u32 *)w.range_base,
                           (const int *)deg, w.fill, w.inbox, w.binoff, w.bins, w.misc + 0, w.cnt, cnt_in, cand);
    } else {
        hipLaunchKernelGGL(k_reverse_scatter, dim3((unsigned)((N * 16 + BLOCK - 1) / BLOCK)), dim3(BLOCK), 0, st, N, W, keys, deg,
                           w.fill, w.inbox, late, over, mark);
        hipLaunchKernelGGL(k_assign_bins, dim3(tb), dim3(1024), 0, st, N, w.fill, INBOX_CAP, INBOX_CAP, INBOX_CAP,
                           w.binoff, w.misc + 0, w.hubs, w.misc + 1, w.cnt, cnt_in, (u64 *)nullptr, deg, R, cand);
        hipLaunchKernelGGL(k_reverse_surplus, dim3(vb), dim3(BLOCK), 0, st, N, W, keys, late, over, mark, w.binoff,
                           w.bins, w.misc + 1);
    }
    static const int rmerge_per_cu = resident_blocks_per_cu(k_reverse_merge, 6);
    const int rm_blocks = cu_count() * rmerge_per_cu;
    hipLaunchKernelGGL(k_reverse_merge, dim3(rm_blocks < (vb + 1) / 2 ? rm_blocks : (vb + 1) / 2), dim3(BLOCK), 0, st, N, W, R, keys,
                       deg, w.fill, w.inbox, w.binoff, w.bins, cand, cnt_in, rowflag, w.vcls, use_classes);
    // in-lists cut to R; only vertices with more than R incoming edges need a bin, and only the flagged lists
    // (class 0 of rowflag[]) are walked: they are compacted into the first active list, which is free until
    // the lists of the next round are rebuilt at the end
    int *flagged = w.lists;
    hipLaunchKernelGGL(k_compact_classes, dim3(256, 1), dim3(1024), 0, st, (const u32 *)nullptr, (u32)N, (const int *)nullptr,
                       (const int8_t *)rowflag, flagged, N, w.misc + 4, 0u, (int8_t *)nullptr);
    hipLaunchKernelGGL(k_assign_bins, dim3(tb), dim3(1024), 0, st, N, cnt_in, R, R, 0, w.binoff, w.misc + 2, w.hubs,
                       w.misc + 3, w.cnt, (int *)nullptr, w.thr, (const int *)nullptr, 0, (int8_t *)nullptr);
    hipLaunchKernelGGL(k_fill_bins, dim3(capped(persistent_blocks(), N)), dim3(BLOCK), 0, st, W, (const u64 *)keys, (const int *)deg,
                       (const int *)flagged, (const u32 *)(w.misc + 4), w.binoff, w.cnt, w.bins, 0u, w.misc + 3);
    hipLaunchKernelGGL(k_incap_threshold, dim3(capped(persistent_blocks(), N)), dim3(BLOCK), 0, st, R, w.hubs, w.misc + 3,
                       cnt_in, w.binoff, w.bins, w.thr);
    hipLaunchKernelGGL(k_incap_filter, dim3(capped(persistent_blocks(), N)), dim3(BLOCK), 0, st, W, keys, deg, w.thr,
                       (const int *)flagged, (const u32 *)(w.misc + 4), w.vcls, use_classes, w.misc + 3);
    if (t_next >= 0) launch_compact_all(w, N, t_next, st, e_stop);
    else if (e_stop) (void)hipEventRecord(e_stop, st);
    return hipGetLastError();
}

static void fill_round_stats(rnnd_stats *s, const RoundCtr *h, int rounds)
{
    s->rounds = rounds;
    for (int t = 0; t < rounds && t < RNND_MAX_ROUNDS; ++t) {
        s->active[t] = 0;
        for (int c = 0; c < NDEG; ++c) s->active[t] += h[t].n_active[c];
        for (int k = 0; k < STAT_SLOTS; ++k) {
            s->algo_evals[t] += (int64_t)h[t].stat[k][0];
            s->exec_evals[t] += (int64_t)h[t].stat[k][1];
            s->gathered_rows[t] += (int64_t)h[t].stat[k][2];
            s->proposals[t] += (int64_t)h[t].stat[k][3];
            s->dropped[t] += (int64_t)h[t].stat[k][4];
        }
    }
}

// --------------------------------------------------------------- where a call's workspace comes from
// 1. the block the library keeps per device between calls (allocated by the first call that needs it, grown
//    when a later call needs more, handed back by rnnd_release_workspace): repeated builds pay no allocation;
// 2. a fresh allocation, freed when the call ends, if another thread's call holds that block;
// 3. for rnnd_build_static only: the file-scope array below, which needs no allocation at all.
#define RNND_MAX_DEVICES 64

static __device__ __align__(256) unsigned char scratch[RNND_STATIC_SCRATCH_BYTES];

struct DeviceSlot {
    char *cached = nullptr;        // the kept block
    size_t cached_bytes = 0;
    bool busy = false;             // a call is using it
    char *static_ptr = nullptr;    // this device's copy of `scratch` (hipGetSymbolAddress, once per device)
};
static std::mutex g_ws_mu;
static DeviceSlot g_dev[RNND_MAX_DEVICES];
static int g_poison = 0;           // testing aid: every workspace is filled with 0xA5 bytes before it is cleared

enum WsSource { WS_NONE = 0, WS_CACHED, WS_FRESH, WS_STATIC };
struct WsLease {
    char *base = nullptr;
    int dev = -1;
    WsSource src = WS_NONE;
};

__global__ void k_fill_u32(u32 *p, size_t n, u32 v)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// No device holds a workspace of this size; asking for one is an allocation failure that needs no device to detect.
#define RNND_WS_HARD_LIMIT ((size_t)1 << 40)

static int ws_acquire(size_t bytes, bool static_only, hipStream_t st, WsLease *out)
{
    int rc = RNND_OK, dev = 0;
    if (!static_only && bytes > RNND_WS_HARD_LIMIT) return RNND_ERR_OOM;
    if (static_only && bytes > RNND_STATIC_SCRATCH_BYTES) return RNND_ERR_SCRATCH;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= RNND_MAX_DEVICES) {
        snprintf(g_last_hip_error, sizeof g_last_hip_error, "device index %d is beyond the %d this library tracks", dev,
                 RNND_MAX_DEVICES);
        return RNND_ERR_HIP;
    }
    {
        std::lock_guard<std::mutex> lock(g_ws_mu);
        DeviceSlot &d = g_dev[dev];
        if (static_only) {
            if (!d.static_ptr) {
                char *ptr = nullptr;
                HIPCHK(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
                d.static_ptr = ptr;
            }
            out->base = d.static_ptr;
            out->src = WS_STATIC;
        } else if (!d.busy) {
            if (d.cached && d.cached_bytes < bytes) {
                (void)hipFree(d.cached);
                d.cached = nullptr;
                d.cached_bytes = 0;
            }
            if (!d.cached) {
                HIPCHK(hipMalloc((void **)&d.cached, bytes));
                d.cached_bytes = bytes;
            }
            d.busy = true;
            out->base = d.cached;
            out->src = WS_CACHED;
        } else {
            HIPCHK(hipMalloc((void **)&out->base, bytes));
            out->src = WS_FRESH;
        }
        out->dev = dev;
    }
    if (g_poison) hipLaunchKernelGGL(k_fill_u32, dim3(2048), dim3(256), 0, st, (u32 *)out->base, bytes / 4, 0xA5A5A5A5u);
done:
    return rc;
}

static void ws_release(WsLease *l)
{
    if (l->src == WS_FRESH) {
        (void)hipFree(l->base);
    } else if (l->src == WS_CACHED) {
        std::lock_guard<std::mutex> lock(g_ws_mu);
        g_dev[l->dev].busy = false;
    }
    l->src = WS_NONE;
    l->base = nullptr;
}

extern "C" int rnnd_release_workspace(void)
{
    int rc = RNND_OK, dev = 0;
    HIPCHK(hipGetDevice(&dev));
    if (dev >= 0 && dev < RNND_MAX_DEVICES) {
        std::lock_guard<std::mutex> lock(g_ws_mu);
        DeviceSlot &d = g_dev[dev];
        if (d.cached && !d.busy) {
            HIPCHK(hipFree(d.cached));
            d.cached = nullptr;
            d.cached_bytes = 0;
        }
    }
done:
    return rc;
}

extern "C" int rnnd_set_workspace_poison(int on)
{
    g_poison = on ? 1 : 0;
    return RNND_OK;
}

extern "C" int rnnd_workspace_bytes(int64_t N, int32_t d, int dtype, int32_t R, int64_t rounds, size_t *bytes)
{
    if (!bytes) return RNND_ERR_NULL;
    if (dtype != RNND_U8 && dtype != RNND_F32 && dtype != RNND_F16 && dtype != RNND_BF16) return RNND_ERR_UNSUPPORTED;
    if (N < 2 || N > 2147483646LL || d < 1) return RNND_ERR_BAD_SHAPE;
    if (R < 1 || R > RNND_MAX_R || rounds < 1 || rounds > RNND_MAX_RUN_SLOTS) return RNND_ERR_BAD_PARAM;
    Workspace w;
    // upper bound: the int8 copy exists only for uint8 rows of 32, 64 or 128 bytes
    *bytes = ws_layout(w, N, R, (int)rounds + 2, true,
                       (dtype == RNND_U8 && (d == 32 || d == 64 || d == 128)) ? (size_t)N * d : 0);
    return RNND_OK;
}

template <int DT>
static void launch_random_graph_dt(const void *X, long long N, int d, int vec_ok, int S, int R, u64 seed, u64 *keys,
                                   int *deg, int8_t *vcls, int use_classes, hipStream_t st)
{
    hipLaunchKernelGGL(k_random_graph<DT>, dim3(vertex_blocks(N)), dim3(BLOCK), 0, st, X, N, d, vec_ok, S, R, seed, keys,
                       deg, vcls, use_classes);
}

static void launch_random_graph(const void *X, long long N, int d, int dtype, int vec_ok, int S, int R, u64 seed,
                                u64 *keys, int *deg, int8_t *vcls, int use_classes, hipStream_t st)
{
    if (dtype == RNND_U8) launch_random_graph_dt<DT_U8>(X, N, d, vec_ok, S, R, seed, keys, deg, vcls, use_classes, st);
    else if (dtype == RNND_F16) launch_random_graph_dt<DT_F16>(X, N, d, vec_ok, S, R, seed, keys, deg, vcls, use_classes, st);
    else if (dtype == RNND_BF16) launch_random_graph_dt<DT_BF16>(X, N, d, vec_ok, S, R, seed, keys, deg, vcls, use_classes, st);
    else launch_random_graph_dt<DT_F32>(X, N, d, vec_ok, S, R, seed, keys, deg, vcls, use_classes, st);
}

// per-pass statistics of a block-sequential run: slot sums of the runs of each pass
static void fill_pass_stats(rnnd_stats *s, const RoundCtr *h, int passes, int per_pass)
{
    rnnd_stats one;
    s->rounds = passes;
    for (int p = 0; p < passes && p < RNND_MAX_ROUNDS; ++p) {
        for (int k = 0; k < per_pass; ++k) {
            memset(&one, 0, sizeof one);
            fill_round_stats(&one, h + (size_t)p * per_pass + k, 1);
            s->active[p] += one.active[0];
            s->algo_evals[p] += one.algo_evals[0];
            s->exec_evals[p] += one.exec_evals[0];
            s->gathered_rows[p] += one.gathered_rows[0];
            s->proposals[p] += one.proposals[0];
            s->dropped[p] += one.dropped[0];
        }
    }
}

// Alg. 6, every variant of the driver.
//   M       slots per row = the bound every UpdateNeighbors merge cuts a list to (M = R: rnnd_build;
//           M > R: rnnd_build_wide, where only AddReverseEdges cuts to R)
//   blocks  0: synchronous rounds; >= 1: block-sequential passes of that many runs (rnnd_build_blocks)
//   fixed   the workspace is the static scratch array: no allocation of any kind, hence no statistics
static int build_impl(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S, int32_t R, int32_t M,
                      int32_t T1, int32_t T2, uint64_t seed, int64_t blocks, int32_t *graph_out,
                      int32_t *degree_out, uint64_t *keys_out, rnnd_stats *stats, void *stream, bool fixed)
{
    int rc = check_data_args(X, N, d, dtype, metric, M);
    if (rc) return rc;
    if (R < 1 || R > M) return RNND_ERR_BAD_PARAM;
    if (!graph_out || !degree_out) return RNND_ERR_NULL;
    if (S < 1 || S > R || (int64_t)S > N - 1 || T1 < 1 || T2 < 1) return RNND_ERR_BAD_PARAM;
    if ((int64_t)T1 * T2 > RNND_MAX_RUN_SLOTS || blocks < 0 || blocks > N) return RNND_ERR_BAD_PARAM;
    const long long per_pass = blocks ? runs_per_pass(N, blocks) : 1;
    if ((long long)T1 * T2 * per_pass > RNND_MAX_RUN_SLOTS) return RNND_ERR_BAD_PARAM;
    hipStream_t st = (hipStream_t)stream;
    const int rounds = T1 * T2, n_ctr = (int)(rounds * per_pass) + 2, vec_ok = vec_ok_for(X, d, dtype);
    const int variant = scan_variant_for(X, d, dtype), use_classes = variant == 2 ? 2 : variant == 3 ? 1 : 0;
    // events (only when statistics are wanted): 0 start, 1 end of init, last: the end.  Per-round times come from the
    // device clock (RoundCtr::t_*), which costs nothing; with rnnd_set_event_timing(1), and for block-sequential
    // passes, from events as well: 2 + 3t .. 4 + 3t = scan start, scan stop, end of round t (block-sequential passes
    // record only the last), then the end of each reverse call
    const bool ev_rounds = stats && (g_event_timing || blocks);
    const int e_rev = 2 + 3 * rounds, e_end = e_rev + T1, n_ev = stats ? e_end + 1 : 0;
    Workspace w;
    WsLease lease;
    hipEvent_t *ev = nullptr;
    RoundCtr *hctr = nullptr;
    int n_ev_made = 0;
    w.bytes = ws_layout(w, N, M, n_ctr, true, xs_bytes_for(N, d, variant));
    rc = ws_acquire(w.bytes, fixed, st, &lease);
    if (rc) return rc;
    w.base = lease.base;
    ws_layout(w, N, M, n_ctr, true, xs_bytes_for(N, d, variant));
    if (stats) {
        ev = (hipEvent_t *)calloc(n_ev + 1, sizeof(hipEvent_t));
        hctr = (RoundCtr *)calloc(n_ctr, sizeof(RoundCtr));
        if (!ev || !hctr) { rc = RNND_ERR_OOM; goto done; }
        for (; n_ev_made < n_ev; ++n_ev_made)
            if (ev_rounds || n_ev_made < 2 || n_ev_made == e_end) HIPCHK(hipEventCreate(&ev[n_ev_made]));
    }
    {
        int t = 0;
        if (stats) HIPCHK(hipEventRecord(ev[0], st));
        ws_clear(w, st);
        if (variant == 2) launch_prepare_u8(w, X, N, d, st);
        launch_random_graph(X, N, d, dtype, vec_ok, S, M, (u64)seed, w.keys, w.deg, w.vcls, use_classes, st);
        if (!blocks) launch_compact_all(w, N, 0, st, stats ? ev[1] : nullptr);
        else if (stats) HIPCHK(hipEventRecord(ev[1], st));
        HIPCHK(hipGetLastError());
        for (int t1 = 0; t1 < T1; ++t1) {
            for (int t2 = 0; t2 < T2; ++t2, ++t) {
                if (blocks) {
                    int used = 0;
                    HIPCHK(launch_update_pass_blocks(w, X, N, d, dtype, vec_ok, variant, M, w.keys, w.deg,
                                                     (int)(t * per_pass), blocks, st, &used));
                    if (stats) HIPCHK(hipEventRecord(ev[4 + 3 * t], st));
                    continue;
                }
                RoundEvents re;
                // a round ends where the next one starts; only the last round before a reverse call or
                // the export needs a mark of its own for that
                if (ev_rounds) {
                    re.scan_start = ev[2 + 3 * t];
                    re.scan_stop = ev[3 + 3 * t];
                    if (t2 == T2 - 1) re.round_stop = ev[4 + 3 * t];
                }
                HIPCHK(launch_update_round(w, X, N, d, dtype, vec_ok, variant, M, w.keys, w.deg, t, st, re));
                if (stats && !ev_rounds && t2 == T2 - 1)
                    hipLaunchKernelGGL(k_stamp, dim3(1), dim3(64), 0, st, &w.ctr[t].t_round_stop);
            }
            if (t1 != T1 - 1) {
                HIPCHK(launch_reverse(w, N, R, use_classes, w.keys, w.deg, blocks ? -1 : t, st,
                                      ev_rounds ? ev[e_rev + t1] : nullptr, M));
            }
        }
        launch_export(N, M, w.keys, w.deg, graph_out, degree_out, st);
        HIPCHK(hipGetLastError());
        if (keys_out)
            HIPCHK(hipMemcpyAsync(keys_out, w.keys, (size_t)N * M * 8, hipMemcpyDeviceToDevice, st));
        if (stats) {
            HIPCHK(hipEventRecord(ev[e_end], st));
            HIPCHK(hipMemcpyAsync(hctr, w.ctr, (size_t)n_ctr * sizeof(RoundCtr), hipMemcpyDeviceToHost, st));
        }
        HIPCHK(hipStreamSynchronize(st));
        if (stats) {
            memset(stats, 0, sizeof *stats);
            if (blocks) fill_pass_stats(stats, hctr, rounds, (int)per_pass);
            else fill_round_stats(stats, hctr, rounds);
            stats->reverse_calls = T1 - 1;
            stats->init_evals = (int64_t)N * S;
            stats->kernel_variant = variant;
            float ms = 0;
            (void)hipEventElapsedTime(&ms, ev[0], ev[1]); stats->init_ms = ms;
            int tt = 0;
            // device clock: ticks per millisecond, and the time between two marks (0 where one is missing)
            int dev = 0, khz = 0;
            (void)hipGetDevice(&dev);
            (void)hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev);
            auto clk_ms = [khz](u64 a, u64 b) { return (a && b > a && khz > 0) ? (float)((double)(b - a) / (double)khz) : 0.f; };
            for (int t1 = 0; t1 < T1 && !ev_rounds; ++t1) {
                for (int t2 = 0; t2 < T2; ++t2, ++tt) {
                    if (tt >= RNND_MAX_ROUNDS) continue;
                    stats->scan_ms[tt] = clk_ms(hctr[tt].t_scan_start, hctr[tt].t_scan_stop);
                    stats->round_ms[tt] = clk_ms(hctr[tt].t_scan_start, t2 == T2 - 1 ? hctr[tt].t_round_stop : hctr[tt + 1].t_scan_start);
                }
                // an AddReverseEdges call ends where the next round's scan starts
                if (t1 != T1 - 1 && t1 < RNND_MAX_ROUNDS) stats->reverse_ms[t1] = clk_ms(hctr[tt - 1].t_round_stop, hctr[tt].t_scan_start);
            }
            for (int t1 = 0; t1 < T1 && ev_rounds; ++t1) {
                for (int t2 = 0; t2 < T2; ++t2, ++tt) {
                    if (tt >= RNND_MAX_ROUNDS) continue;
                    if (blocks) {
                        // a pass starts where the one before it, the init or the reverse call ended
                        hipEvent_t from = t2 > 0 ? ev[4 + 3 * (tt - 1)] : (t1 == 0 ? ev[1] : ev[e_rev + t1 - 1]);
                        (void)hipEventElapsedTime(&ms, from, ev[4 + 3 * tt]); stats->round_ms[tt] = ms;
                        continue;
                    }
                    (void)hipEventElapsedTime(&ms, ev[2 + 3 * tt], ev[3 + 3 * tt]); stats->scan_ms[tt] = ms;
                    (void)hipEventElapsedTime(&ms, ev[2 + 3 * tt], t2 == T2 - 1 ? ev[4 + 3 * tt] : ev[2 + 3 * (tt + 1)]);
                    stats->round_ms[tt] = ms;
                }
                if (t1 != T1 - 1 && t1 < RNND_MAX_ROUNDS) {
                    // from the end of the last round before the call to the end of the call
                    (void)hipEventElapsedTime(&ms, ev[4 + 3 * (tt - 1)], ev[e_rev + t1]);
                    stats->reverse_ms[t1] = ms;
                }
            }
            (void)hipEventElapsedTime(&ms, ev[0], ev[e_end]); stats->total_ms = ms;
        }
    }
done:
    if (rc == RNND_ERR_HIP || rc == RNND_ERR_OOM) (void)hipStreamSynchronize(st);   // nothing may still use the workspace
    for (int i = 0; i < n_ev_made; ++i)
        if (ev[i]) (void)hipEventDestroy(ev[i]);
    free(ev);
    free(hctr);
    ws_release(&lease);
    return rc;
}

extern "C" int rnnd_build_ex(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S,
                             int32_t R, int32_t T1, int32_t T2, uint64_t seed, int32_t *graph_out,
                             int32_t *degree_out, uint64_t *keys_out, rnnd_stats *stats, void *stream)
{
    return build_impl(X, N, d, dtype, metric, S, R, R, T1, T2, seed, 0, graph_out, degree_out, keys_out, stats, stream, false);
}

extern "C" int rnnd_build_wide(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S, int32_t R,
                               int32_t M, int32_t T1, int32_t T2, uint64_t seed, int32_t *graph_out,
                               int32_t *degree_out, uint64_t *keys_out, rnnd_stats *stats, void *stream)
{
    if (M < 1 || M > RNND_MAX_R) return X ? RNND_ERR_BAD_PARAM : RNND_ERR_NULL;
    return build_impl(X, N, d, dtype, metric, S, R, M, T1, T2, seed, 0, graph_out, degree_out, keys_out, stats, stream, false);
}

extern "C" int rnnd_build(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S, int32_t R,
                          int32_t T1, int32_t T2, uint64_t seed, int32_t *graph_out, int32_t *degree_out,
                          void *stream)
{
    return build_impl(X, N, d, dtype, metric, S, R, R, T1, T2, seed, 0, graph_out, degree_out, nullptr, nullptr, stream, false);
}

extern "C" int rnnd_build_static(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S, int32_t R,
                                 int32_t T1, int32_t T2, uint64_t seed, int32_t *graph_out, int32_t *degree_out,
                                 void *stream)
{
    return build_impl(X, N, d, dtype, metric, S, R, R, T1, T2, seed, 0, graph_out, degree_out, nullptr, nullptr, stream, true);
}

extern "C" int rnnd_build_blocks(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S,
                                 int32_t R, int32_t T1, int32_t T2, uint64_t seed, int64_t blocks,
                                 int32_t *graph_out, int32_t *degree_out, uint64_t *keys_out, rnnd_stats *stats,
                                 void *stream)
{
    if (blocks < 1) return X ? RNND_ERR_BAD_PARAM : RNND_ERR_NULL;
    return build_impl(X, N, d, dtype, metric, S, R, R, T1, T2, seed, blocks, graph_out, degree_out, keys_out, stats, stream, false);
}

extern "C" int rnnd_random_graph(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S,
                                 int32_t R, uint64_t seed, uint64_t *keys, int32_t *deg, void *stream)
{
    int rc = check_data_args(X, N, d, dtype, metric, R);
    if (rc) return rc;
    if (!keys || !deg) return RNND_ERR_NULL;
    if (S < 1 || S > R || (int64_t)S > N - 1) return RNND_ERR_BAD_PARAM;
    hipStream_t st = (hipStream_t)stream;
    launch_random_graph(X, N, d, dtype, vec_ok_for(X, d, dtype), S, R, (u64)seed, (u64 *)keys, deg, (int8_t *)nullptr, 0, st);
    HIPCHK(hipGetLastError());
    HIPCHK(hipStreamSynchronize(st));
done:
    return rc;
}

// UpdateNeighbors applied in place to a caller's snapshot: n_rounds synchronous rounds (blocks = 0) or
// block-sequential passes of `blocks` runs.
static int update_impl(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t R, uint64_t *keys,
                       int32_t *deg, int32_t n_rounds, int64_t blocks, rnnd_stats *stats, void *stream)
{
    int rc = check_data_args(X, N, d, dtype, metric, R);
    if (rc) return rc;
    if (!keys || !deg) return RNND_ERR_NULL;
    if (n_rounds < 1 || n_rounds > RNND_MAX_RUN_SLOTS || blocks < 0 || blocks > N) return RNND_ERR_BAD_PARAM;
    const long long per_pass = blocks ? runs_per_pass(N, blocks) : 1;
    if ((long long)n_rounds * per_pass > RNND_MAX_RUN_SLOTS) return RNND_ERR_BAD_PARAM;
    hipStream_t st = (hipStream_t)stream;
    const int n_ctr = (int)(n_rounds * per_pass) + 2, vec_ok = vec_ok_for(X, d, dtype);
    const int variant = scan_variant_for(X, d, dtype), use_classes = variant == 2 ? 2 : variant == 3 ? 1 : 0;
    Workspace w;
    WsLease lease;
    RoundCtr *hctr = nullptr;
    w.bytes = ws_layout(w, N, R, n_ctr, false, xs_bytes_for(N, d, variant));
    rc = ws_acquire(w.bytes, false, st, &lease);
    if (rc) return rc;
    w.base = lease.base;
    ws_layout(w, N, R, n_ctr, false, xs_bytes_for(N, d, variant));
    if (stats) {
        hctr = (RoundCtr *)calloc(n_ctr, sizeof(RoundCtr));
        if (!hctr) { rc = RNND_ERR_OOM; goto done; }
    }
    ws_clear(w, st);
    if (variant == 2) launch_prepare_u8(w, X, N, d, st);
    hipLaunchKernelGGL(k_classify, dim3(vertex_blocks(N)), dim3(BLOCK), 0, st, (long long)N, R, (const u64 *)keys,
                       deg, w.vcls, use_classes);
    if (!blocks) launch_compact_all(w, N, 0, st);
    HIPCHK(hipGetLastError());
    for (int t = 0; t < n_rounds; ++t) {
        if (blocks) {
            int used = 0;
            HIPCHK(launch_update_pass_blocks(w, X, N, d, dtype, vec_ok, variant, R, (u64 *)keys, deg,
                                             (int)(t * per_pass), blocks, st, &used));
        } else {
            HIPCHK(launch_update_round(w, X, N, d, dtype, vec_ok, variant, R, (u64 *)keys, deg, t, st));
        }
    }
    if (stats) {
        if (!blocks) hipLaunchKernelGGL(k_stamp, dim3(1), dim3(64), 0, st, &w.ctr[n_rounds - 1].t_round_stop);
        HIPCHK(hipMemcpyAsync(hctr, w.ctr, (size_t)n_ctr * sizeof(RoundCtr), hipMemcpyDeviceToHost, st));
    }
    HIPCHK(hipStreamSynchronize(st));
    if (stats) {
        memset(stats, 0, sizeof *stats);
        if (blocks) fill_pass_stats(stats, hctr, n_rounds, (int)per_pass);
        else fill_round_stats(stats, hctr, n_rounds);
        stats->kernel_variant = variant;
        if (!blocks) {      // per-round times from the device clock (see build_impl)
            int dev = 0, khz = 0;
            (void)hipGetDevice(&dev);
            (void)hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev);
            auto clk_ms = [khz](u64 a, u64 b) { return (a && b > a && khz > 0) ? (float)((double)(b - a) / (double)khz) : 0.f; };
            for (int t = 0; t < n_rounds && t < RNND_MAX_ROUNDS; ++t) {
                stats->scan_ms[t] = clk_ms(hctr[t].t_scan_start, hctr[t].t_scan_stop);
                stats->round_ms[t] = clk_ms(hctr[t].t_scan_start, t == n_rounds - 1 ? hctr[t].t_round_stop : hctr[t + 1].t_scan_start);
            }
        }
    }
done:
    if (rc == RNND_ERR_HIP || rc == RNND_ERR_OOM) (void)hipStreamSynchronize(st);
    free(hctr);
    ws_release(&lease);
    return rc;
}

extern "C" int rnnd_update_neighbors(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t R,
                                     uint64_t *keys, int32_t *deg, int32_t n_rounds, rnnd_stats *stats,
                                     void *stream)
{
    return update_impl(X, N, d, dtype, metric, R, keys, deg, n_rounds, 0, stats, stream);
}

extern "C" int rnnd_update_neighbors_blocks(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t R,
                                            uint64_t *keys, int32_t *deg, int32_t n_passes, int64_t blocks,
                                            rnnd_stats *stats, void *stream)
{
    if (blocks < 1) return X ? RNND_ERR_BAD_PARAM : RNND_ERR_NULL;
    return update_impl(X, N, d, dtype, metric, R, keys, deg, n_passes, blocks, stats, stream);
}

extern "C" int rnnd_add_reverse_edges_wide(int64_t N, int32_t R, int32_t M, uint64_t *keys, int32_t *deg,
                                           void *stream)
{
    int rc = RNND_OK;
    if (!keys || !deg) return RNND_ERR_NULL;
    if (N < 2 || N > 2147483646LL) return RNND_ERR_BAD_SHAPE;
    if (R < 1 || M < R || M > RNND_MAX_R) return RNND_ERR_BAD_PARAM;
    if ((unsigned long long)N * (unsigned long long)M > RNND_MAX_SLOTS) return RNND_ERR_BAD_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    Workspace w;
    WsLease lease;
    w.bytes = ws_layout(w, N, M, 2, false, 0);
    rc = ws_acquire(w.bytes, false, st, &lease);
    if (rc) return rc;
    w.base = lease.base;
    ws_layout(w, N, M, 2, false, 0);
    ws_clear(w, st);      // launch_reverse expects fill[] == 0, cnt[] == 0 and zeroed counters
    HIPCHK(launch_reverse(w, N, R, 0, (u64 *)keys, deg, 0, st, nullptr, M));
    HIPCHK(hipStreamSynchronize(st));
done:
    if (rc == RNND_ERR_HIP || rc == RNND_ERR_OOM) (void)hipStreamSynchronize(st);
    ws_release(&lease);
    return rc;
}

extern "C" int rnnd_add_reverse_edges(int64_t N, int32_t R, uint64_t *keys, int32_t *deg, void *stream)
{
    return rnnd_add_reverse_edges_wide(N, R, R, keys, deg, stream);
}

extern "C" int rnnd_export_graph(int64_t N, int32_t R, const uint64_t *keys, const int32_t *deg,
                                 int32_t *graph_out, int32_t *degree_out, void *stream)
{
    int rc = RNND_OK;
    if (!keys || !deg || !graph_out || !degree_out) return RNND_ERR_NULL;
    if (N < 1 || N > 2147483646LL) return RNND_ERR_BAD_SHAPE;
    if (R < 1 || R > RNND_MAX_R) return RNND_ERR_BAD_PARAM;
    hipStream_t st = (hipStream_t)stream;
    launch_export(N, R, (const u64 *)keys, deg, graph_out, degree_out, st);
    HIPCHK(hipGetLastError());
    HIPCHK(hipStreamSynchronize(st));
done:
    return rc;
}

extern "C" int rnnd_search(const void *X, int64_t N, int32_t d, int dtype, int metric, const int32_t *graph,
                           const int32_t *degree, int32_t row_stride, const void *Q, int64_t nq, int32_t L,
                           int32_t K, int32_t k, uint64_t seed, int32_t *out_ids, uint32_t *out_dist_bits,
                           int64_t *dist_evals, void *stream)
{
    int rc = check_data_args(X, N, d, dtype, metric, 1);
    if (rc) return rc;
    if (nq < 0 || nq > 2147483646LL) return RNND_ERR_BAD_SHAPE;
    if (row_stride < 1 || L < 1 || L > SEARCH_MAX_L || K < 1 || k < 1 || k > L) return RNND_ERR_BAD_PARAM;
    if (!graph || !degree || ((!out_ids || !Q) && nq > 0)) return RNND_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    if (dist_evals) *dist_evals = 0;
    if (nq == 0) return RNND_OK;
    const size_t rowbytes = (size_t)d * dt_size(dtype);
    const int vec_ok = (rowbytes % 16 == 0) && (((uintptr_t)X) % 16 == 0) && (((uintptr_t)Q) % 16 == 0);
    // one bitmap of N bits per wavefront in flight; at most 1 GiB of them, at most 8 wavefronts per SIMD
    const size_t bitmap_words = (((size_t)N + 31) / 32 + 63) / 64 * 64;
    long long waves = (long long)cu_count() * 32;
    const long long by_mem = (long long)((1ull << 30) / (bitmap_words * 4));
    if (waves > by_mem) waves = by_mem;
    if (waves > nq) waves = nq;
    if (waves < 1) waves = 1;
    const unsigned blocks = (unsigned)((waves + 3) / 4);
    const size_t bm_bytes = (size_t)blocks * 4 * bitmap_words * 4;
    char *base = nullptr;
    unsigned long long h_evals = 0;
    WsLease lease;
    rc = ws_acquire(bm_bytes + 256, false, st, &lease);      // the block kept between calls, like the builds' workspace
    if (rc) return rc;
    base = lease.base;
    // the evaluation counter; the bitmaps are cleared by their wavefronts before every query
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, st, (u32 *)(base + bm_bytes), (size_t)64);
    {
        u32 *bitmaps = (u32 *)base;
        unsigned long long *d_evals = (unsigned long long *)(base + bm_bytes);
#define RNND_SEARCH_LAUNCH(DT, E)                                                                            \
    hipLaunchKernelGGL((k_search<DT, E>), dim3(blocks), dim3(256), 0, st, X, (long long)N, d, vec_ok, graph, \
                       degree, row_stride, Q, (long long)nq, L, K, k, (u64)seed, bitmaps, bitmap_words,      \
                       out_ids, out_dist_bits, d_evals)
        if (dtype == RNND_U8) {
            if (L <= 64) RNND_SEARCH_LAUNCH(DT_U8, 1); else RNND_SEARCH_LAUNCH(DT_U8, 2);
        } else if (dtype == RNND_F16) {
            if (L <= 64) RNND_SEARCH_LAUNCH(DT_F16, 1); else RNND_SEARCH_LAUNCH(DT_F16, 2);
        } else if (dtype == RNND_BF16) {
            if (L <= 64) RNND_SEARCH_LAUNCH(DT_BF16, 1); else RNND_SEARCH_LAUNCH(DT_BF16, 2);
        } else {
            if (L <= 64) RNND_SEARCH_LAUNCH(DT_F32, 1); else RNND_SEARCH_LAUNCH(DT_F32, 2);
        }
#undef RNND_SEARCH_LAUNCH
        HIPCHK(hipGetLastError());
        HIPCHK(hipMemcpyAsync(&h_evals, d_evals, sizeof h_evals, hipMemcpyDeviceToHost, st));
        HIPCHK(hipStreamSynchronize(st));
        if (dist_evals) *dist_evals = (int64_t)h_evals;
    }
done:
    if (rc == RNND_ERR_HIP || rc == RNND_ERR_OOM) (void)hipStreamSynchronize(st);
    ws_release(&lease);
    return rc;
}

template <int LPR>
static void launch_probe_gather(const void *X, u32 n_rows, u32 pieces, u64 trips, u64 seed, u32 *sink, int blocks,
                                hipStream_t st)
{
    hipLaunchKernelGGL(k_probe_gather<LPR>, dim3(blocks), dim3(256), 0, st, (const uint4 *)X, n_rows, pieces, trips,
                       seed, sink);
}

template <int LPR>
static void launch_probe_gather_map(int ppl, const void *X, u32 n_rows, u64 trips, u64 seed, u32 *sink, int blocks,
                                    hipStream_t st)
{
    const uint4 *x = (const uint4 *)X;
    if (ppl == 1) hipLaunchKernelGGL((k_probe_gather_map<LPR, 1>), dim3(blocks), dim3(256), 0, st, x, n_rows, trips, seed, sink);
    else if (ppl == 2) hipLaunchKernelGGL((k_probe_gather_map<LPR, 2>), dim3(blocks), dim3(256), 0, st, x, n_rows, trips, seed, sink);
    else if (ppl == 4) hipLaunchKernelGGL((k_probe_gather_map<LPR, 4>), dim3(blocks), dim3(256), 0, st, x, n_rows, trips, seed, sink);
    else hipLaunchKernelGGL((k_probe_gather_map<LPR, 8>), dim3(blocks), dim3(256), 0, st, x, n_rows, trips, seed, sink);
}

// lanes_per_row 0: the probe of the benchmark line (the largest power of two that divides the number of 16-byte
// pieces, at most 8 lanes per row; four rows per lane in flight, any row length); otherwise the map probe
static int probe_gather_impl(const void *X, int64_t n_rows, int64_t row_bytes, int64_t n_gather, int lanes_per_row,
                             uint64_t seed, double *gbytes_per_s, void *stream)
{
    int rc = RNND_OK;
    if (!X || !gbytes_per_s) return RNND_ERR_NULL;
    if (n_rows < 1 || n_rows > 2147483646LL || n_gather < 1) return RNND_ERR_BAD_SHAPE;
    if (row_bytes < 16 || row_bytes % 16 != 0 || row_bytes > (1 << 20) || ((uintptr_t)X & 15) != 0)
        return RNND_ERR_BAD_PARAM;
    hipStream_t st = (hipStream_t)stream;
    const u32 pieces = (u32)(row_bytes / 16);
    int ppl = 0;        // pieces per lane of the map probe
    if (lanes_per_row != 0) {
        if (lanes_per_row != 1 && lanes_per_row != 2 && lanes_per_row != 4 && lanes_per_row != 8) return RNND_ERR_BAD_PARAM;
        if (pieces % (u32)lanes_per_row != 0) return RNND_ERR_BAD_PARAM;
        ppl = (int)(pieces / (u32)lanes_per_row);
        if (ppl != 1 && ppl != 2 && ppl != 4 && ppl != 8) return RNND_ERR_BAD_PARAM;
    }
    const int lpr = lanes_per_row ? lanes_per_row : pieces % 8 == 0 ? 8 : pieces % 4 == 0 ? 4 : pieces % 2 == 0 ? 2 : 1;
    const int rows_per_trip = ppl ? (8 / ppl) * (64 / lpr) : 4 * (64 / lpr);
    const u64 trips = ((u64)n_gather + rows_per_trip - 1) / rows_per_trip;
    const int blocks = persistent_blocks();
    u32 *sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    float ms = 0;
    HIPCHK(hipMalloc((void **)&sink, (size_t)blocks * 256 * 4));
    HIPCHK(hipEventCreate(&e0));
    HIPCHK(hipEventCreate(&e1));
    for (int rep = 0; rep < 2; ++rep) {     // the second pass is the one that is timed
        HIPCHK(hipEventRecord(e0, st));
        if (ppl) {
            if (lpr == 8) launch_probe_gather_map<8>(ppl, X, (u32)n_rows, trips, seed + rep, sink, blocks, st);
            else if (lpr == 4) launch_probe_gather_map<4>(ppl, X, (u32)n_rows, trips, seed + rep, sink, blocks, st);
            else if (lpr == 2) launch_probe_gather_map<2>(ppl, X, (u32)n_rows, trips, seed + rep, sink, blocks, st);
            else launch_probe_gather_map<1>(ppl, X, (u32)n_rows, trips, seed + rep, sink, blocks, st);
        } else if (lpr == 8) launch_probe_gather<8>(X, (u32)n_rows, pieces, trips, seed + rep, sink, blocks, st);
        else if (lpr == 4) launch_probe_gather<4>(X, (u32)n_rows, pieces, trips, seed + rep, sink, blocks, st);
        else if (lpr == 2) launch_probe_gather<2>(X, (u32)n_rows, pieces, trips, seed + rep, sink, blocks, st);
        else launch_probe_gather<1>(X, (u32)n_rows, pieces, trips, seed + rep, sink, blocks, st);
        HIPCHK(hipGetLastError());
        HIPCHK(hipEventRecord(e1, st));
        HIPCHK(hipStreamSynchronize(st));
    }
    HIPCHK(hipEventElapsedTime(&ms, e0, e1));
    *gbytes_per_s = ms > 0 ? (double)trips * rows_per_trip * (double)row_bytes / (ms * 1e-3) / 1e9 : 0.0;
done:
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    return rc;
}

extern "C" int rnnd_probe_gather(const void *X, int64_t n_rows, int64_t row_bytes, int64_t n_gather, uint64_t seed,
                                 double *gbytes_per_s, void *stream)
{
    return probe_gather_impl(X, n_rows, row_bytes, n_gather, 0, seed, gbytes_per_s, stream);
}

extern "C" int rnnd_probe_gather_map(const void *X, int64_t n_rows, int64_t row_bytes, int64_t n_gather,
                                     int lanes_per_row, uint64_t seed, double *gbytes_per_s, void *stream)
{
    if (lanes_per_row == 0) return RNND_ERR_BAD_PARAM;
    return probe_gather_impl(X, n_rows, row_bytes, n_gather, lanes_per_row, seed, gbytes_per_s, stream);
}

// 0: automatic; 1: generic scan for every input; 2: automatic, but the float matrix-core scan runs in
// double precision only (no single-precision first pass)
extern "C" int rnnd_set_kernel_variant(int variant)
{
    if (variant < 0 || variant > 2) return RNND_ERR_BAD_PARAM;
    g_kernel_variant = variant;
    return RNND_OK;
}

extern "C" int rnnd_set_scan_launches(int mode)
{
    if (mode < 0 || mode > 3) return RNND_ERR_BAD_PARAM;
    g_scan_launches = mode;
    return RNND_OK;
}

extern "C" int rnnd_set_event_timing(int on)
{
    g_event_timing = on ? 1 : 0;
    return RNND_OK;
}

extern "C" int rnnd_set_transpose_path(int path)
{
    if (path < 0 || path > 2) return RNND_ERR_BAD_PARAM;
    g_transpose_path = path;
    return RNND_OK;
}

extern "C" const char *rnnd_strerror(int status)
{
    switch (status) {
    case RNND_OK: return "ok";
    case RNND_ERR_NULL: return "a required pointer is NULL";
    case RNND_ERR_BAD_SHAPE: return "bad shape (N < 2, N too large, d < 1, or uint8 d > 33025)";
    case RNND_ERR_BAD_PARAM: return "bad parameter (S, R, T1 or T2 out of range)";
    case RNND_ERR_UNSUPPORTED: return "unsupported dtype or metric";
    case RNND_ERR_OOM: return "out of device memory";
    case RNND_ERR_SCRATCH: return "the workspace for these sizes does not fit the static scratch array (rnnd_build_static)";
    case RNND_ERR_HIP: return g_last_hip_error[0] ? g_last_hip_error : "HIP error";
    default: return "unknown status";
    }
}

extern "C" int rnnd_version(void) { return 200; }
