// librnnd: Relative NN-Descent graph construction (arXiv 2310.20419, Alg. 4-6) on gfx950.
// One wavefront owns one vertex in every per-vertex kernel; rounds are synchronous: a scan kernel
// reads the snapshot and emits redirected edges, a merge kernel rebuilds the touched lists.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../include/rnnd.h"
#include "dist.h"
#include "wave_prims.h"

#define WAVES_PER_BLOCK 4
#define BLOCK (64 * WAVES_PER_BLOCK)
#define GOLDEN64 0x9E3779B97F4A7C15ull

// Per-round device counters.  Round t reads ctr[t].n_active and fills the rest; its merge step
// writes ctr[t+1].n_active.  Zeroed once per call, never reset, so they double as statistics.
struct RoundCtr {
    u32 n_active;      // length of this round's active list
    u32 n_props;       // redirected edges emitted
    u32 n_touched;     // distinct targets of those edges
    u32 bin_cursor;    // space handed out in the bin array
    u64 algo_evals;
    u64 exec_evals;
    u64 gathered_rows;
    u64 pad;
};

struct Prop {          // one redirected edge (Alg. 4 line 13): `key` enters `tgt`'s list
    u64 key;
    u32 tgt;
    u32 slot;          // arrival number among the edges for tgt (gives its place in tgt's bin)
};

// ------------------------------------------------------------------ RandomGraph
__device__ __forceinline__ u64 mix64(u64 z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

// Alg. 6 lines 1-2.  Draws are examined 64 at a time; a draw is accepted iff its id differs from
// every earlier draw's id, which is the same set, in the same order, as accepting one by one.
template <int DT>
__global__ __launch_bounds__(BLOCK) void k_random_graph(const void *X, long long N, int d, int vec_ok,
                                                        int S, int R, u64 seed, u64 *keys, int *deg,
                                                        int *active, u32 *n_active)
{
    __shared__ int s_ids[WAVES_PER_BLOCK][RNND_MAX_R];
    __shared__ u32 s_dist[WAVES_PER_BLOCK][RNND_MAX_R];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, sub = lane & 7, grp = lane >> 3;
    const long long u = (long long)blockIdx.x * WAVES_PER_BLOCK + wave;
    if (u >= N) return;
    int *ids = s_ids[wave];
    const size_t rowbytes = (size_t)d * (DT == DT_U8 ? 1 : 4);
    const u64 hu = mix64(seed + GOLDEN64 * (u64)(u + 1));
    const u64 jmax = 64ull * (u64)S + 1024ull;
    int cnt = 0;
    for (u64 j0 = 0; j0 < jmax && cnt < S; j0 += 64) {
        u64 j = j0 + lane;
        u64 z = mix64(hu + GOLDEN64 * (j + 1));
        u64 c = ((z >> 32) * (u64)(N - 1)) >> 32;
        int id = (int)(c + (c >= (u64)u ? 1 : 0));
        bool ok = j < jmax;
        for (int k = 0; k < cnt; ++k) ok = ok && (ids[k] != id);
        for (int l = 0; l < 63; ++l) {
            int o = __shfl(id, l);
            if (l < lane && o == id) ok = false;
        }
        u64 m = __builtin_amdgcn_ballot_w64(ok);
        int pos = cnt + __popcll(m & lanes_below(lane));
        if (ok && pos < S) ids[pos] = id;
        cnt += __popcll(m);
        if (cnt > S) cnt = S;
        wave_sync();
    }
    if (cnt < S) {   // fallback, practically unreachable: smallest unused ids
        for (long long id = 0; id < N && cnt < S; ++id) {
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
    // delta(u, id): 8 rows at a time, 8 lanes per row
    const char *xu = (const char *)X + (size_t)u * rowbytes;
    for (int b = 0; b < S; b += 8) {
        int p = b + grp;
        int id = ids[p < S ? p : S - 1];
        u32 db = group8_dist_bits<DT>(xu, (const char *)X + (size_t)id * rowbytes, d, vec_ok, sub);
        if (p < S && sub == 0) s_dist[wave][p] = db;
    }
    wave_sync();
    u64 k[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        int e = r * 64 + lane;
        k[r] = e < S ? make_key(s_dist[wave][e], (u32)ids[e], 1u) : KEY_PAD;
    }
    wave_sort<2>(k, lane);
    u64 *row = keys + (size_t)u * R;
    if (lane < S) row[lane] = k[0];
    if (lane + 64 < S) row[lane + 64] = k[1];
    if (lane == 0) {
        deg[u] = S;
        active[u] = (int)u;
        if (u == 0 && n_active) *n_active = (u32)N;   // every vertex starts with "new" entries
    }
}

// ------------------------------------------------- UpdateNeighbors: scan (generic kernel)
// Alg. 4 lines 2-15 for one vertex per wavefront, in the algorithm's own order: v runs over the
// sorted list; the kept set U' so far is a bit mask; the delta(v,w) of up to 8 eligible w (kept,
// not old/old) are evaluated at once by 8-lane groups in ascending w, and the first failing one
// prunes v and redirects it.  Kept entries are written back in place with the flag cleared.
template <int DT>
__global__ __launch_bounds__(BLOCK) void k_update_scan(const void *X, int d, int vec_ok, int R,
                                                       u64 *keys, int *deg, const int *active,
                                                       RoundCtr *ctr, Prop *props, int *cnt,
                                                       int *touched)
{
    __shared__ u64 s_key[WAVES_PER_BLOCK][RNND_MAX_R];
    __shared__ u64 s_pkey[WAVES_PER_BLOCK][RNND_MAX_R];
    __shared__ u32 s_ptgt[WAVES_PER_BLOCK][RNND_MAX_R];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, sub = lane & 7, grp = lane >> 3;
    const u32 gw = blockIdx.x * WAVES_PER_BLOCK + wave, nw = gridDim.x * WAVES_PER_BLOCK;
    const u32 n_active = ctr->n_active;
    const size_t rowbytes = (size_t)d * (DT == DT_U8 ? 1 : 4);
    u64 *sk = s_key[wave];
    u64 evals_algo = 0, evals_exec = 0, rows = 0;
    for (u32 it = gw; it < n_active; it += nw) {
        const int u = active[it];
        const int m = deg[u];
        u64 *row = keys + (size_t)u * R;
        u64 k0 = lane < m ? row[lane] : KEY_PAD;
        u64 k1 = lane + 64 < m ? row[lane + 64] : KEY_PAD;
        wave_sync();
        sk[lane] = k0;
        sk[lane + 64] = k1;
        const u64 new0 = __builtin_amdgcn_ballot_w64(lane < m && (k0 & 1ull));
        const u64 new1 = __builtin_amdgcn_ballot_w64(lane + 64 < m && (k1 & 1ull));
        wave_sync();
        if ((new0 | new1) == 0) continue;
        rows += m;
        u64 K0 = 0, K1 = 0;   // U' as positions in the sorted list
        int np = 0;
        for (int i = 0; i < m; ++i) {
            const u64 ki = sk[i];
            const u32 di = key_dist(ki), idv = key_id(ki);
            const bool newv = ki & 1ull;
            u64 e0 = newv ? K0 : (K0 & new0);   // lines 8-9: old/old pairs are skipped
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
                const bool fail = mypos >= 0 && di >= db;   // line 11
                const u64 fm = __builtin_amdgcn_ballot_w64(fail && sub == 0);
                if (fm) {
                    const int fl = __builtin_ctzll(fm);     // first failing w in list order
                    const u32 fdb = __shfl(db, fl), fidw = __shfl(idw, fl);
                    if (lane == 0) {                        // line 13: (u,v) leaves, (w,v) enters
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
                if (i < 64) K0 |= 1ull << i; else K1 |= 1ull << (i - 64);   // lines 17-18
            }
        }
        // line 15 + compaction: kept entries, flag old, back into the row
        const int nk0 = __popcll(K0);
        if ((K0 >> lane) & 1ull) row[__popcll(K0 & lanes_below(lane))] = k0 & ~1ull;
        if ((K1 >> lane) & 1ull) row[nk0 + __popcll(K1 & lanes_below(lane))] = k1 & ~1ull;
        if (lane == 0) deg[u] = nk0 + __popcll(K1);
        wave_sync();
        if (np > 0) {
            u32 base = 0;
            if (lane == 0) base = atomicAdd(&ctr->n_props, (u32)np);
            base = __shfl(base, 0);
            for (int p = lane; p < np; p += 64) {
                const u32 tgt = s_ptgt[wave][p];
                const u32 slot = (u32)atomicAdd(&cnt[tgt], 1);
                if (slot == 0) touched[atomicAdd(&ctr->n_touched, 1u)] = (int)tgt;
                Prop pr;
                pr.key = s_pkey[wave][p];
                pr.tgt = tgt;
                pr.slot = slot;
                props[base + p] = pr;
            }
        }
    }
    if (lane == 0 && rows) {
        atomicAdd(&ctr->algo_evals, evals_algo);
        atomicAdd(&ctr->exec_evals, evals_exec);
        atomicAdd(&ctr->gathered_rows, rows);
    }
}

// ------------------------------------------------------ UpdateNeighbors: merge
__global__ void k_bin_offsets(const int *touched, const int *cnt, int *binoff, RoundCtr *ctr)
{
    const u32 n = ctr->n_touched;
    for (u32 i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        int x = touched[i];
        binoff[x] = (int)atomicAdd(&ctr->bin_cursor, (u32)cnt[x]);
    }
}

__global__ void k_bin_scatter(const Prop *props, const int *binoff, u64 *bins, const RoundCtr *ctr)
{
    const u32 n = ctr->n_props;
    for (u32 i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        Prop p = props[i];
        bins[(size_t)binoff[p.tgt] + p.slot] = p.key;
    }
}

// For every touched vertex x: list <- first R distinct of (kept entries + edges redirected to x).
// Vertices whose new list holds a "new" entry form the next round's active list.
__global__ __launch_bounds__(BLOCK) void k_merge(int R, u64 *keys, int *deg, const int *touched,
                                                 int *cnt, const int *binoff, const u64 *bins,
                                                 const RoundCtr *ctr, RoundCtr *next, int *active_next)
{
    __shared__ u64 s_stage[WAVES_PER_BLOCK][RNND_MAX_R];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const u32 gw = blockIdx.x * WAVES_PER_BLOCK + wave, nw = gridDim.x * WAVES_PER_BLOCK;
    const u32 n = ctr->n_touched;
    for (u32 it = gw; it < n; it += nw) {
        const int x = touched[it];
        bool any_new = false;
        const int nd = wave_merge_row(keys + (size_t)x * R, deg[x], bins + binoff[x], cnt[x], R,
                                      s_stage[wave], lane, &any_new);
        if (lane == 0) {
            deg[x] = nd;
            cnt[x] = 0;
            if (any_new) active_next[atomicAdd(&next->n_active, 1u)] = x;
        }
    }
}

// ------------------------------------------------------------ AddReverseEdges
// cnt[v] += 1 for every edge (u, v)
__global__ __launch_bounds__(BLOCK) void k_count_targets(long long N, int R, const u64 *keys,
                                                         const int *deg, int *cnt)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long u = (long long)blockIdx.x * WAVES_PER_BLOCK + wave;
    if (u >= N) return;
    const int m = deg[u];
    for (int e = lane; e < m; e += 64) atomicAdd(&cnt[key_id(keys[(size_t)u * R + e])], 1);
}

// Gives every vertex with cnt[v] > min_cnt a bin of cnt[v] keys; others get binoff = -1.
// Clears fill[] and (thread 0) the counter the next step appends to.
__global__ void k_assign_bins(long long N, const int *cnt, int min_cnt, int *binoff, int *fill,
                              u32 *cursor, int *list, u32 *n_list, u64 *thr)
{
    long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= N) return;
    fill[v] = 0;
    if (thr) thr[v] = KEY_PAD;
    if (cnt[v] > min_cnt) {
        binoff[v] = (int)atomicAdd(cursor, (u32)cnt[v]);
        if (list) list[atomicAdd(n_list, 1u)] = (int)v;
    } else {
        binoff[v] = -1;
    }
}

// For every edge (u, v) whose v owns a bin: bins[v] <- key(delta, u, flag)
__global__ __launch_bounds__(BLOCK) void k_fill_bins(long long N, int R, const u64 *keys, const int *deg,
                                                     const int *binoff, int *fill, u64 *bins, u32 flag)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long u = (long long)blockIdx.x * WAVES_PER_BLOCK + wave;
    if (u >= N) return;
    const int m = deg[u];
    for (int e = lane; e < m; e += 64) {
        const u64 k = keys[(size_t)u * R + e];
        const u32 v = key_id(k);
        const int off = binoff[v];
        if (off >= 0) bins[(size_t)off + atomicAdd(&fill[v], 1)] = make_key(key_dist(k), (u32)u, flag);
    }
}

// Alg. 5 lines 1-5: list(x) <- first R distinct of list(x) + reversed edges into x (flag new).
__global__ __launch_bounds__(BLOCK) void k_reverse_merge(long long N, int R, u64 *keys, int *deg,
                                                         int *cnt, const int *binoff, const u64 *bins)
{
    __shared__ u64 s_stage[WAVES_PER_BLOCK][RNND_MAX_R];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long x = (long long)blockIdx.x * WAVES_PER_BLOCK + wave;
    if (x >= N) return;
    const int c = cnt[x];
    if (c > 0) {
        bool any_new;
        const int nd = wave_merge_row(keys + (size_t)x * R, deg[x], bins + binoff[x], c, R,
                                      s_stage[wave], lane, &any_new);
        if (lane == 0) deg[x] = nd;
    }
    if (lane == 0) cnt[x] = 0;
}

// Alg. 5 lines 6-8, first half: thr[v] <- the R-th smallest (delta, source) among the edges into v.
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
        const int nd = wave_merge_row(s_row[wave], 0, bins + binoff[v], cnt[v], R, s_stage[wave], lane,
                                      &any_new);
        wave_sync();
        if (lane == 0) thr[v] = s_row[wave][nd - 1];
    }
}

// Alg. 5 lines 6-8, second half: edge (u, v) survives iff (delta, u) <= thr[v].  Also rebuilds the
// active list (vertices holding a "new" entry) for the next UpdateNeighbors round and clears cnt.
__global__ __launch_bounds__(BLOCK) void k_incap_filter(long long N, int R, u64 *keys, int *deg,
                                                        const u64 *thr, int *cnt, RoundCtr *next,
                                                        int *active_next)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long u = (long long)blockIdx.x * WAVES_PER_BLOCK + wave;
    if (u >= N) return;
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
        deg[u] = c0 + __popcll(m1);
        cnt[u] = 0;
        if (n0 | n1) active_next[atomicAdd(&next->n_active, 1u)] = (int)u;
    }
}

__global__ void k_zero_u32(u32 *p, int n)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// Rebuilds the active list from the flags of a snapshot handed in by the caller.
__global__ __launch_bounds__(BLOCK) void k_collect_active(long long N, int R, const u64 *keys,
                                                          const int *deg, RoundCtr *next, int *active_next)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long u = (long long)blockIdx.x * WAVES_PER_BLOCK + wave;
    if (u >= N) return;
    const int m = deg[u];
    bool nw = false;
    for (int e = lane; e < m; e += 64) nw = nw || (keys[(size_t)u * R + e] & 1ull);
    const u64 b = __builtin_amdgcn_ballot_w64(nw);
    if (lane == 0 && b) active_next[atomicAdd(&next->n_active, 1u)] = (int)u;
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

// ===================================================================== host side
#define HIPCHK(x)                                                                  \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            snprintf(g_last_hip_error, sizeof g_last_hip_error, "%s: %s", #x, hipGetErrorString(e_)); \
            rc = (e_ == hipErrorOutOfMemory) ? RNND_ERR_OOM : RNND_ERR_HIP;        \
            goto done;                                                             \
        }                                                                          \
    } while (0)

static char g_last_hip_error[512];
static int g_kernel_variant = 0;

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

struct Workspace {
    char *base = nullptr;
    size_t bytes = 0;
    u64 *keys = nullptr;    // [N*R]   (unless the caller supplies a snapshot)
    int *deg = nullptr;     // [N]
    Prop *props = nullptr;  // [N*R]
    u64 *bins = nullptr;    // [N*R]
    u64 *thr = nullptr;     // [N]
    int *cnt = nullptr, *binoff = nullptr, *fill = nullptr, *touched = nullptr, *hubs = nullptr;
    int *active[2] = {nullptr, nullptr};
    RoundCtr *ctr = nullptr;   // [n_ctr]
    u32 *misc = nullptr;       // [8]: small cursors for AddReverseEdges
    int n_ctr = 0;
};

static size_t ws_layout(Workspace &w, long long N, int R, int n_ctr, bool own_graph)
{
    size_t off = 0;
    auto take = [&](size_t b) { size_t o = off; off += align_up(b); return o; };
    size_t o_keys = own_graph ? take((size_t)N * R * 8) : 0;
    size_t o_deg = own_graph ? take((size_t)N * 4) : 0;
    size_t o_props = take((size_t)N * R * sizeof(Prop));
    size_t o_bins = take((size_t)N * R * 8);
    size_t o_thr = take((size_t)N * 8);
    size_t o_cnt = take((size_t)N * 4), o_binoff = take((size_t)N * 4), o_fill = take((size_t)N * 4);
    size_t o_touched = take((size_t)N * 4), o_hubs = take((size_t)N * 4);
    size_t o_a0 = take((size_t)N * 4), o_a1 = take((size_t)N * 4);
    size_t o_ctr = take((size_t)n_ctr * sizeof(RoundCtr));
    size_t o_misc = take(8 * 4);
    if (w.base) {
        if (own_graph) { w.keys = (u64 *)(w.base + o_keys); w.deg = (int *)(w.base + o_deg); }
        w.props = (Prop *)(w.base + o_props);
        w.bins = (u64 *)(w.base + o_bins);
        w.thr = (u64 *)(w.base + o_thr);
        w.cnt = (int *)(w.base + o_cnt);
        w.binoff = (int *)(w.base + o_binoff);
        w.fill = (int *)(w.base + o_fill);
        w.touched = (int *)(w.base + o_touched);
        w.hubs = (int *)(w.base + o_hubs);
        w.active[0] = (int *)(w.base + o_a0);
        w.active[1] = (int *)(w.base + o_a1);
        w.ctr = (RoundCtr *)(w.base + o_ctr);
        w.misc = (u32 *)(w.base + o_misc);
        w.n_ctr = n_ctr;
    }
    return off;
}

static int check_data_args(const void *X, long long N, int d, int dtype, int metric, int R)
{
    if (!X) return RNND_ERR_NULL;
    if (dtype != RNND_U8 && dtype != RNND_F32) return RNND_ERR_UNSUPPORTED;
    if (metric != RNND_L2SQ) return RNND_ERR_UNSUPPORTED;
    if (N < 2 || N > 2147483646LL || d < 1) return RNND_ERR_BAD_SHAPE;
    if (dtype == RNND_U8 && d > 33025) return RNND_ERR_BAD_SHAPE;
    if (R < 1 || R > RNND_MAX_R) return RNND_ERR_BAD_PARAM;
    return RNND_OK;
}

static int vec_ok_for(const void *X, int d, int dtype)
{
    size_t rowbytes = (size_t)d * (dtype == RNND_U8 ? 1 : 4);
    return (rowbytes % 16 == 0) && (((uintptr_t)X) % 16 == 0);
}

static int persistent_blocks()
{
    static int nb = 0;
    if (!nb) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        nb = cus * 8;   // 32 wavefronts per CU
    }
    return nb;
}

static inline int vertex_blocks(long long N) { return (int)((N + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK); }

// One synchronous UpdateNeighbors round t (ctr[t] -> ctr[t+1]).
static hipError_t launch_update_round(const Workspace &w, const void *X, int d, int dtype, int vec_ok,
                                      int R, u64 *keys, int *deg, int t, hipStream_t st,
                                      hipEvent_t after_scan = nullptr)
{
    const int pb = persistent_blocks();
    RoundCtr *c = w.ctr + t;
    const int *act = w.active[t & 1];
    int *act_next = w.active[(t + 1) & 1];
    if (dtype == RNND_U8)
        hipLaunchKernelGGL(k_update_scan<DT_U8>, dim3(pb), dim3(BLOCK), 0, st, X, d, vec_ok, R, keys, deg,
                           act, c, w.props, w.cnt, w.touched);
    else
        hipLaunchKernelGGL(k_update_scan<DT_F32>, dim3(pb), dim3(BLOCK), 0, st, X, d, vec_ok, R, keys, deg,
                           act, c, w.props, w.cnt, w.touched);
    if (after_scan) (void)hipEventRecord(after_scan, st);
    hipLaunchKernelGGL(k_bin_offsets, dim3(pb), dim3(256), 0, st, w.touched, w.cnt, w.binoff, c);
    hipLaunchKernelGGL(k_bin_scatter, dim3(pb), dim3(256), 0, st, w.props, w.binoff, w.bins, c);
    hipLaunchKernelGGL(k_merge, dim3(pb), dim3(BLOCK), 0, st, R, keys, deg, w.touched, w.cnt, w.binoff,
                       w.bins, c, c + 1, act_next);
    return hipGetLastError();
}

// AddReverseEdges; the active list for round t_next is rebuilt from scratch.
static hipError_t launch_reverse(const Workspace &w, long long N, int R, u64 *keys, int *deg, int t_next,
                                 hipStream_t st)
{
    const int vb = vertex_blocks(N), tb = (int)((N + 255) / 256);
    RoundCtr *next = w.ctr + t_next;
    int *act_next = w.active[t_next & 1];
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, st, w.misc, 8);
    hipLaunchKernelGGL(k_zero_u32, dim3(1), dim3(64), 0, st, &next->n_active, 1);
    // lines 1-5: union with reversed edges, out-lists cut to R
    hipLaunchKernelGGL(k_count_targets, dim3(vb), dim3(BLOCK), 0, st, N, R, keys, deg, w.cnt);
    hipLaunchKernelGGL(k_assign_bins, dim3(tb), dim3(256), 0, st, N, w.cnt, 0, w.binoff, w.fill, w.misc + 0,
                       (int *)nullptr, (u32 *)nullptr, (u64 *)nullptr);
    hipLaunchKernelGGL(k_fill_bins, dim3(vb), dim3(BLOCK), 0, st, N, R, keys, deg, w.binoff, w.fill, w.bins, 1u);
    hipLaunchKernelGGL(k_reverse_merge, dim3(vb), dim3(BLOCK), 0, st, N, R, keys, deg, w.cnt, w.binoff, w.bins);
    // lines 6-8: in-lists cut to R; only vertices with more than R incoming edges need a bin
    hipLaunchKernelGGL(k_count_targets, dim3(vb), dim3(BLOCK), 0, st, N, R, keys, deg, w.cnt);
    hipLaunchKernelGGL(k_assign_bins, dim3(tb), dim3(256), 0, st, N, w.cnt, R, w.binoff, w.fill, w.misc + 1,
                       w.hubs, w.misc + 2, w.thr);
    hipLaunchKernelGGL(k_fill_bins, dim3(vb), dim3(BLOCK), 0, st, N, R, keys, deg, w.binoff, w.fill, w.bins, 0u);
    hipLaunchKernelGGL(k_incap_threshold, dim3(persistent_blocks()), dim3(BLOCK), 0, st, R, w.hubs, w.misc + 2,
                       w.cnt, w.binoff, w.bins, w.thr);
    hipLaunchKernelGGL(k_incap_filter, dim3(vb), dim3(BLOCK), 0, st, N, R, keys, deg, w.thr, w.cnt, next,
                       act_next);
    return hipGetLastError();
}

static void fill_round_stats(rnnd_stats *s, const RoundCtr *h, int rounds)
{
    s->rounds = rounds;
    for (int t = 0; t < rounds && t < RNND_MAX_ROUNDS; ++t) {
        s->active[t] = h[t].n_active;
        s->proposals[t] = h[t].n_props;
        s->algo_evals[t] = (int64_t)h[t].algo_evals;
        s->exec_evals[t] = (int64_t)h[t].exec_evals;
        s->gathered_rows[t] = (int64_t)h[t].gathered_rows;
    }
}

extern "C" int rnnd_workspace_bytes(int64_t N, int32_t d, int dtype, int32_t R, size_t *bytes)
{
    if (!bytes) return RNND_ERR_NULL;
    if (dtype != RNND_U8 && dtype != RNND_F32) return RNND_ERR_UNSUPPORTED;
    if (N < 2 || N > 2147483646LL || d < 1) return RNND_ERR_BAD_SHAPE;
    if (R < 1 || R > RNND_MAX_R) return RNND_ERR_BAD_PARAM;
    Workspace w;
    *bytes = ws_layout(w, N, R, RNND_MAX_ROUNDS + 2, true);
    return RNND_OK;
}

extern "C" int rnnd_build_ex(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S,
                             int32_t R, int32_t T1, int32_t T2, uint64_t seed, int32_t *graph_out,
                             int32_t *degree_out, uint64_t *keys_out, rnnd_stats *stats, void *stream)
{
    int rc = check_data_args(X, N, d, dtype, metric, R);
    if (rc) return rc;
    if (!graph_out || !degree_out) return RNND_ERR_NULL;
    if (S < 1 || S > R || (int64_t)S > N - 1 || T1 < 1 || T2 < 1) return RNND_ERR_BAD_PARAM;
    if ((int64_t)T1 * T2 > 1000000) return RNND_ERR_BAD_PARAM;
    hipStream_t st = (hipStream_t)stream;
    const int rounds = T1 * T2, n_ctr = rounds + 2, vec_ok = vec_ok_for(X, d, dtype);
    // events: start, after init, (after scan, after round) per round, after each reverse, end
    const int n_ev = 2 * rounds + T1 + 3;
    Workspace w;
    hipEvent_t *ev = nullptr;
    RoundCtr *hctr = nullptr;
    int n_ev_made = 0;
    w.bytes = ws_layout(w, N, R, n_ctr, true);
    HIPCHK(hipMalloc((void **)&w.base, w.bytes));
    ws_layout(w, N, R, n_ctr, true);
    ev = (hipEvent_t *)calloc(n_ev, sizeof(hipEvent_t));
    hctr = (RoundCtr *)calloc(n_ctr, sizeof(RoundCtr));
    if (!ev || !hctr) { rc = RNND_ERR_OOM; goto done; }
    for (; n_ev_made < n_ev; ++n_ev_made) HIPCHK(hipEventCreate(&ev[n_ev_made]));
    {
        int e = 0, t = 0;
        HIPCHK(hipEventRecord(ev[e++], st));
        HIPCHK(hipMemsetAsync(w.ctr, 0, (size_t)n_ctr * sizeof(RoundCtr), st));
        HIPCHK(hipMemsetAsync(w.cnt, 0, (size_t)N * 4, st));
        if (dtype == RNND_U8)
            hipLaunchKernelGGL(k_random_graph<DT_U8>, dim3(vertex_blocks(N)), dim3(BLOCK), 0, st, X, (long long)N, d,
                               vec_ok, S, R, (u64)seed, w.keys, w.deg, w.active[0], &w.ctr[0].n_active);
        else
            hipLaunchKernelGGL(k_random_graph<DT_F32>, dim3(vertex_blocks(N)), dim3(BLOCK), 0, st, X, (long long)N, d,
                               vec_ok, S, R, (u64)seed, w.keys, w.deg, w.active[0], &w.ctr[0].n_active);
        HIPCHK(hipGetLastError());
        HIPCHK(hipEventRecord(ev[e++], st));
        for (int t1 = 0; t1 < T1; ++t1) {
            for (int t2 = 0; t2 < T2; ++t2, ++t) {
                HIPCHK(launch_update_round(w, X, d, dtype, vec_ok, R, w.keys, w.deg, t, st, ev[e]));
                ++e;
                HIPCHK(hipEventRecord(ev[e++], st));
            }
            if (t1 != T1 - 1) {
                HIPCHK(launch_reverse(w, N, R, w.keys, w.deg, t, st));
                HIPCHK(hipEventRecord(ev[e++], st));
            }
        }
        hipLaunchKernelGGL(k_export, dim3((unsigned)(((size_t)N * R + 255) / 256)), dim3(256), 0, st, (long long)N, R,
                           w.keys, w.deg, graph_out, degree_out);
        HIPCHK(hipGetLastError());
        if (keys_out)
            HIPCHK(hipMemcpyAsync(keys_out, w.keys, (size_t)N * R * 8, hipMemcpyDeviceToDevice, st));
        HIPCHK(hipEventRecord(ev[e++], st));
        HIPCHK(hipMemcpyAsync(hctr, w.ctr, (size_t)n_ctr * sizeof(RoundCtr), hipMemcpyDeviceToHost, st));
        HIPCHK(hipStreamSynchronize(st));
        if (stats) {
            memset(stats, 0, sizeof *stats);
            fill_round_stats(stats, hctr, rounds);
            stats->reverse_calls = T1 - 1;
            stats->init_evals = (int64_t)N * S;
            float ms = 0;
            (void)hipEventElapsedTime(&ms, ev[0], ev[1]); stats->init_ms = ms;
            int q = 1, tt = 0;   // ev[q] = end of the previous phase
            for (int t1 = 0; t1 < T1; ++t1) {
                for (int t2 = 0; t2 < T2; ++t2, ++tt, q += 2) {
                    if (tt >= RNND_MAX_ROUNDS) continue;
                    (void)hipEventElapsedTime(&ms, ev[q], ev[q + 1]); stats->scan_ms[tt] = ms;
                    (void)hipEventElapsedTime(&ms, ev[q], ev[q + 2]); stats->round_ms[tt] = ms;
                }
                if (t1 != T1 - 1) {
                    (void)hipEventElapsedTime(&ms, ev[q], ev[q + 1]);
                    if (t1 < RNND_MAX_ROUNDS) stats->reverse_ms[t1] = ms;
                    ++q;
                }
            }
            (void)hipEventElapsedTime(&ms, ev[0], ev[e - 1]); stats->total_ms = ms;
        }
    }
done:
    for (int i = 0; i < n_ev_made; ++i) (void)hipEventDestroy(ev[i]);
    free(ev);
    free(hctr);
    if (w.base) (void)hipFree(w.base);
    return rc;
}

extern "C" int rnnd_build(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S, int32_t R,
                          int32_t T1, int32_t T2, uint64_t seed, int32_t *graph_out, int32_t *degree_out,
                          void *stream)
{
    return rnnd_build_ex(X, N, d, dtype, metric, S, R, T1, T2, seed, graph_out, degree_out, nullptr, nullptr,
                         stream);
}

extern "C" int rnnd_random_graph(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S,
                                 int32_t R, uint64_t seed, uint64_t *keys, int32_t *deg, void *stream)
{
    int rc = check_data_args(X, N, d, dtype, metric, R);
    if (rc) return rc;
    if (!keys || !deg) return RNND_ERR_NULL;
    if (S < 1 || S > R || (int64_t)S > N - 1) return RNND_ERR_BAD_PARAM;
    hipStream_t st = (hipStream_t)stream;
    int *scratch = nullptr;
    const int vec_ok = vec_ok_for(X, d, dtype);
    HIPCHK(hipMalloc((void **)&scratch, (size_t)N * 4));
    if (dtype == RNND_U8)
        hipLaunchKernelGGL(k_random_graph<DT_U8>, dim3(vertex_blocks(N)), dim3(BLOCK), 0, st, X, (long long)N, d, vec_ok,
                           S, R, (u64)seed, (u64 *)keys, deg, scratch, (u32 *)nullptr);
    else
        hipLaunchKernelGGL(k_random_graph<DT_F32>, dim3(vertex_blocks(N)), dim3(BLOCK), 0, st, X, (long long)N, d, vec_ok,
                           S, R, (u64)seed, (u64 *)keys, deg, scratch, (u32 *)nullptr);
    HIPCHK(hipGetLastError());
    HIPCHK(hipStreamSynchronize(st));
done:
    if (scratch) (void)hipFree(scratch);
    return rc;
}

extern "C" int rnnd_update_neighbors(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t R,
                                     uint64_t *keys, int32_t *deg, int32_t n_rounds, rnnd_stats *stats,
                                     void *stream)
{
    int rc = check_data_args(X, N, d, dtype, metric, R);
    if (rc) return rc;
    if (!keys || !deg) return RNND_ERR_NULL;
    if (n_rounds < 1 || n_rounds > 1000000) return RNND_ERR_BAD_PARAM;
    hipStream_t st = (hipStream_t)stream;
    const int n_ctr = n_rounds + 2, vec_ok = vec_ok_for(X, d, dtype);
    Workspace w;
    RoundCtr *hctr = (RoundCtr *)calloc(n_ctr, sizeof(RoundCtr));
    if (!hctr) return RNND_ERR_OOM;
    w.bytes = ws_layout(w, N, R, n_ctr, false);
    HIPCHK(hipMalloc((void **)&w.base, w.bytes));
    ws_layout(w, N, R, n_ctr, false);
    HIPCHK(hipMemsetAsync(w.ctr, 0, (size_t)n_ctr * sizeof(RoundCtr), st));
    HIPCHK(hipMemsetAsync(w.cnt, 0, (size_t)N * 4, st));
    hipLaunchKernelGGL(k_collect_active, dim3(vertex_blocks(N)), dim3(BLOCK), 0, st, (long long)N, R,
                       (const u64 *)keys, deg, w.ctr, w.active[0]);
    HIPCHK(hipGetLastError());
    for (int t = 0; t < n_rounds; ++t)
        HIPCHK(launch_update_round(w, X, d, dtype, vec_ok, R, (u64 *)keys, deg, t, st));
    HIPCHK(hipMemcpyAsync(hctr, w.ctr, (size_t)n_ctr * sizeof(RoundCtr), hipMemcpyDeviceToHost, st));
    HIPCHK(hipStreamSynchronize(st));
    if (stats) {
        memset(stats, 0, sizeof *stats);
        fill_round_stats(stats, hctr, n_rounds);
    }
done:
    free(hctr);
    if (w.base) (void)hipFree(w.base);
    return rc;
}

extern "C" int rnnd_add_reverse_edges(int64_t N, int32_t R, uint64_t *keys, int32_t *deg, void *stream)
{
    int rc = RNND_OK;
    if (!keys || !deg) return RNND_ERR_NULL;
    if (N < 2 || N > 2147483646LL) return RNND_ERR_BAD_SHAPE;
    if (R < 1 || R > RNND_MAX_R) return RNND_ERR_BAD_PARAM;
    hipStream_t st = (hipStream_t)stream;
    Workspace w;
    w.bytes = ws_layout(w, N, R, 2, false);
    HIPCHK(hipMalloc((void **)&w.base, w.bytes));
    ws_layout(w, N, R, 2, false);
    HIPCHK(hipMemsetAsync(w.ctr, 0, 2 * sizeof(RoundCtr), st));
    HIPCHK(hipMemsetAsync(w.cnt, 0, (size_t)N * 4, st));
    HIPCHK(launch_reverse(w, N, R, (u64 *)keys, deg, 0, st));
    HIPCHK(hipStreamSynchronize(st));
done:
    if (w.base) (void)hipFree(w.base);
    return rc;
}

extern "C" int rnnd_export_graph(int64_t N, int32_t R, const uint64_t *keys, const int32_t *deg,
                                 int32_t *graph_out, int32_t *degree_out, void *stream)
{
    int rc = RNND_OK;
    if (!keys || !deg || !graph_out || !degree_out) return RNND_ERR_NULL;
    if (N < 1 || N > 2147483646LL) return RNND_ERR_BAD_SHAPE;
    if (R < 1 || R > RNND_MAX_R) return RNND_ERR_BAD_PARAM;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(k_export, dim3((unsigned)(((size_t)N * R + 255) / 256)), dim3(256), 0, st, (long long)N, R,
                       (const u64 *)keys, deg, graph_out, degree_out);
    HIPCHK(hipGetLastError());
    HIPCHK(hipStreamSynchronize(st));
done:
    return rc;
}

extern "C" int rnnd_set_kernel_variant(int variant)
{
    if (variant < 0 || variant > 2) return RNND_ERR_BAD_PARAM;
    g_kernel_variant = variant;
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
    case RNND_ERR_HIP: return g_last_hip_error[0] ? g_last_hip_error : "HIP error";
    default: return "unknown status";
    }
}

extern "C" int rnnd_version(void) { return 100; }
