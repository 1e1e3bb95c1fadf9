// UpdateNeighbors scan (Alg. 4, the body of the vertex loop) for uint8 rows on the matrix cores.
//
// One wavefront owns one vertex u with m <= 32*NG list entries.  The rows x_v of its whole list are
// gathered straight into MFMA operand registers (lane l: row l%32 of a 32-row group, bytes
// [32s + 16(l/32), +16) of K-step s) from a copy of X made once per build in which every byte is
// the int8 x-128 (this leaves every difference, hence every delta, unchanged).  n_v = |x_v - 128|^2
// is read off the diagonal of the Gram tile of v's block with itself.
// For a block I of 32 list positions (rows v_i) and a block J <= I (candidates w_j) the tile
//     T_ij = 2 <x_i, x_j> - n_j - t_i ,   t_i = n_i - delta(u, v_i)
// is formed from the Gram tile G(I, J) of v_mfma_i32_32x32x32_i8 (for J = I the one that gave the norms) by
// one shift-add per entry.  The first operand is block J, the second block I, so a lane holds ROW i = l%32 of the tile
// and 16 of its columns, j = 8(a/4) + 4(l/32) + a%4: by the symmetry of the Gram matrix no transpose
// is needed.  Both operands use the same byte order, so however the hardware pairs the K bytes, the
// two sides pair alike.  With delta(v_i, w_j) = n_i + n_j - 2<x_i, x_j> (exact in int32):
//     the prune test fires  <=>  delta(u, v_i) >= delta(v_i, w_j)  <=>  T_ij >= 0 ,
// Each half-wave collects the outcomes for its 16 columns as bits of one word per row.  The loop over v
// then run on bit masks: the kept set U' is the unique solution K of
//     K_i = not exists j < i : F_ij and K_j
// (F already masked by the old/old skip), found per 32-row block by iterating
// K <- Phi(K) from "all kept" until it stops changing (row i is final after i+1 sweeps).  A pruned
// row's redirect target is the first set bit of F_i & K, and delta(v,w) for the new edge comes from
// the tile kept in LDS:  delta(v_i, w_j) = delta(u, v_i) - T_ij.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wave_prims.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define GT_STRIDE 36   // dwords per row of a tile in LDS (32 + 4: conflict-free b128 stores)

template <int NG>
struct alignas(16) MfmaScanSmem {
    int gt[NG * 32 * GT_STRIDE];   // tiles T(I, J) of the current block I: [(32J + i) * GT_STRIDE + j]
    int nrm[32 * NG];              // n_j by list position
    int id[32 * NG];               // vertex id by list position
};

// What the scan holds in registers for one vertex of its work list before it is that vertex's turn.
struct ScanItem {
    int u;          // vertex, -1 past the end of the list
    int m;          // its degree
    u64 k[2];       // its list: positions lane and lane + 64
};

template <int NG>
__device__ __forceinline__ ScanItem scan_item_load(int u, const u64 *__restrict__ keys,
                                                   const int *__restrict__ deg, int R, int lane)
{
    // the list is read without waiting for the degree: slots past it exist (rows are R wide) and are masked later
    // past the end of the work list (u < 0) vertex 0 is read instead and given degree 0: loads without branches
    ScanItem it;
    const u64 *row = keys + (size_t)(u >= 0 ? u : 0) * R;
    const int m = deg[u >= 0 ? u : 0];
    it.u = u;
    it.m = u >= 0 ? m : 0;
    it.k[0] = row[lane < R ? lane : R - 1];                                  // positions past the degree are masked later
    it.k[1] = NG > 2 ? row[lane + 64 < R ? lane + 64 : R - 1] : KEY_PAD;
    return it;
}

// Issues the loads of one vertex's rows of X into MFMA operand layout (no arithmetic on them yet).
template <int NG, int KS>
__device__ __forceinline__ void scan_gather(const int8_t *__restrict__ X, const ScanItem &it, int l32,
                                            int half, v4i (&A)[NG][KS])
{
    constexpr int d = KS * 32;
    const int m = it.m < 32 * NG ? it.m : 32 * NG;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const u32 idr = key_id(it.k[g >> 1]);
        const int id = __shfl((int)idr, 32 * (g & 1) + l32);
        // a lane without a list entry reads row 0 of X (every load unconditional: no registers to clear, no
        // branch); what such a row contributes is never selected by a mask
        const bool valid = it.u >= 0 && 32 * g + l32 < m;
        const int8_t *p = X + (size_t)(valid ? id : 0) * d + half * 16;
#pragma unroll
        for (int s = 0; s < KS; ++s) A[g][s] = *(const v4i *)(p + s * 32);
    }
}

// Once per build: Xs <- X - 128 as int8 (n bytes, a multiple of 16).
__global__ __launch_bounds__(256) void k_prepare_u8(const uint8_t *__restrict__ X, size_t n,
                                                    int8_t *__restrict__ Xs)
{
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 16;
    if (i < n) {
        v4i x = *(const v4i *)(X + i);
        x ^= (int)0x80808080;
        *(v4i *)(Xs + i) = x;
    }
}

// What a trip has in flight for the trips after it: the rows of the next vertex (or group) and the
// list of the one after.  The memory counter of a wavefront is in order and counts stores as well, so a
// wait for these loads that stood after the trip's stores would also wait for the stores to be
// acknowledged; naming the registers as inputs of an empty statement just before the stores puts the
// wait there, where the loads are a whole trip old and the stores are not yet issued.
__device__ __forceinline__ void arrived(const v4i &x) { asm volatile("" ::"v"(x)); }
__device__ __forceinline__ void arrived(u64 x) { asm volatile("" ::"v"(x)); }
__device__ __forceinline__ void arrived(int x) { asm volatile("" ::"v"(x)); }

// The body of Alg. 4's vertex loop for the vertex in `cur`, whose rows are in A and whose norms are in nr.
template <int NG, int KS>
__device__ __forceinline__ void scan_vertex_u8(const ScanItem &cur, v4i (&A)[NG][KS], MfmaScanSmem<NG> &sm, int R, u64 *__restrict__ keys,
                                               int *__restrict__ deg, Prop *__restrict__ props,
                                               int *__restrict__ nprop, int lane, u64 &tiles, u64 &rows,
                                               u64 &nprops_total, u32 &ev_lane, const v4i (&An)[NG][KS],
                                               const ScanItem &aft, int u_after)
{
    const int l32 = lane & 31, half = lane >> 5;
    const int u = __builtin_amdgcn_readfirstlane(cur.u);      // same in every lane: keep it scalar
    int m = __builtin_amdgcn_readfirstlane(cur.m);
    if (m > 32 * NG) m = 32 * NG;   // cannot happen: the list is built per degree class
    if (m > R) m = R;
    u64 *row = keys + (size_t)u * R;
    u64 kreg[2];
    kreg[0] = lane < m ? cur.k[0] : KEY_PAD;
    kreg[1] = (NG > 2 && lane + 64 < m) ? cur.k[1] : KEY_PAD;
    u64 newm[2];
    newm[0] = __builtin_amdgcn_ballot_w64(lane < m && (kreg[0] & 1ull));
    newm[1] = __builtin_amdgcn_ballot_w64(NG > 2 && lane + 64 < m && (kreg[1] & 1ull));
    const bool any_new = (newm[0] | newm[1]) != 0;   // else every pair was tested before
    // what the scan leaves to be stored: per block one redirected edge per lane, and the kept set
    u64 ekey[NG];
    u32 etgt[NG];
    int eslot[NG];
    u32 Kw[NG];                             // U' as bit masks over list positions, 32 per word (uniform)
#pragma unroll
    for (int I = 0; I < NG; ++I) eslot[I] = -1, Kw[I] = 0, ekey[I] = 0, etgt[I] = 0;
    int np_base = 0;
    if (any_new) {
    wave_sync();   // the previous vertex is done with the LDS tables
    if (lane < 32 * NG) sm.id[lane] = (int)key_id(kreg[0]);
    if (NG > 2 && lane + 64 < 32 * NG) sm.id[64 + lane] = (int)key_id(kreg[1]);
    rows += m;
    const u32 hm = 0x0F0F0F0Fu << (4 * half);   // the columns this half-wave holds

#pragma unroll
    for (int I = 0; I < NG; ++I) {
        if (32 * I < m) {                   // wave-uniform
            // the Gram tile of the block with itself; n of its rows is the diagonal, read back through
            // LDS (rows past the list hold row 0 of X; no mask ever selects them)
            v16i G = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < KS; ++s) G = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[I][s], A[I][s], G, 0, 0, 0);
            {
                int4 *gt = (int4 *)(sm.gt + (32 * I + l32) * GT_STRIDE + 4 * half);
                gt[0] = make_int4(G[0], G[1], G[2], G[3]);
                gt[2] = make_int4(G[4], G[5], G[6], G[7]);
                gt[4] = make_int4(G[8], G[9], G[10], G[11]);
                gt[6] = make_int4(G[12], G[13], G[14], G[15]);
            }
            wave_sync();
            const int nrI = sm.gt[(32 * I + l32) * GT_STRIDE + l32];
            if (half == 0) sm.nrm[32 * I + l32] = nrI;
            wave_sync();
            // this block's rows in lane-per-row form (lane l32 <-> list position 32 I + l32), in both halves
            const u64 kb = shfl_u64(kreg[I >> 1], 32 * (I & 1) + l32);
            const int posi = 32 * I + l32;
            const bool validi = posi < m;
            const bool newi = kb & 1ull;
            const int di = (int)key_dist(kb);
            const int negt = di - nrI;
            const u32 new_I = (u32)(newm[I >> 1] >> (32 * (I & 1)));
            u32 F[NG], E[NG];
#pragma unroll
            for (int J = 0; J < NG; ++J) F[J] = E[J] = 0;
#pragma unroll
            for (int J = 0; J <= I; ++J) {
                // a tile without a new row and without a new column holds only old/old pairs, which Alg. 4 skips
                const u32 new_J = (u32)(newm[J >> 1] >> (32 * (J & 1)));
                if ((new_I | new_J) == 0) continue;
                tiles += 1;
                // the old/old skip: a pair is tested only if v or w is new; only w before v count
                u32 e = newi ? 0xFFFFFFFFu : new_J;
                if (J == I) e &= (1u << l32) - 1u;
                if (!validi) e = 0;
                E[J] = e & hm;
                // lane: row l32 of block I; acc[a]: column 8(a/4) + 4 half + a%4 of block J
                v16i acc = G;
                if (J < I) {
                    acc = (v16i){0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                    for (int s = 0; s < KS; ++s)
                        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[J][s], A[I][s], acc, 0, 0, 0);
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int4 nj = ((const int4 *)sm.nrm)[8 * J + 2 * q + half];
                    acc[4 * q + 0] = (acc[4 * q + 0] << 1) + (negt - nj.x);
                    acc[4 * q + 1] = (acc[4 * q + 1] << 1) + (negt - nj.y);
                    acc[4 * q + 2] = (acc[4 * q + 2] << 1) + (negt - nj.z);
                    acc[4 * q + 3] = (acc[4 * q + 3] << 1) + (negt - nj.w);
                }
                int4 *gt = (int4 *)(sm.gt + (32 * J + l32) * GT_STRIDE + 4 * half);
                gt[0] = make_int4(acc[0], acc[1], acc[2], acc[3]);
                gt[2] = make_int4(acc[4], acc[5], acc[6], acc[7]);
                gt[4] = make_int4(acc[8], acc[9], acc[10], acc[11]);
                gt[6] = make_int4(acc[12], acc[13], acc[14], acc[15]);
                // bit a of ok: T < 0, v passes the prune test against column a
                u32 ok = 0;
#pragma unroll
                for (int a = 15; a >= 0; --a) ok = __builtin_amdgcn_alignbit(ok, (u32)acc[a], 31);
                // bit 4q + k  ->  column 8q + 4 half + k
                ok = (ok | (ok << 8)) & 0x00FF00FFu;
                ok = (ok | (ok << 4)) & 0x0F0F0F0Fu;
                ok <<= 4 * half;
                F[J] = E[J] & ~ok;
            }
            // the loop over v on masks; what the two half-waves find for a row is joined through ballots
            bool pre = false;
#pragma unroll
            for (int J = 0; J < I; ++J) pre = pre || ((F[J] & Kw[J]) != 0);
            const u64 preb = __builtin_amdgcn_ballot_w64(pre);
            const u32 rem = (u32)(m - 32 * I);
            const u32 vmask = rem >= 32u ? 0xFFFFFFFFu : ((1u << rem) - 1u);
            const u32 Kmax = vmask & ~((u32)preb | (u32)(preb >> 32));
            u32 Kcur = Kmax;
            for (int sweep = 0; sweep < 33; ++sweep) {
                const u64 hit = __builtin_amdgcn_ballot_w64((F[I] & Kcur) != 0);
                const u32 Knew = Kmax & ~((u32)hit | (u32)(hit >> 32));
                if (Knew == Kcur) break;
                Kcur = Knew;
            }
            Kw[I] = Kcur;
            const bool kept = (Kcur >> l32) & 1u;
            const bool pruned = validi && !kept && half == 0;
            // first failing w over both halves
            int tgt = 0x7FFFFFFF;
#pragma unroll
            for (int J = I; J >= 0; --J) {
                const u32 fk = F[J] & Kw[J];
                if (fk) tgt = 32 * J + __builtin_ctz(fk);
            }
            {
                const int other = __shfl_xor(tgt, 32);
                tgt = other < tgt ? other : tgt;
            }
            // the evaluations Alg. 4 makes for this row: tested candidates up to and including w
            int ev = 0;
#pragma unroll
            for (int J = 0; J <= I; ++J) {
                const int rel = tgt - 32 * J;
                const u32 upto = rel >= 31 ? 0xFFFFFFFFu : (rel < 0 ? 0u : ((2u << rel) - 1u));
                ev += __popc(E[J] & Kw[J] & upto);
            }
            ev_lane += (u32)ev;
            wave_sync();   // the tiles are in LDS
            const u64 pm = __builtin_amdgcn_ballot_w64(pruned);
            if (pruned) {
                const int tv = sm.gt[((tgt & ~31) + l32) * GT_STRIDE + (tgt & 31)];
                const u32 dvw = (u32)(di - tv);
                // the redirect: v enters w's list
                ekey[I] = make_key(dvw, key_id(kb), 1u);
                etgt[I] = (u32)sm.id[tgt];
                eslot[I] = np_base + __popcll(pm & lanes_below(lane));
            }
            np_base += __popcll(pm);
            if (I + 1 < NG) wave_sync();   // before the next block overwrites the tiles
        }
    }
    }
    // every store of the trip comes after this point
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int s = 0; s < KS; ++s) arrived(An[g][s]);
    arrived(aft.k[0]), arrived(aft.m), arrived(u_after);
    if (NG > 2) arrived(aft.k[1]);
#pragma unroll
    for (int I = 0; I < NG; ++I)
        if (eslot[I] >= 0) emit_redirect(ekey[I], etgt[I], props + (size_t)u * R + eslot[I]);
    // kept entries, flag old, compacted back into the row
    const u64 K0 = (u64)Kw[0] | (NG > 1 ? ((u64)Kw[NG > 1 ? 1 : 0] << 32) : 0ull);
    const u64 K1 = NG > 2 ? ((u64)Kw[NG > 2 ? 2 : 0] | (NG > 3 ? ((u64)Kw[NG > 3 ? 3 : 0] << 32) : 0ull)) : 0ull;
    const int nk0 = __popcll(K0);
    if ((K0 >> lane) & 1ull) row[__popcll(K0 & lanes_below(lane))] = kreg[0] & ~1ull;
    if (NG > 2 && ((K1 >> lane) & 1ull)) row[nk0 + __popcll(K1 & lanes_below(lane))] = kreg[1] & ~1ull;
    if (lane == 0) {
        if (any_new) deg[u] = nk0 + __popcll(K1);
        nprop[u] = np_base;
    }
    nprops_total += np_base;
}

// The work list is walked with a two-deep software pipeline: while vertex i is computed, the rows of
// vertex i+1 are already in flight and the list of vertex i+2 is being fetched, so that the chain
// list -> degree/list entries -> rows of X is paid once per wavefront, not once per vertex.  The loop
// body is written out twice so that the two row buffers swap roles without being copied.
// block `block` of `nblocks` walks the work list
template <int NG, int KS>
__device__ __forceinline__ void scan_list_body(const int8_t *__restrict__ X, int R, u64 *__restrict__ keys,
                                               int *__restrict__ deg, const int *__restrict__ list, u32 n_active,
                                               Prop *__restrict__ props, int *__restrict__ nprop,
                                               RoundCtr *__restrict__ ctr, MfmaScanSmem<NG> &sm, u32 block, u32 nblocks)
{
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: the loop control stays on the scalar unit
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    const u32 gw = block * 4 + wave, nw = nblocks * 4;
    u64 tiles = 0, rows = 0, nprops_total = 0;   // tiles: 32x32 blocks of pair distances computed
    u32 ev_lane = 0;   // per-lane share of the algorithmic evaluation count, summed at the end

    if (gw >= n_active) return;
    ScanItem cur = scan_item_load<NG>(list[gw], keys, deg, R, lane);
    ScanItem nxt = scan_item_load<NG>(gw + nw < n_active ? list[gw + nw] : -1, keys, deg, R, lane);
    int u_after = gw + 2 * nw < n_active ? list[gw + 2 * nw] : -1;
    v4i A0[NG][KS], A1[NG][KS];
    scan_gather<NG, KS>(X, cur, l32, half, A0);
    // once per wavefront: the loop starts with nothing in flight
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int s = 0; s < KS; ++s) arrived(A0[g][s]);
    arrived(nxt.k[0]), arrived(nxt.k[1]), arrived(nxt.m), arrived(u_after);

    u32 it = gw;
    while (true) {
        // ---- even trip: `cur` lives in A0, the next vertex is fetched into A1
        scan_gather<NG, KS>(X, nxt, l32, half, A1);
        ScanItem aft = scan_item_load<NG>(u_after, keys, deg, R, lane);
        {
            const unsigned long long j = (unsigned long long)it + 3ull * nw;
            u_after = j < n_active ? list[j] : -1;
        }
        scan_vertex_u8<NG, KS>(cur, A0, sm, R, keys, deg, props, nprop, lane, tiles, rows, nprops_total,
                               ev_lane, A1, aft, u_after);
        cur = nxt;
        nxt = aft;
        if ((unsigned long long)it + nw >= n_active) break;
        it += nw;
        // ---- odd trip: roles of the two buffers exchanged
        scan_gather<NG, KS>(X, nxt, l32, half, A0);
        aft = scan_item_load<NG>(u_after, keys, deg, R, lane);
        {
            const unsigned long long j = (unsigned long long)it + 3ull * nw;
            u_after = j < n_active ? list[j] : -1;
        }
        scan_vertex_u8<NG, KS>(cur, A1, sm, R, keys, deg, props, nprop, lane, tiles, rows, nprops_total,
                               ev_lane, A0, aft, u_after);
        cur = nxt;
        nxt = aft;
        if ((unsigned long long)it + nw >= n_active) break;
        it += nw;
    }
    u64 evals_algo = ev_lane;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) evals_algo += shfl_xor_u64(evals_algo, o);
    if (lane == 0 && rows) add_round_stats(ctr, evals_algo, tiles * 1024ull, rows, nprops_total);
}

template <int NG, int KS>
__global__ __launch_bounds__(256, (NG == 1 ? 5 : NG == 2 ? 3 : 2)) void k_update_scan_mfma_u8(
    const int8_t *__restrict__ X, int R, u64 *__restrict__ keys,
    int *__restrict__ deg, const int *__restrict__ list, const u32 *__restrict__ n_list,
    Prop *__restrict__ props, int *__restrict__ nprop, RoundCtr *__restrict__ ctr)
{
    __shared__ MfmaScanSmem<NG> smem[4];
    scan_list_body<NG, KS>(X, R, keys, deg, list, *n_list, props, nprop, ctr, smem[threadIdx.x >> 6], blockIdx.x, gridDim.x);
}

// ---------------------------------------------------------------------------------------------
// Lists of at most 32 entries: P = 1, 2 or 4 vertices share a wavefront, each owning W = 32/P of
// the 32 rows of one tile (rows [W p, W p + W) belong to the p-th vertex of the group).  The Gram tile
// then holds P independent diagonal blocks; the masks keep every row inside its own block, so the
// fixed-point sweeps of all P vertices run together on one 32-bit word.  Every lane (both
// half-waves) holds the list entry of its row.
struct PackItem {
    int u;          // vertex of this lane's segment, -1 past the end of the list
    int m;          // its degree
    u64 k;          // the list entry at this lane's position (KEY_PAD past R)
};

template <int P>
__device__ __forceinline__ PackItem pack_item_load(int u, const u64 *__restrict__ keys,
                                                   const int *__restrict__ deg, int R, int pos)
{
    // past the end of the work list (u < 0) vertex 0 is read instead and given degree 0: loads without branches
    PackItem it;
    const int m = deg[u >= 0 ? u : 0];
    it.u = u;
    it.m = u >= 0 ? m : 0;
    it.k = keys[(size_t)(u >= 0 ? u : 0) * R + (pos < R ? pos : R - 1)];   // slots past the degree exist and are masked later
    return it;
}

template <int P, int KS>
__device__ __forceinline__ void pack_gather(const int8_t *__restrict__ X, const PackItem &it, int pos,
                                            int half, v4i (&A)[KS])
{
    constexpr int d = KS * 32, W = 32 / P;
    // a lane without a list entry reads row 0 of X (see scan_gather)
    const bool valid = it.u >= 0 && pos < (it.m < W ? it.m : W);
    const int8_t *p = X + (size_t)(valid ? key_id(it.k) : 0u) * d + half * 16;
#pragma unroll
    for (int s = 0; s < KS; ++s) A[s] = *(const v4i *)(p + s * 32);
}

template <int P, int KS>
__device__ __forceinline__ void pack_vertices_u8(const PackItem &cur, v4i (&A)[KS], MfmaScanSmem<1> &sm, int R,
                                                 u64 *__restrict__ keys, int *__restrict__ deg,
                                                 Prop *__restrict__ props, int *__restrict__ nprop, int lane,
                                                 u32 &tiles, u32 &rows, u32 &nprops_total, u32 &ev_lane,
                                                 const v4i (&An)[KS], const PackItem &aft, int u_after)
{
    constexpr int W = 32 / P;
    const int l32 = lane & 31, half = lane >> 5, seg = l32 / W, pos = l32 % W;
    const int u = cur.u;
    int m = cur.m;
    if (m > W) m = W;   // cannot happen: the list is built per degree class
    if (m > R) m = R;
    const bool valid = u >= 0 && pos < m;
    const u64 kb = valid ? cur.k : KEY_PAD;
    const bool newi = valid && (kb & 1ull);
    const bool leader = u >= 0 && pos == 0 && half == 0;
    const u32 new32 = (u32)__builtin_amdgcn_ballot_w64(newi && half == 0);
    const bool any_new = new32 != 0;   // else nothing is new in any of the P lists: every pair was tested before
    const u32 segmask = (W == 32 ? 0xFFFFFFFFu : ((1u << (W & 31)) - 1u) << (seg * W));
    const u32 below = (1u << l32) - 1u;
    // what the scan leaves to be stored
    bool pruned = false, kept = false;
    u32 Kcur = 0, pm = 0, dvw = 0, tgt_id = 0;
    if (any_new) {
        const u32 vmask = (u32)__builtin_amdgcn_ballot_w64(valid && half == 0);
        wave_sync();   // the previous group is done with the LDS tables
        if (half == 0) sm.id[l32] = (int)key_id(kb);
        // n of every row: the diagonal of the Gram tile, through LDS (rows past a list hold row 0 of X;
        // no mask ever selects them)
        // lane: row l32; G[a]: <x_row, x_col> for column 8(a/4) + 4 half + a%4
        v16i G = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < KS; ++s) G = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[s], A[s], G, 0, 0, 0);
        {
            int4 *gt = (int4 *)(sm.gt + l32 * GT_STRIDE + 4 * half);
            gt[0] = make_int4(G[0], G[1], G[2], G[3]);
            gt[2] = make_int4(G[4], G[5], G[6], G[7]);
            gt[4] = make_int4(G[8], G[9], G[10], G[11]);
            gt[6] = make_int4(G[12], G[13], G[14], G[15]);
        }
        wave_sync();
        const int ni = sm.gt[l32 * GT_STRIDE + l32];
        if (half == 0) sm.nrm[l32] = ni;
        rows += __popc(vmask);
        tiles += 1;
        wave_sync();

        const int di = (int)key_dist(kb);
        const int negt = di - ni;
        const u32 hm = 0x0F0F0F0Fu << (4 * half);   // the columns this half-wave holds
        // the old/old skip: a pair is tested only if v or w is new; only w before v (in v's own list) count
        u32 E = newi ? segmask : (new32 & segmask);
        E &= below;
        if (!valid) E = 0;
        E &= hm;
        // T = 2 G - n_j - t_i from the Gram tile that gave the norms
        v16i acc;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int4 nj = ((const int4 *)sm.nrm)[2 * q + half];
            acc[4 * q + 0] = (G[4 * q + 0] << 1) + (negt - nj.x);
            acc[4 * q + 1] = (G[4 * q + 1] << 1) + (negt - nj.y);
            acc[4 * q + 2] = (G[4 * q + 2] << 1) + (negt - nj.z);
            acc[4 * q + 3] = (G[4 * q + 3] << 1) + (negt - nj.w);
        }
        {
            int4 *gt = (int4 *)(sm.gt + l32 * GT_STRIDE + 4 * half);
            gt[0] = make_int4(acc[0], acc[1], acc[2], acc[3]);
            gt[2] = make_int4(acc[4], acc[5], acc[6], acc[7]);
            gt[4] = make_int4(acc[8], acc[9], acc[10], acc[11]);
            gt[6] = make_int4(acc[12], acc[13], acc[14], acc[15]);
        }
        // bit a of ok: T < 0, v passes the prune test against column a
        u32 ok = 0;
#pragma unroll
        for (int a = 15; a >= 0; --a) ok = __builtin_amdgcn_alignbit(ok, (u32)acc[a], 31);
        // bit 4q + k  ->  column 8q + 4 half + k
        ok = (ok | (ok << 8)) & 0x00FF00FFu;
        ok = (ok | (ok << 4)) & 0x0F0F0F0Fu;
        ok <<= 4 * half;
        const u32 F = E & ~ok;
        // the loop over v on masks; what the two half-waves find for a row is joined through ballots
        Kcur = vmask;
        for (int sweep = 0; sweep < 33; ++sweep) {
            const u64 hit = __builtin_amdgcn_ballot_w64((F & Kcur) != 0);
            const u32 Knew = vmask & ~((u32)hit | (u32)(hit >> 32));
            if (Knew == Kcur) break;
            Kcur = Knew;
        }
        kept = (Kcur >> l32) & 1u;
        pruned = valid && !kept && half == 0;
        // first failing w over both halves
        int tgt = 0x7FFFFFFF;
        {
            const u32 fk = F & Kcur;
            if (fk) tgt = __builtin_ctz(fk);
            const int other = __shfl_xor(tgt, 32);
            tgt = other < tgt ? other : tgt;
        }
        // the evaluations Alg. 4 makes for this row: tested candidates up to and including w
        {
            const u32 upto = tgt >= 31 ? 0xFFFFFFFFu : ((2u << tgt) - 1u);
            ev_lane += (u32)__popc(E & Kcur & upto);
        }
        wave_sync();   // the tile is in LDS
        pm = (u32)__builtin_amdgcn_ballot_w64(pruned);
        if (pruned) {
            dvw = (u32)(di - sm.gt[l32 * GT_STRIDE + tgt]);
            tgt_id = (u32)sm.id[tgt];
        }
        nprops_total += __popc(pm);
    }
    // every store of the trip comes after this point
#pragma unroll
    for (int s = 0; s < KS; ++s) arrived(An[s]);
    arrived(aft.k), arrived(aft.m), arrived(u_after);
    // the redirect: v enters w's list
    if (pruned) emit_redirect(make_key(dvw, key_id(kb), 1u), tgt_id, props + (size_t)u * R + __popc(pm & segmask & below));
    // kept entries, flag old, compacted back into the row
    if (kept && half == 0) keys[(size_t)u * R + __popc(Kcur & segmask & below)] = kb & ~1ull;
    if (leader) {
        if (any_new) deg[u] = __popc(Kcur & segmask);
        nprop[u] = __popc(pm & segmask);
    }
}

// Same two-deep software pipeline as k_update_scan_mfma_u8; trip g of a wavefront takes list entries
// [P g, P g + P).
template <int P, int KS>
__device__ __forceinline__ void scan_packed_body(const int8_t *__restrict__ X, int R, u64 *__restrict__ keys,
                                                 int *__restrict__ deg, const int *__restrict__ list,
                                                 u32 n_active, Prop *__restrict__ props,
                                                 int *__restrict__ nprop, RoundCtr *__restrict__ ctr,
                                                 MfmaScanSmem<1> &sm, u32 block, u32 nblocks)
{
    constexpr int W = 32 / P;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: the loop control stays on the scalar unit
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    const int seg = l32 / W, pos = l32 % W;
    const u32 gw = block * 4 + wave, nw = nblocks * 4;
    const u32 n_groups = (n_active + (u32)P - 1u) / (u32)P;
    u32 tiles = 0, rows = 0, nprops_total = 0;   // per wavefront: far below 2^32
    u32 ev_lane = 0;

    if (gw >= n_groups) return;
    auto vertex_of = [&](unsigned long long g) -> int {
        const unsigned long long idx = g * P + (unsigned)seg;
        return (g < n_groups && idx < n_active) ? list[idx] : -1;
    };
    PackItem cur = pack_item_load<P>(vertex_of(gw), keys, deg, R, pos);
    PackItem nxt = pack_item_load<P>(vertex_of((unsigned long long)gw + nw), keys, deg, R, pos);
    int u_after = vertex_of((unsigned long long)gw + 2ull * nw);
    v4i A0[KS], A1[KS];
    pack_gather<P, KS>(X, cur, pos, half, A0);
    // once per wavefront: the loop starts with nothing in flight
#pragma unroll
    for (int s = 0; s < KS; ++s) arrived(A0[s]);
    arrived(nxt.k), arrived(nxt.m), arrived(u_after);

    u32 it = gw;
    while (true) {
        // ---- even trip: `cur` lives in A0, the next group is fetched into A1
        pack_gather<P, KS>(X, nxt, pos, half, A1);
        PackItem aft = pack_item_load<P>(u_after, keys, deg, R, pos);
        u_after = vertex_of((unsigned long long)it + 3ull * nw);
        pack_vertices_u8<P, KS>(cur, A0, sm, R, keys, deg, props, nprop, lane, tiles, rows, nprops_total, ev_lane,
                                A1, aft, u_after);
        cur = nxt;
        nxt = aft;
        if ((unsigned long long)it + nw >= n_groups) break;
        it += nw;
        // ---- odd trip: roles of the two buffers exchanged
        pack_gather<P, KS>(X, nxt, pos, half, A0);
        aft = pack_item_load<P>(u_after, keys, deg, R, pos);
        u_after = vertex_of((unsigned long long)it + 3ull * nw);
        pack_vertices_u8<P, KS>(cur, A1, sm, R, keys, deg, props, nprop, lane, tiles, rows, nprops_total, ev_lane,
                                A0, aft, u_after);
        cur = nxt;
        nxt = aft;
        if ((unsigned long long)it + nw >= n_groups) break;
        it += nw;
    }
    u64 evals_algo = ev_lane;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) evals_algo += shfl_xor_u64(evals_algo, o);
    if (lane == 0 && rows) add_round_stats(ctr, evals_algo, (u64)tiles * 1024ull, rows, nprops_total);
}

// The three short-list classes in one launch: blockIdx.y = degree class (lists of at most 8, 16, 32
// entries: 4, 2, 1 vertices per wavefront).  Each class is walked by the gridDim.x blocks of its row.
template <int KS>
__global__ __launch_bounds__(256, 4) void k_update_scan_mfma_u8_small(
    const int8_t *__restrict__ X, int R, u64 *__restrict__ keys, int *__restrict__ deg,
    const int *__restrict__ lists, long long N, Prop *__restrict__ props, int *__restrict__ nprop,
    RoundCtr *__restrict__ ctr)
{
    __shared__ MfmaScanSmem<1> smem[4];
    MfmaScanSmem<1> &sm = smem[threadIdx.x >> 6];
    const int y = blockIdx.y;
    const int *list = lists + (size_t)y * N;
    const u32 n = ctr->n_active[y];
    stamp_scan_start(ctr);
    if (y == 0) scan_packed_body<4, KS>(X, R, keys, deg, list, n, props, nprop, ctr, sm, blockIdx.x, gridDim.x);
    else if (y == 1) scan_packed_body<2, KS>(X, R, keys, deg, list, n, props, nprop, ctr, sm, blockIdx.x, gridDim.x);
    else scan_packed_body<1, KS>(X, R, keys, deg, list, n, props, nprop, ctr, sm, blockIdx.x, gridDim.x);
}

// Classes C0 .. NC - 1 in one launch, all of them resident together: the grid's blocks are divided among the
// classes in proportion to their work (active lists x matrix tiles per list), one block at least for a class
// that has any; every block derives the same division from the round's counters.  The classes then share the
// start-up and the tail that each launch of its own pays.  NC classes: 3 short-list ones, then lists of at
// most 64, 96, 128 entries.  Every block carries the registers and the LDS of the longest class (two blocks
// per CU).  C0 = 0, every class: for inputs so small that no class alone has enough lists to fill the chip
// (the short-list classes lose occupancy: with many active lists their own launch is faster).  C0 = 3, the
// long-list classes only, next to k_update_scan_mfma_u8_small: for large inputs.
template <int KS, int NC, int C0 = 0>
__global__ __launch_bounds__(256, 2) void k_update_scan_mfma_u8_all(
    const int8_t *__restrict__ X, int R, u64 *__restrict__ keys, int *__restrict__ deg,
    const int *__restrict__ lists, long long N, Prop *__restrict__ props, int *__restrict__ nprop,
    RoundCtr *__restrict__ ctr)
{
    constexpr int NGMAX = NC - 2;
    static_assert(NC >= 4 && NC <= 6, "short lists plus one to three long-list classes");
    __shared__ MfmaScanSmem<NGMAX> smem[4];
    if (C0 == 0) stamp_scan_start(ctr);
    // work per list: 4, 2, 1 lists share a tile; among the longer classes in proportion to their NG (NG + 1) / 2
    // tiles (3 : 6 : 10; the division is sensitive there: 3 : 4.5 or 3 : 8 costs the 1M build 4 % of its scan time),
    // and a 64-entry list weighted 2.25 short tiles (measured on 100,000 vertices: 1.5 -> 1.60 ms, 2 -> 1.51, 2.25 ->
    // 1.49, 3 -> 1.53, 4 -> 1.70 ms of scan time per build)
    constexpr u32 weight[6] = {4u, 8u, 16u, 36u, 72u, 120u};
    u32 n[NC];
    u64 total = 0;
    u32 nonempty = 0;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        n[c] = c >= C0 ? ctr->n_active[c] : 0u;
        total += (u64)n[c] * weight[c];
        nonempty += n[c] != 0u;
    }
    if (total == 0) return;
    // A class gets one block plus its share of the rest: the shares are differences of one non-decreasing
    // function of the running sum that ends at `spare` exactly (total / total = 1), so they add up to the grid
    // whatever the rounding of the single-precision quotient; every block computes the same numbers.
    const u32 spare = gridDim.x - nonempty;      // the grid has more blocks than there are classes (and < 2^24)
    const float scale = (float)spare, ftotal = (float)total;
    u32 first = 0, mine = 0, below = 0;
    int cls = -1;
    u64 cum = 0;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        cum += (u64)n[c] * weight[c];
        const u32 upto = (u32)(scale * ((float)cum / ftotal));
        const u32 nb = n[c] ? 1u + upto - below : 0u;
        below = upto;
        if (cls < 0 && blockIdx.x < first + nb) {
            cls = c;
            mine = nb;
        }
        if (cls < 0) first += nb;
    }
    if (cls < 0) return;      // cannot happen: the shares add up to the grid
    const u32 block = blockIdx.x - first;
    const int *list = lists + (size_t)cls * N;
    const int wave = threadIdx.x >> 6;
    MfmaScanSmem<1> &sm1 = *reinterpret_cast<MfmaScanSmem<1> *>(&smem[wave]);
    if (C0 == 0 && cls == 0) scan_packed_body<4, KS>(X, R, keys, deg, list, n[0], props, nprop, ctr, sm1, block, mine);
    else if (C0 == 0 && cls == 1) scan_packed_body<2, KS>(X, R, keys, deg, list, n[1], props, nprop, ctr, sm1, block, mine);
    else if (C0 == 0 && cls == 2) scan_packed_body<1, KS>(X, R, keys, deg, list, n[2], props, nprop, ctr, sm1, block, mine);
    else if (cls == 3)
        scan_list_body<2, KS>(X, R, keys, deg, list, n[3], props, nprop, ctr, *reinterpret_cast<MfmaScanSmem<2> *>(&smem[wave]), block, mine);
    else if (NC > 4 && cls == 4)
        scan_list_body<3, KS>(X, R, keys, deg, list, n[NC > 4 ? 4 : 0], props, nprop, ctr, *reinterpret_cast<MfmaScanSmem<3> *>(&smem[wave]), block, mine);
    else if (NC > 5 && cls == 5)
        scan_list_body<4, KS>(X, R, keys, deg, list, n[NC > 5 ? 5 : 0], props, nprop, ctr, *reinterpret_cast<MfmaScanSmem<4> *>(&smem[wave]), block, mine);
}
