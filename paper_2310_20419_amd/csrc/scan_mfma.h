// UpdateNeighbors scan (Alg. 4 lines 2-15) for uint8 rows on the matrix cores.
//
// One wavefront owns one vertex u with m <= 32*NG list entries.  The rows x_v of its whole list are
// gathered straight into MFMA operand registers (lane l: row l%32 of a 32-row group, bytes
// [32s + 16(l/32), +16) of K-step s), turned into int8 by x-128 (which leaves every difference, hence
// every delta, unchanged), and the Gram block  G = A A^T  is formed 32x32 tile by tile with
// v_mfma_i32_32x32x32_i8.  The A and B operand of a tile are the same registers, so whatever order the
// hardware pairs the K bytes in, both sides pair them alike.  With n_i = G_ii:
//     delta(v_i, v_j) = n_i + n_j - 2 G_ij                                   (exact in int32)
//     line 11 fails  <=>  delta(u, v_i) >= delta(v_i, v_j)  <=>  2 G_ij - n_j >= n_i - delta(u, v_i).
// Every lane collects the outcomes for its column as bits of one word (the matrix "v_i fails against
// v_j", one column per lane), and a 5-step butterfly transposes it to one row per lane.
// Lines 5-18 then run on bit masks: the kept set U' is the unique solution K of
//     K_i = not exists j < i : F_ij and K_j
// (F already masked by the old/old skip of lines 8-9), found per 32-row block by iterating
// K <- Phi(K) from "all kept" until it stops changing (row i is final after i+1 sweeps).  A pruned
// row's redirect target is the first set bit of F_i & K, and delta(v,w) for the new edge comes from
// the G tile kept in LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wave_prims.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define GT_STRIDE 36   // dwords per column of the transposed G tile in LDS (32 + 4: conflict-free b128 stores)

template <int NG>
struct alignas(16) MfmaScanSmem {
    int gt[NG * 32 * GT_STRIDE];   // G^T of the current 32-row block: [(32J + c) * GT_STRIDE + r]
    int t[32];                     // n_i - delta(u, v_i) of the current block
    int nrm[32 * NG];              // n_j by list position
    int id[32 * NG];               // vertex id by list position
};

// One butterfly step of a bit-matrix transpose: lanes l and l^SH exchange the blocks of bits
// whose position differs from the lane in bit SH.  M = positions b with (b & SH) == 0.
template <int SH, u32 M>
__device__ __forceinline__ u32 transpose_step(u32 w, int lane)
{
    const u32 p = (u32)__shfl_xor((int)w, SH);
    const u32 lo = (w & M) | ((p & M) << SH);
    const u32 hi = ((p >> SH) & M) | (w & ~M);
    return (lane & SH) ? hi : lo;
}

// Transposes a 32x32 bit matrix held one word per lane (lane i: word i), within each half-wave.
__device__ __forceinline__ u32 transpose32_bits(u32 w, int lane)
{
    w = transpose_step<16, 0x0000FFFFu>(w, lane);
    w = transpose_step<8, 0x00FF00FFu>(w, lane);
    w = transpose_step<4, 0x0F0F0F0Fu>(w, lane);
    w = transpose_step<2, 0x33333333u>(w, lane);
    w = transpose_step<1, 0x55555555u>(w, lane);
    return w;
}

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
    ScanItem it;
    it.u = u;
    it.m = 0;
    it.k[0] = it.k[1] = KEY_PAD;
    if (u >= 0) {
        const u64 *row = keys + (size_t)u * R;
        it.m = deg[u];
        if (lane < R) it.k[0] = row[lane];
        if (NG > 2 && lane + 64 < R) it.k[1] = row[lane + 64];
    }
    return it;
}

// Issues the loads of one vertex's rows of X into MFMA operand layout (no arithmetic on them yet).
template <int NG, int KS>
__device__ __forceinline__ void scan_gather(const uint8_t *__restrict__ X, const ScanItem &it, int l32,
                                            int half, v4i (&A)[NG][KS])
{
    constexpr int d = KS * 32;
    const int m = it.m < 32 * NG ? it.m : 32 * NG;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const u32 idr = key_id(it.k[g >> 1]);
        const int id = __shfl((int)idr, 32 * (g & 1) + l32);
        const bool valid = it.u >= 0 && 32 * g + l32 < m;
        const uint8_t *p = X + (size_t)id * d + half * 16;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            v4i v = {0, 0, 0, 0};
            if (valid) v = *(const v4i *)(p + s * 32);
            A[g][s] = v;
        }
    }
}

// The work list is walked with a two-deep software pipeline: while vertex i is computed, the rows of
// vertex i+1 are already in flight and the list of vertex i+2 is being fetched, so that the chain
// list -> degree/list entries -> rows of X is paid once per wavefront, not once per vertex.
template <int NG, int KS>
__global__ __launch_bounds__(64 * 4) void k_update_scan_mfma_u8(
    const uint8_t *__restrict__ X, int R, u64 *__restrict__ keys, int *__restrict__ deg,
    const int *__restrict__ list, const u32 *__restrict__ n_list, Prop *__restrict__ props,
    int *__restrict__ nprop, RoundCtr *__restrict__ ctr)
{
    __shared__ MfmaScanSmem<NG> smem[4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    const u32 gw = blockIdx.x * 4 + wave, nw = gridDim.x * 4;
    const u32 n_active = *n_list;
    MfmaScanSmem<NG> &sm = smem[wave];
    u64 tiles = 0, rows = 0, nprops_total = 0;   // tiles: 32x32 blocks of pair distances computed
    u32 ev_lane = 0;   // per-lane share of the algorithmic evaluation count, summed at the end

    if (gw >= n_active) return;
    ScanItem cur = scan_item_load<NG>(list[gw], keys, deg, R, lane);
    ScanItem nxt = scan_item_load<NG>(gw + nw < n_active ? list[gw + nw] : -1, keys, deg, R, lane);
    int u_after = gw + 2 * nw < n_active ? list[gw + 2 * nw] : -1;
    v4i A[NG][KS], An[NG][KS];
    scan_gather<NG, KS>(X, cur, l32, half, A);

    for (u32 it = gw; it < n_active; it += nw) {
        // ---- keep the pipeline full
        scan_gather<NG, KS>(X, nxt, l32, half, An);
        ScanItem aft = scan_item_load<NG>(u_after, keys, deg, R, lane);
        {
            const unsigned long long j = (unsigned long long)it + 3ull * nw;
            u_after = j < n_active ? list[j] : -1;
        }

        // ---- vertex `cur`
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
        if ((newm[0] | newm[1]) == 0) {   // nothing new: every pair was tested before
            if (lane == 0) nprop[u] = 0;
        } else {
            wave_sync();   // the previous vertex is done with the LDS tables
            if (lane < 32 * NG) sm.id[lane] = (int)key_id(kreg[0]);
            if (NG > 2 && lane + 64 < 32 * NG) sm.id[64 + lane] = (int)key_id(kreg[1]);
            rows += m;

            // ---- rows as int8 (x - 128) and their squared norms
            int nrm[NG];
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                const int pos = 32 * g + l32;
                const bool valid = pos < m;
                int acc = 0;
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    v4i v = A[g][s];
                    if (valid) v ^= (int)0x80808080;
                    A[g][s] = v;
                    acc = __builtin_amdgcn_sdot4(v.x, v.x, acc, false);
                    acc = __builtin_amdgcn_sdot4(v.y, v.y, acc, false);
                    acc = __builtin_amdgcn_sdot4(v.z, v.z, acc, false);
                    acc = __builtin_amdgcn_sdot4(v.w, v.w, acc, false);
                }
                acc += __shfl_xor(acc, 32);
                nrm[g] = acc;                       // n of row l32 of group g, in both half-waves
                if (half == 0) sm.nrm[pos] = acc;
            }

            u32 Kw[NG];                             // U' as bit masks over list positions, 32 per word
            int np_base = 0;
#pragma unroll
            for (int I = 0; I < NG; ++I) {
                Kw[I] = 0;
                if (32 * I < m) {                   // wave-uniform
                    // this block's rows in lane-per-row form (lane l32 <-> list position 32 I + l32)
                    const u64 kb = shfl_u64(kreg[I >> 1], 32 * (I & 1) + l32);
                    const int posi = 32 * I + l32;
                    const bool validi = posi < m;
                    const bool newi = kb & 1ull;
                    const int di = (int)key_dist(kb);
                    if (half == 0) sm.t[l32] = nrm[I] - di;
                    wave_sync();
                    int4 t4[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) t4[q] = ((const int4 *)sm.t)[2 * q + half];
                    u32 F[NG];
#pragma unroll
                    for (int J = 0; J < NG; ++J) F[J] = 0;
#pragma unroll
                    for (int J = 0; J <= I; ++J) {
                        // a tile without a new row and without a new column holds only old/old pairs (lines 8-9)
                        const u32 new_I = (u32)(newm[I >> 1] >> (32 * (I & 1)));
                        const u32 new_J = (u32)(newm[J >> 1] >> (32 * (J & 1)));
                        if ((new_I | new_J) == 0) continue;
                        tiles += 1;
                        v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                        for (int s = 0; s < KS; ++s)
                            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[I][s], A[J][s], acc, 0, 0, 0);
                        // lane holds column l32 (row l32 of group J) and rows 8(a/4) + 4 half + a%4 of group I
                        const int negn = -nrm[J];
                        // bit (8(a/4) + a%4) of ft: does row 8(a/4) + 4 half + a%4 fail against column l32?
                        u32 ft = 0;
#define RNND_ROW(a, tq, comp) \
    ft |= (((acc[a] << 1) + negn) >= tq.comp) ? (1u << (8 * ((a) / 4) + ((a) % 4))) : 0u;
                        RNND_ROW(0, t4[0], x) RNND_ROW(1, t4[0], y) RNND_ROW(2, t4[0], z) RNND_ROW(3, t4[0], w)
                        RNND_ROW(4, t4[1], x) RNND_ROW(5, t4[1], y) RNND_ROW(6, t4[1], z) RNND_ROW(7, t4[1], w)
                        RNND_ROW(8, t4[2], x) RNND_ROW(9, t4[2], y) RNND_ROW(10, t4[2], z) RNND_ROW(11, t4[2], w)
                        RNND_ROW(12, t4[3], x) RNND_ROW(13, t4[3], y) RNND_ROW(14, t4[3], z) RNND_ROW(15, t4[3], w)
#undef RNND_ROW
                        ft <<= 4 * half;
                        ft |= (u32)__shfl_xor((int)ft, 32);          // column l32 against all 32 rows
                        F[J] = transpose32_bits(ft, lane);           // row l32 against all 32 columns
                        int4 *gt = (int4 *)(sm.gt + (32 * J + l32) * GT_STRIDE + 4 * half);
                        gt[0] = make_int4(acc[0], acc[1], acc[2], acc[3]);
                        gt[2] = make_int4(acc[4], acc[5], acc[6], acc[7]);
                        gt[4] = make_int4(acc[8], acc[9], acc[10], acc[11]);
                        gt[6] = make_int4(acc[12], acc[13], acc[14], acc[15]);
                    }
                    // lines 8-9: a pair is tested only if v or w is new; only w before v count
                    u32 E[NG];
#pragma unroll
                    for (int J = 0; J < NG; ++J) {
                        const u32 neww = (u32)(newm[J >> 1] >> (32 * (J & 1)));
                        u32 e = newi ? 0xFFFFFFFFu : neww;
                        if (J == I) e &= (1u << l32) - 1u;
                        if (J > I || !validi) e = 0;
                        E[J] = e;
                        F[J] &= e;
                    }
                    // lines 5-18 on masks
                    bool pre = false;
#pragma unroll
                    for (int J = 0; J < I; ++J) pre = pre || ((F[J] & Kw[J]) != 0);
                    u32 Kcur = (u32)__builtin_amdgcn_ballot_w64(validi && half == 0);
                    for (int sweep = 0; sweep < 33; ++sweep) {
                        const bool keep = validi && !pre && ((F[I] & Kcur) == 0);
                        const u32 Knew = (u32)__builtin_amdgcn_ballot_w64(keep && half == 0);
                        if (Knew == Kcur) break;
                        Kcur = Knew;
                    }
                    Kw[I] = Kcur;
                    const bool kept = (Kcur >> l32) & 1u;
                    const bool pruned = validi && !kept && half == 0;
                    // first failing w, and the evaluations Alg. 4 would have made for this row
                    int tgt = -1, ev = 0;
#pragma unroll
                    for (int J = 0; J <= I; ++J) {
                        const u32 fk = F[J] & Kw[J], ek = E[J] & Kw[J];
                        if (tgt < 0) {
                            if (fk) {
                                const int b = __builtin_ctz(fk);
                                tgt = 32 * J + b;
                                ev += __popc(ek & (0xFFFFFFFFu >> (31 - b)));
                            } else {
                                ev += __popc(ek);
                            }
                        }
                    }
                    if (half == 0) ev_lane += (u32)ev;
                    wave_sync();   // G^T tiles are in LDS
                    const u64 pm = __builtin_amdgcn_ballot_w64(pruned);
                    if (pruned) {
                        const int g = sm.gt[tgt * GT_STRIDE + l32];
                        const u32 dvw = (u32)(nrm[I] + sm.nrm[tgt] - 2 * g);
                        // line 13: v enters w's list
                        emit_redirect(make_key(dvw, key_id(kb), 1u), (u32)sm.id[tgt],
                                      props + (size_t)u * R + np_base + __popcll(pm & lanes_below(lane)));
                    }
                    np_base += __popcll(pm);
                    wave_sync();   // before the next block overwrites t and G^T
                }
            }
            // line 15 + compaction: kept entries, flag old, back into the row
            const u64 K0 = (u64)Kw[0] | (NG > 1 ? ((u64)Kw[NG > 1 ? 1 : 0] << 32) : 0ull);
            const u64 K1 = NG > 2 ? ((u64)Kw[NG > 2 ? 2 : 0] | (NG > 3 ? ((u64)Kw[NG > 3 ? 3 : 0] << 32) : 0ull)) : 0ull;
            const int nk0 = __popcll(K0);
            if ((K0 >> lane) & 1ull) row[__popcll(K0 & lanes_below(lane))] = kreg[0] & ~1ull;
            if (NG > 2 && ((K1 >> lane) & 1ull)) row[nk0 + __popcll(K1 & lanes_below(lane))] = kreg[1] & ~1ull;
            if (lane == 0) {
                deg[u] = nk0 + __popcll(K1);
                nprop[u] = np_base;
            }
            nprops_total += np_base;
        }

        // ---- rotate the pipeline
        cur = nxt;
        nxt = aft;
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int s = 0; s < KS; ++s) A[g][s] = An[g][s];
    }
    u64 evals_algo = ev_lane;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) evals_algo += shfl_xor_u64(evals_algo, o);
    if (lane == 0 && rows) add_round_stats(ctr, evals_algo, tiles * 1024ull, rows, nprops_total);
}
