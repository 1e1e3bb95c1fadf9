// UpdateNeighbors scan (Alg. 4 lines 2-15) for float32 rows on the double-precision matrix cores.
//
// One wavefront owns one vertex u with m <= 32*NG list entries, handled as NR = 2*NG groups of 16 rows.
// The rows of the whole list are streamed through registers 16 dimensions (64 bytes per row) at a time:
// lane l loads 4 floats of row l%16 of every group, widens them to double, and for each of the 4 it feeds
// v_mfma_f64_16x16x4_f64 for every 16x16 tile (I >= J) of the Gram block G = A A^T.  The A and B operand
// of a tile come from the same loads with the same lane -> dimension mapping, so the products pair up
// whatever that mapping is.  Products of floats are exact in double, so with n_i = sum_k x_ik^2
//     delta(v_i, v_j) ~= float(n_i + n_j - 2 G_ij)
// differs from the reference value (double accumulation of (a-b)^2, rounded once) only when the two
// doubles straddle a rounding boundary of float, about 1e-8 of the time; it is used for the DECISION of
// line 11 only.  Every distance that is STORED (the delta(v,w) of a redirected edge) is recomputed by
// the one routine all stored distances come from (dist.h), so equal edges always carry equal keys.
// The outcomes are packed and transposed into one 32-bit row word per lane and 32-row block exactly as
// in the uint8 kernel, and lines 5-18 run on those masks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wave_prims.h"

typedef double v4d __attribute__((ext_vector_type(4)));

template <int NG>
struct alignas(16) F32ScanSmem {
    double nrm[32 * NG];   // n_j by list position
    u32 dist[32 * NG];     // delta(u, v_j) as float bits
    int id[32 * NG];       // vertex id by list position
    u32 ppos[32 * NG];     // redirected entries: list position of v ...
    u32 ptgt[32 * NG];     // ... and of the w it failed against
};

template <int SH, u32 M>
__device__ __forceinline__ u32 transpose_step16(u32 w, int lane)
{
    const u32 p = (u32)__shfl_xor((int)w, SH);
    const u32 lo = (w & M) | ((p & M) << SH);
    const u32 hi = ((p >> SH) & M) | (w & ~M);
    return (lane & SH) ? hi : lo;
}

// Transposes 16x16 bit matrices held one 16-bit word per lane within every group of 16 lanes.
__device__ __forceinline__ u32 transpose16_bits(u32 w, int lane)
{
    w = transpose_step16<8, 0x00FFu>(w, lane);
    w = transpose_step16<4, 0x0F0Fu>(w, lane);
    w = transpose_step16<2, 0x3333u>(w, lane);
    w = transpose_step16<1, 0x5555u>(w, lane);
    return w & 0xFFFFu;
}

// The Gram block of all NR 16-row groups over all d dimensions.  Per iteration: wait for the chunk,
// widen it to double, immediately issue the loads of the next chunk into the same registers, then run
// the matrix instructions on the doubles -- the next chunk travels while the matrix cores work.  The
// body is straight-line: loads are unconditional (lanes without a row read row 0 of X; what they
// produce is masked later) and the last iteration re-reads the last chunk.
template <int NR, int CH>
__device__ __forceinline__ void gram_f64_loop(const float *const (&rp)[NR], int nchunk, v4d (&acc)[NR * (NR + 1) / 2],
                                              double (&nr)[NR], u32 need)
{
    float4 x[NR][CH];
#pragma unroll
    for (int g = 0; g < NR; ++g)
#pragma unroll
        for (int j = 0; j < CH; ++j) x[g][j] = *(const float4 *)(rp[g] + 16 * j);
#pragma unroll 1
    for (int c = 0; c < nchunk; ++c) {
        double a[NR][CH][4];
#pragma unroll
        for (int g = 0; g < NR; ++g)
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                a[g][j][0] = (double)x[g][j].x;
                a[g][j][1] = (double)x[g][j].y;
                a[g][j][2] = (double)x[g][j].z;
                a[g][j][3] = (double)x[g][j].w;
            }
        const int cn = c + 1 < nchunk ? c + 1 : c;
        __builtin_amdgcn_sched_barrier(0);   // keep the three phases in this order
#pragma unroll
        for (int g = 0; g < NR; ++g)
#pragma unroll
            for (int j = 0; j < CH; ++j) x[g][j] = *(const float4 *)(rp[g] + 16 * (CH * cn + j));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < CH; ++j)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
#pragma unroll
                for (int g = 0; g < NR; ++g) nr[g] = fma(a[g][j][t], a[g][j][t], nr[g]);
#pragma unroll
                for (int I = 0; I < NR; ++I)
#pragma unroll
                    for (int J = 0; J <= I; ++J)
                        if (NR <= 2 || ((need >> (I * (I + 1) / 2 + J)) & 1u))   // wave-uniform
                            acc[I * (I + 1) / 2 + J] = __builtin_amdgcn_mfma_f64_16x16x4f64(
                                a[I][j][t], a[J][j][t], acc[I * (I + 1) / 2 + J], 0, 0, 0);
            }
    }
}

// CH = 16-dimension chunks fetched per loop iteration (d must be a multiple of 16*CH): a longer iteration
// gives the prefetch of the next one more matrix work to hide behind.
// NRC = 16-row groups whose rows are fetched and multiplied: 2 NG - 1 or 2 NG (lists of at most 16 NRC
// entries).
template <int NG, int CH, int NRC = 2 * NG>
__global__ __launch_bounds__(64 * 4, (NRC <= 2 ? 4 : NRC <= 5 ? 2 : 1)) void k_update_scan_mfma_f32(
    const float *__restrict__ X, int d, int R, u64 *__restrict__ keys, int *__restrict__ deg,
    const int *__restrict__ list, const u32 *__restrict__ n_list, Prop *__restrict__ props,
    int *__restrict__ nprop, RoundCtr *__restrict__ ctr)
{
    constexpr int NR = 2 * NG;
    constexpr int NT = NRC * (NRC + 1) / 2;
    static_assert(NRC == NR || NRC == NR - 1, "a list of at most 16 NRC entries spans NG 32-row blocks");
    __shared__ F32ScanSmem<NG> smem[4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, q = lane >> 4, l32 = lane & 31, half = lane >> 5, sub = lane & 7, grp = lane >> 3;
    const u32 gw = blockIdx.x * 4 + wave, nw = gridDim.x * 4;
    const u32 n_active = *n_list;
    F32ScanSmem<NG> &sm = smem[wave];
    const int nchunk = d / (16 * CH);
    u64 tiles = 0, rows = 0, nprops_total = 0;
    u32 ev_lane = 0;

    if (gw >= n_active) return;
    ScanItem cur = scan_item_load<NG>(list[gw], keys, deg, R, lane);
    ScanItem nxt = scan_item_load<NG>(gw + nw < n_active ? list[gw + nw] : -1, keys, deg, R, lane);

    for (u32 it = gw; it < n_active; it += nw) {
        int u_after = -1;
        {
            const unsigned long long j = (unsigned long long)it + 2ull * nw;
            if (j < n_active) u_after = list[j];
        }
        ScanItem aft = scan_item_load<NG>(u_after, keys, deg, R, lane);

        const int u = __builtin_amdgcn_readfirstlane(cur.u);      // same in every lane: keep it scalar
        int m = __builtin_amdgcn_readfirstlane(cur.m);
        if (m > 16 * NRC) m = 16 * NRC;   // cannot happen: the list is built per degree class
        if (m > R) m = R;
        u64 *row = keys + (size_t)u * R;
        u64 kreg[2];
        kreg[0] = lane < m ? cur.k[0] : KEY_PAD;
        kreg[1] = (NG > 2 && lane + 64 < m) ? cur.k[1] : KEY_PAD;
        u64 newm[2];
        newm[0] = __builtin_amdgcn_ballot_w64(lane < m && (kreg[0] & 1ull));
        newm[1] = __builtin_amdgcn_ballot_w64(NG > 2 && lane + 64 < m && (kreg[1] & 1ull));
        if ((newm[0] | newm[1]) == 0) {
            if (lane == 0) nprop[u] = 0;
        } else {
            wave_sync();
            if (lane < 32 * NG) { sm.id[lane] = (int)key_id(kreg[0]); sm.dist[lane] = key_dist(kreg[0]); }
            if (NG > 2 && lane + 64 < 32 * NG) {
                sm.id[64 + lane] = (int)key_id(kreg[1]);
                sm.dist[64 + lane] = key_dist(kreg[1]);
            }
            rows += m;

            // ---- which 16x16 tiles hold a pair with a new entry (lines 8-9 skip the others)
            u32 new16[NR];
            const float *rp[NRC];
#pragma unroll
            for (int g = 0; g < NR; ++g) {
                const int p = 16 * g;   // positions p .. p+15
                new16[g] = (u32)(newm[p >> 6] >> (p & 63)) & 0xFFFFu;
            }
#pragma unroll
            for (int g = 0; g < NRC; ++g) {
                const int p = 16 * g;
                const u32 idr = key_id(kreg[p >> 6]);
                const int id = __shfl((int)idr, (p & 63) + r16);
                rp[g] = X + (size_t)(p + r16 < m ? id : 0) * d + 4 * q;   // lanes without a row read row 0
            }

            // ---- Gram block over d in chunks of 16 dimensions
            v4d acc[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = (v4d){0.0, 0.0, 0.0, 0.0};
            double nr[NRC];
#pragma unroll
            for (int g = 0; g < NRC; ++g) nr[g] = 0.0;
            // tiles worth computing: rows in use, and a new entry among the rows or the columns (lines 8-9)
            u32 need = 0;
#pragma unroll
            for (int I = 0; I < NRC; ++I)
#pragma unroll
                for (int J = 0; J <= I; ++J)
                    if (16 * I < m && (new16[I] | new16[J]) != 0) need |= 1u << (I * (I + 1) / 2 + J);
            if (NRC <= 2) need = (1u << NT) - 1u;
            need = (u32)__builtin_amdgcn_readfirstlane((int)need);
            gram_f64_loop<NRC, CH>(rp, nchunk, acc, nr, need);
#pragma unroll
            for (int g = 0; g < NRC; ++g) {
                nr[g] += __shfl_xor(nr[g], 16);
                nr[g] += __shfl_xor(nr[g], 32);     // n of row r16 of group g, in all four quarter-waves
                if (q == 0) sm.nrm[16 * g + r16] = nr[g];
            }
            wave_sync();

            // ---- line 11 for every computed pair; T[I][J]: lane r16 = row r16 of group I, bit c = column c of group J
            u32 T[NR * (NR + 1) / 2];
#pragma unroll
            for (int I = 0; I < NR; ++I) {
#pragma unroll
                for (int J = 0; J <= I; ++J) {
                    const int t = I * (I + 1) / 2 + J;
                    T[t] = 0;
                    if (I >= NRC) continue;   // rows past the list (half-size form)
                    if ((need >> t) & 1u) tiles += 1;
                    if (16 * I < m && (new16[I] | new16[J]) != 0) {
                        u32 ft = 0;   // lane = column r16 (row r16 of group J); accumulator v = row 4v + q of group I
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int rowpos = 16 * I + 4 * v + q;
                            const float dvw = (float)(sm.nrm[rowpos] + nr[J < NRC ? J : 0] - 2.0 * acc[t < NT ? t : 0][v]);
                            const float di = __uint_as_float(sm.dist[rowpos]);
                            ft |= (di >= dvw) ? (1u << (4 * v + q)) : 0u;
                        }
                        ft |= (u32)__shfl_xor((int)ft, 16);
                        ft |= (u32)__shfl_xor((int)ft, 32);
                        T[t] = transpose16_bits(ft, lane);
                    }
                }
            }

            // ---- lines 5-18 on masks, one 32-row block at a time (same as the uint8 kernel)
            u32 Kw[NG];
            int np_base = 0;
            wave_sync();
#pragma unroll
            for (int I = 0; I < NG; ++I) {
                Kw[I] = 0;
                if (32 * I < m) {
                    const u64 kb = shfl_u64(kreg[I >> 1], 32 * (I & 1) + l32);
                    const int posi = 32 * I + l32;
                    const bool validi = posi < m;
                    const bool newi = kb & 1ull;
                    const bool upper = (l32 & 16) != 0;   // my row is in 16-row group 2I+1 (else 2I)
                    u32 F[NG], E[NG];
#pragma unroll
                    for (int J = 0; J < NG; ++J) {
                        u32 f = 0;
                        if (J <= I) {
                            // row group a = 2I or 2I+1, column groups 2J and 2J+1 (only tiles with column group <= row group exist)
                            const int a0 = 2 * I, a1 = 2 * I + 1;
                            const u32 lo0 = T[a0 * (a0 + 1) / 2 + 2 * J];
                            const u32 lo1 = T[a1 * (a1 + 1) / 2 + 2 * J];
                            const u32 hi0 = (2 * J + 1 <= a0) ? T[a0 * (a0 + 1) / 2 + (2 * J + 1 <= a0 ? 2 * J + 1 : 0)] : 0u;
                            const u32 hi1 = T[a1 * (a1 + 1) / 2 + 2 * J + 1];
                            f = upper ? (lo1 | (hi1 << 16)) : (lo0 | (hi0 << 16));
                        }
                        const u32 neww = (u32)(newm[J >> 1] >> (32 * (J & 1)));
                        u32 e = newi ? 0xFFFFFFFFu : neww;
                        if (J == I) e &= (1u << l32) - 1u;
                        if (J > I || !validi) e = 0;
                        E[J] = e;
                        F[J] = f & e;
                    }
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
                    const u64 pm = __builtin_amdgcn_ballot_w64(pruned);
                    if (pruned) {
                        const int p = np_base + __popcll(pm & lanes_below(lane));
                        sm.ppos[p] = (u32)posi;
                        sm.ptgt[p] = (u32)tgt;
                    }
                    np_base += __popcll(pm);
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
            wave_sync();
            // line 13: the redirected edges, with delta(v,w) from the routine every stored distance comes from
            for (int b = 0; b < np_base; b += 8) {
                const int p = b + grp;
                const bool have = p < np_base;
                const int pi = (int)sm.ppos[have ? p : 0], pt = (int)sm.ptgt[have ? p : 0];
                const int idv = sm.id[pi], idw = sm.id[pt];
                u32 db = 0;
                if (have) db = group8_dist_bits<DT_F32>(X + (size_t)idv * d, X + (size_t)idw * d, d, 1, sub);
                if (have && sub == 0) emit_redirect(make_key(db, (u32)idv, 1u), (u32)idw, props + (size_t)u * R + p);
            }
        }
        cur = nxt;
        nxt = aft;
    }
    u64 evals_algo = ev_lane;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) evals_algo += shfl_xor_u64(evals_algo, o);
    if (lane == 0 && rows) add_round_stats(ctr, evals_algo, tiles * 256ull, rows, nprops_total);
}
