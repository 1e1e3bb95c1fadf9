// UpdateNeighbors scan (Alg. 4, the body of the vertex loop) for float32 rows on the double-precision matrix cores.
//
// One wavefront owns one vertex u with m <= 16*NRC list entries, handled as NRC groups of 16 rows.
// The rows are streamed through registers 16 dimensions (64 bytes per row) at a time: lane l loads 4
// floats of row l%16 of every group, widens them to double, and for each of the 4 it feeds
// v_mfma_f64_16x16x4_f64 for every needed 16x16 tile (I >= J) of the Gram block G = A A^T.  The A and B
// operand of a tile come from the same loads with the same lane -> dimension mapping, so the products
// pair up whatever that mapping is.  Products of floats are exact in double, so with n_i = sum_k x_ik^2
//     delta(v_i, v_j) ~= float(n_i + n_j - 2 G_ij)
// differs from the reference value (double accumulation of (a-b)^2, rounded once) only when the two
// doubles straddle a rounding boundary of float, about 1e-8 of the time; it is used for the DECISION of
// the prune test only.  Every distance that is STORED (the delta(v,w) of a redirected edge) is recomputed by
// the one routine all stored distances come from (dist.h), so equal edges always carry equal keys.
//
// Alg. 4 never tests two old entries against each other (the old/old skip), so only pairs with a new member need a
// distance.  The list is therefore laid out in SLOTS: its new entries first, then its old ones, each in
// list order.  A tile is needed only if its column group J holds a new slot, i.e. J < ceil(#new / 16):
// with few new entries a list of 6 groups costs 6 tiles instead of 21.  Everything after the tiles
// works on slots; list order is carried by masks: before(s) = the slots whose entry precedes s's in
// the list = a prefix of the new slots and a prefix of the old slots.  Row s fails against column t
// (t before s, one of them new) iff delta(u, s) >= delta(s, t); the kept set is the fixed point of
//     K_s = not exists t in before(s): F_st and K_t ,
// found by sweeps over the whole list at once (row s is final after rank(s)+1 sweeps); the redirect
// target of a pruned row is its failing kept column that comes first in the list.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wave_prims.h"

typedef double v4d __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

#define F32_AMB_CAP 256   // pairs of one vertex that the single-precision form may leave undecided

template <int NRC>
struct alignas(16) F32ScanSmem {
    u64 key[16 * NRC];      // list entry by slot
    double nrm[16 * NRC];   // n by slot
    int pos[16 * NRC];      // list position by slot
    u32 pv[16 * NRC];       // redirected entries: slot of v ...
    u32 pw[16 * NRC];       // ... and of the w it failed against
    float nrmf[16 * NRC];   // n by slot, rounded to float (single-precision form)
    float distf[16 * NRC];  // delta(u, .) by slot
    uint16_t amb[F32_AMB_CAP];   // undecided pairs: row slot << 8 | column slot; bit 15 <- the exact outcome
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

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

template <bool FAST> struct GramAcc { typedef v4d type; typedef double norm; };
template <> struct GramAcc<true> { typedef v4f type; typedef float norm; };

// A lane's load is 16 bytes of a row: 4 float coordinates, or 8 16-bit coordinates (DT_F16: IEEE binary16, DT_BF16: bfloat16
// storage, each coordinate standing for the float it converts to exactly).  Coordinate t of such a load:
template <int DT>
__device__ __forceinline__ float chunk_coord(const uint4 &raw, int t)
{
    if (DT == DT_F16 || DT == DT_BF16) {
        const u32 w = (t >> 1) == 0 ? raw.x : (t >> 1) == 1 ? raw.y : (t >> 1) == 2 ? raw.z : raw.w;
        return coord16_to_float<DT>((unsigned short)((t & 1) ? (w >> 16) : (w & 0xFFFFu)));
    }
    return __uint_as_float(t == 0 ? raw.x : t == 1 ? raw.y : t == 2 ? raw.z : raw.w);
}
template <int DT> struct ChunkCoords { static constexpr int n = (DT == DT_F16 || DT == DT_BF16) ? 8 : 4; };

// One chunk (64 bytes of every row: lane (r16, q) holds bytes 16 q .. 16 q + 15 of row r16 of every group)
// into the norms and the Gram tiles.  The matrix instruction multiplies, for each of its 4 k slots, what
// lane quarter q supplies for the row with what it supplies for the column: the same coordinate of both,
// whichever coordinate that is.  ACC = v4f: v_mfma_f32_16x16x4_f32 on the floats; v4d: the f64 instruction.
// TM != 0: the tiles to compute are fixed at compile time (bit I(I+1)/2 + J of TM); TM == 0: bit of `need`.
template <int NR, int CH, u32 TM, int DT, typename ACC, typename NRT>
__device__ __forceinline__ void gram_chunk(const uint4 (&x)[NR][CH], ACC (&acc)[NR * (NR + 1) / 2], NRT (&nr)[NR], u32 need)
{
    if constexpr (sizeof(acc[0][0]) == 4 && (DT == DT_F16 || DT == DT_BF16)) {
        // 16-bit rows, single-precision form: the 16 bytes a lane holds are 8 coordinates in the operand format of
        // v_mfma_f32_16x16x32_{f16,bf16} as they are (products of two such numbers are exact in float); the norms
        // come from the diagonal tiles afterwards, so `need` includes those
#pragma unroll
        for (int j = 0; j < CH; ++j)
#pragma unroll
            for (int I = 0; I < NR; ++I)
#pragma unroll
                for (int J = 0; J <= I; ++J)
                    if (TM ? ((TM >> (I * (I + 1) / 2 + J)) & 1u) != 0 : ((need >> (I * (I + 1) / 2 + J)) & 1u) != 0) {   // wave-uniform
                        if constexpr (DT == DT_F16)
                            acc[I * (I + 1) / 2 + J] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                                __builtin_bit_cast(v8h, x[I][j]), __builtin_bit_cast(v8h, x[J][j]), acc[I * (I + 1) / 2 + J], 0, 0, 0);
                        else
                            acc[I * (I + 1) / 2 + J] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(v8bf, x[I][j]), __builtin_bit_cast(v8bf, x[J][j]), acc[I * (I + 1) / 2 + J], 0, 0, 0);
                    }
        return;
    }
#pragma unroll
    for (int j = 0; j < CH; ++j)
#pragma unroll
        for (int t = 0; t < ChunkCoords<DT>::n; ++t) {
            if constexpr (sizeof(acc[0][0]) == 4) {
                float a[NR];
#pragma unroll
                for (int g = 0; g < NR; ++g) {
                    a[g] = chunk_coord<DT>(x[g][j], t);
                    nr[g] = fmaf(a[g], a[g], nr[g]);      // float: its error is part of the bound
                }
#pragma unroll
                for (int I = 0; I < NR; ++I)
#pragma unroll
                    for (int J = 0; J <= I; ++J)
                        if (TM ? ((TM >> (I * (I + 1) / 2 + J)) & 1u) != 0 : ((need >> (I * (I + 1) / 2 + J)) & 1u) != 0)   // wave-uniform
                            acc[I * (I + 1) / 2 + J] =
                                __builtin_amdgcn_mfma_f32_16x16x4f32(a[I], a[J], acc[I * (I + 1) / 2 + J], 0, 0, 0);
            } else {
                double ad[NR];
#pragma unroll
                for (int g = 0; g < NR; ++g) {
                    ad[g] = (double)chunk_coord<DT>(x[g][j], t);
                    nr[g] = fma(ad[g], ad[g], nr[g]);
                }
#pragma unroll
                for (int I = 0; I < NR; ++I)
#pragma unroll
                    for (int J = 0; J <= I; ++J)
                        if (TM ? ((TM >> (I * (I + 1) / 2 + J)) & 1u) != 0 : ((need >> (I * (I + 1) / 2 + J)) & 1u) != 0)   // wave-uniform
                            acc[I * (I + 1) / 2 + J] =
                                __builtin_amdgcn_mfma_f64_16x16x4f64(ad[I], ad[J], acc[I * (I + 1) / 2 + J], 0, 0, 0);
            }
            // half rows: eight coordinates per load; keep the conversions of one step next to its matrix
            // instructions instead of letting all eight steps' worth pile up in registers
            if (DT == DT_F16 || DT == DT_BF16) __builtin_amdgcn_sched_barrier(0);
        }
}

// The Gram block of all NR 16-row groups over the whole rows, double precision.  Per iteration: wait for
// the chunk, set it aside, immediately issue the loads of the next chunk into the same registers, then run
// the matrix instructions -- the next chunk travels while the matrix cores work.  The body is
// straight-line: loads are unconditional (lanes without a row read row 0 of X; what they produce is
// masked later) and the last iteration re-reads the last chunk.  rp: byte pointers, 16 q into each row.
template <int NR, int CH, u32 TM, int DT>
__device__ __forceinline__ void gram_f64_loop(const char *const (&rp)[NR], int nchunk, v4d (&acc)[NR * (NR + 1) / 2],
                                              double (&nr)[NR], u32 need)
{
    uint4 x[NR][CH];
#pragma unroll
    for (int g = 0; g < NR; ++g)
#pragma unroll
        for (int j = 0; j < CH; ++j) x[g][j] = *(const uint4 *)(rp[g] + 64 * j);
#pragma unroll 1
    for (int c = 0; c < nchunk; ++c) {
        uint4 xc[NR][CH];
#pragma unroll
        for (int g = 0; g < NR; ++g)
#pragma unroll
            for (int j = 0; j < CH; ++j) xc[g][j] = x[g][j];
        const int cn = c + 1 < nchunk ? c + 1 : c;
        __builtin_amdgcn_sched_barrier(0);   // keep the three phases in this order
#pragma unroll
        for (int g = 0; g < NR; ++g)
#pragma unroll
            for (int j = 0; j < CH; ++j) x[g][j] = *(const uint4 *)(rp[g] + 64 * (CH * cn + j));
        __builtin_amdgcn_sched_barrier(0);
        gram_chunk<NR, CH, TM, DT, v4d, double>(xc, acc, nr, need);
    }
}

// Single-precision form: the coordinates go to v_mfma_f32_16x16x4_f32 as floats (twice the rate of the
// double-precision instruction, half the accumulator registers).  That instruction adds its four products
// one after the other, each product exact and each sum rounded to nearest, so after d dimensions
// |G - G_exact| <= d 2^-24 sum_k |x_ik x_jk| (1 + 2 d 2^-24) <= 1.01 d 2^-24 sqrt(n_i n_j).  The norms are
// summed in float as well (each lane a quarter of the coordinates).  Three buffers in rotation: while the matrix cores work on one chunk, the loads of the next
// two are in flight (the instruction is fast enough that one chunk of lead does not cover the latency of
// the gathers).  Loads past the end re-read the last chunk.
template <int NR, int CH, u32 TM, int DT>
__device__ __forceinline__ void gram_f32_loop(const char *const (&rp)[NR], int nchunk, v4f (&acc)[NR * (NR + 1) / 2],
                                              float (&nr)[NR], u32 need)
{
    uint4 x0[NR][CH], x1[NR][CH], x2[NR][CH];
    const int last = nchunk - 1;
    auto fetch = [&](uint4 (&x)[NR][CH], int c) {
        const int cc = c < last ? c : last;
#pragma unroll
        for (int g = 0; g < NR; ++g)
#pragma unroll
            for (int j = 0; j < CH; ++j) x[g][j] = *(const uint4 *)(rp[g] + 64 * (CH * cc + j));
    };
    fetch(x0, 0);
    fetch(x1, 1);
#pragma unroll 1
    for (int c = 0; c < nchunk; c += 3) {
        fetch(x2, c + 2);
        __builtin_amdgcn_sched_barrier(0);
        gram_chunk<NR, CH, TM, DT, v4f, float>(x0, acc, nr, need);
        __builtin_amdgcn_sched_barrier(0);
        if (c + 1 < nchunk) {
            fetch(x0, c + 3);
            __builtin_amdgcn_sched_barrier(0);
            gram_chunk<NR, CH, TM, DT, v4f, float>(x1, acc, nr, need);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (c + 2 < nchunk) {
            fetch(x1, c + 4);
            __builtin_amdgcn_sched_barrier(0);
            gram_chunk<NR, CH, TM, DT, v4f, float>(x2, acc, nr, need);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// bits [lo, hi) of a 96-bit mask, as word c (bits 32c .. 32c+31)
__device__ __forceinline__ u32 range_word(int lo, int hi, int c)
{
    const int a = lo - 32 * c, b = hi - 32 * c;
    const u32 below_b = b >= 32 ? 0xFFFFFFFFu : (b <= 0 ? 0u : ((1u << b) - 1u));
    const u32 below_a = a >= 32 ? 0xFFFFFFFFu : (a <= 0 ? 0u : ((1u << a) - 1u));
    return below_b & ~below_a;
}

__device__ __forceinline__ int popc_below(u64 m0, u64 m1, int p)   // set bits of the 128-bit (m0, m1) below p
{
    if (p <= 0) return 0;
    if (p < 64) return __popcll(m0 & ((1ull << p) - 1ull));
    if (p == 64) return __popcll(m0);
    return __popcll(m0) + __popcll(m1 & ((p >= 128) ? ~0ull : ((1ull << (p - 64)) - 1ull)));
}
// the same when the mask has at most 64 bits in use (ONE_WORD: m1 == 0) and 0 <= p <= 64
template <bool ONE_WORD>
__device__ __forceinline__ int popc_below_w(u64 m0, u64 m1, int p)
{
    if constexpr (ONE_WORD) return p >= 64 ? __popcll(m0) : __popcll(m0 & ((1ull << (p & 63)) - 1ull));
    else return popc_below(m0, m1, p);
}

// NRC = 16-row groups of the list (lists of at most 16 NRC entries); NG = ceil(NRC / 2) names the
// degree class family; CH = 64-byte chunks of every row fetched per loop iteration (rows a multiple of
// 64 CH bytes: a longer iteration gives the prefetch more matrix work to hide behind); DT = DT_F32 or
// DT_F16 / DT_BF16 (16-bit storage of the same kind of rows).
// FAST: the Gram block in single precision (gram_f32_loop).  A pair is then decided only if the outcome of
// the prune test is beyond the error bound of that block, eps_ij = (1.5 d + 20) 2^-24 (n_i + n_j), which
// covers the accumulation of G (2 x 1.01 d 2^-24 sqrt(n_i n_j) <= 1.01 d 2^-24 (n_i + n_j)), the norms summed
// in float (d / 4 + 2 roundings per norm), the evaluation of n_i + n_j - 2 G_ij in float and the roundings
// of delta(v,w) to float on either side (delta <= 2 (n_i + n_j)); the few undecided pairs get the exact
// delta(v,w) from the routine every stored distance comes from, so the decisions are those of the
// reference arithmetic.  A vertex with more than F32_AMB_CAP undecided pairs (ties in bulk: duplicates,
// lattices) is left untouched and appended to `redo`, which the double-precision form (FAST = false)
// takes afterwards.
// FAST with 16-bit rows: the block comes from v_mfma_f32_16x16x32_{f16,bf16} on the rows as stored (exact
// products), norms included (diagonals of the diagonal tiles).  One instruction sums 32 products and the
// accumulator; taking its error as at most 8 x 2^-24 of the sum of their magnitudes (an in-bounds probe
// against double precision stays below 2.3 x 2^-24 per instruction, also for operands spread over 20
// binades, and shows that subnormal halves count), G and either norm are off by at most
// (d / 4) 2^-24 of sqrt(n_i n_j) resp. n, hence eps_ij = (0.5 d + 20) 2^-24 (n_i + n_j).
template <int NG, int CH, int NRC = 2 * NG, bool FAST = false, int DT = DT_F32>
__global__ __launch_bounds__(64 * 4, (FAST ? (NRC <= 2 ? 4 : NRC <= 4 ? 3 : 2) : (NRC <= 2 ? 4 : NRC <= 5 ? 2 : 1))) void k_update_scan_mfma_f32(
    const char *__restrict__ X, int d, int R, u64 *__restrict__ keys, int *__restrict__ deg,
    const int *__restrict__ list, const u32 *__restrict__ n_list, Prop *__restrict__ props,
    int *__restrict__ nprop, RoundCtr *__restrict__ ctr, int *__restrict__ redo, u32 *__restrict__ n_redo)
{
    typedef typename GramAcc<FAST>::type acc_t;
    // 16-bit rows in the single-precision form: the matrix instruction takes them as they are
    constexpr bool NATIVE16 = FAST && (DT == DT_F16 || DT == DT_BF16);
    const double epsk = NATIVE16 ? (0.5 * (double)d + 20.0) * 5.9604644775390625e-08
                                 : (1.5 * (double)d + 20.0) * 5.9604644775390625e-08;
    constexpr int NT = NRC * (NRC + 1) / 2;
    constexpr int NWD = (NRC + 1) / 2;        // 32-bit words of a mask over slots
    constexpr int NSET = NRC > 4 ? 2 : 1;     // lane (r16, q) owns rows 16 q + r16 and, if NRC > 4, 64 + 16 q + r16
    static_assert(NRC >= 1 && NRC <= 6 && (NRC == 2 * NG || NRC == 2 * NG - 1), "lists of at most 96 entries");
    __shared__ F32ScanSmem<NRC> smem[4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, q = lane >> 4, sub = lane & 7, grp = lane >> 3;
    const u32 gw = blockIdx.x * 4 + wave, nw = gridDim.x * 4;
    const u32 n_active = *n_list;
    F32ScanSmem<NRC> &sm = smem[wave];
    const u32 rowbytes = (u32)d * (u32)dt_size(DT);     // at most a few hundred KB
    const int nchunk = (int)(rowbytes / (64u * CH));
    u64 tiles = 0, rows = 0, nprops_total = 0;
    u32 ev_lane = 0;

    stamp_scan_start(ctr);
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
        kreg[1] = (NRC > 4 && lane + 64 < m) ? cur.k[1] : KEY_PAD;
        // by list position: which entries are new, which old
        const u64 new0 = __builtin_amdgcn_ballot_w64(lane < m && (kreg[0] & 1ull));
        const u64 new1 = __builtin_amdgcn_ballot_w64(NRC > 4 && lane + 64 < m && (kreg[1] & 1ull));
        if ((new0 | new1) == 0) {
            if (lane == 0) nprop[u] = 0;
        } else {
            const u64 val0 = m >= 64 ? ~0ull : ((1ull << m) - 1ull);
            const u64 val1 = m > 64 ? ((1ull << (m - 64)) - 1ull) : 0ull;
            const u64 old0 = val0 & ~new0, old1 = val1 & ~new1;
            const int n_new = __popcll(new0) + __popcll(new1);
            const int g_new = (n_new + 15) >> 4;          // column groups that hold a new slot
            // ---- slots: new entries first, then old ones, each in list order
            wave_sync();
#pragma unroll
            for (int h = 0; h < (NRC > 4 ? 2 : 1); ++h) {
                const int p = 64 * h + lane;
                if (p < 16 * NRC) {
                    // a position past the list fills the slot of its own number: vertex 0, never tested
                    const bool in = p < m, isnew = kreg[h] & 1ull;
                    const int sn = popc_below_w<(NRC <= 4)>(new0, new1, p), so = n_new + popc_below_w<(NRC <= 4)>(old0, old1, p);
                    const int s = in ? (isnew ? sn : so) : p;
                    sm.key[s] = in ? kreg[h] : 0ull;
                    sm.pos[s] = p;
                    sm.distf[s] = in ? __uint_as_float(key_dist(kreg[h])) : 0.f;
                }
            }
            rows += m;
            wave_sync();

            // ---- rows of the slots, 16 per group
            const char *rp[NRC];
#pragma unroll
            for (int g = 0; g < NRC; ++g) {
                const int s = 16 * g + r16;
                const int id = s < m ? (int)key_id(sm.key[s]) : 0;      // lanes without a row read row 0
                rp[g] = X + (size_t)id * rowbytes + 16 * q;
            }
            // ---- Gram block over d in chunks of 16 dimensions: the tiles whose column group holds a new slot
            acc_t acc[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = (acc_t)(0);
            typename GramAcc<FAST>::norm nr[NRC];
#pragma unroll
            for (int g = 0; g < NRC; ++g) nr[g] = 0;
            u32 need = 0;
#pragma unroll
            for (int I = 0; I < NRC; ++I)
#pragma unroll
                for (int J = 0; J <= I; ++J)
                    if (16 * I < m && J < g_new) need |= 1u << (I * (I + 1) / 2 + J);
            need = (u32)__builtin_amdgcn_readfirstlane((int)need);
            // the tiles the Gram loop computes: those, and for 16-bit rows in the single-precision form the diagonal
            // tile of every group in use (its diagonal is the group's norms)
            u32 need_g = need;
            if constexpr (NATIVE16) {
#pragma unroll
                for (int I = 0; I < NRC; ++I)
                    if (16 * I < m) need_g |= 1u << (I * (I + 1) / 2 + I);
                need_g = (u32)__builtin_amdgcn_readfirstlane((int)need_g);
            }
            if constexpr (FAST) {
                if (NRC == 1) {
                    gram_f32_loop<NRC, CH, 1u, DT>(rp, nchunk, acc, nr, need_g);
                } else if (NRC == 2) {
                    if (NATIVE16 || need == 7u) gram_f32_loop<NRC, CH, 7u, DT>(rp, nchunk, acc, nr, need_g);
                    else gram_f32_loop<NRC, CH, 3u, DT>(rp, nchunk, acc, nr, need_g);
                } else {
                    gram_f32_loop<NRC, CH, 0u, DT>(rp, nchunk, acc, nr, need_g);
                }
            } else {
                if (NRC == 1) {
                    gram_f64_loop<NRC, CH, 1u, DT>(rp, nchunk, acc, nr, need);
                } else if (NRC == 2) {
                    // two straight-line loops instead of per-tile branches: all three tiles, or (new entries in
                    // the first group only) the two tiles of column group 0
                    if (need == 7u) gram_f64_loop<NRC, CH, 7u, DT>(rp, nchunk, acc, nr, need);
                    else gram_f64_loop<NRC, CH, 3u, DT>(rp, nchunk, acc, nr, need);
                } else {
                    gram_f64_loop<NRC, CH, 0u, DT>(rp, nchunk, acc, nr, need);
                }
            }
#pragma unroll
            for (int g = 0; g < NRC; ++g) {
                if constexpr (NATIVE16) {
                    // entry (i, i) of the group's diagonal tile sits in lane (r16 = i, q = i / 4), accumulator i % 4
                    const v4f dt = acc[g * (g + 1) / 2 + g];
                    const int vs = r16 & 3;
                    const float dv = vs == 0 ? dt[0] : vs == 1 ? dt[1] : vs == 2 ? dt[2] : dt[3];
                    nr[g] = __shfl(dv, r16 + 16 * (r16 >> 2));
                } else {
                    nr[g] += __shfl_xor(nr[g], 16);
                    nr[g] += __shfl_xor(nr[g], 32);     // n of slot 16 g + r16, in all four quarter-waves
                }
                // all four quarter-waves hold the same sum and store it (no branch)
                if (FAST) sm.nrmf[16 * g + r16] = (float)nr[g];
                else sm.nrm[16 * g + r16] = (double)nr[g];
            }
            wave_sync();

            // ---- the prune test for every pair of a computed tile, both ways round.  FA[t]: lane r16 = slot r16 of
            // group I as the tested row, bit c = column slot c of group J.  FB[t] (I != J): lane r16 = slot r16
            // of group J as the tested row, bit c = column slot c of group I.  (Same in all quarter-waves.)
            u32 FA[NT], FB[NT];
            const float epskf = (float)epsk;
#pragma unroll
            for (int I = 0; I < NRC; ++I) {
                // single-precision form: the rows of group I that this lane's accumulators stand for
                float nIf[4], dIf[4];
                if (FAST) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        nIf[v] = sm.nrmf[16 * I + 4 * q + v];
                        dIf[v] = sm.distf[16 * I + 4 * q + v];
                    }
                }
#pragma unroll
                for (int J = 0; J <= I; ++J) {
                    const int t = I * (I + 1) / 2 + J;
                    FA[t] = FB[t] = 0;
                    if (NRC == 1 || (NRC == 2 && (NATIVE16 || (need != 7u && t < 2))) || ((need_g >> t) & 1u)) tiles += 1;   // what the loop above computed
                    if ((need >> t) & 1u) {     // wave-uniform
                        // lane = slot r16 of group J; accumulator v = slot 4v + q of group I (4q + v in the
                        // single-precision instruction).  Low half of a word: the test fires; high half: undecided.
                        u32 fa = 0, fb = 0;
                        if constexpr (FAST) {
                            // all in float: the evaluation adds at most 4 x 2^-24 (n_i + n_j) to the error of
                            // delta(v,w), which the bound's constant covers
                            const float dj = sm.distf[16 * J + r16];
                            const float nJf = (float)nr[J];
                            // The outcomes with group I's slot as the tested row are taken as wavefront-wide masks:
                            // accumulator v of lane (r16, q) is (row 4q + v, column r16), so bit 16q + c of the mask
                            // of accumulator v is (row 4q + v, column c), and the row a lane stands for, r16, finds
                            // its 16 column bits in mask r16 % 4 at 16 (r16 / 4): no transposition.
                            u64 fire_m[4], amb_m[4];
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                const int rsel = 4 * q + v;
                                const float nsum = nIf[v] + nJf;
                                const float dvw = fmaf(-2.f, acc[t][v], nsum);
                                const float tol = epskf * nsum;
                                const float ta = dIf[v] - dvw, tb = dj - dvw;
                                fire_m[v] = __builtin_amdgcn_ballot_w64(ta >= 0.f);
                                amb_m[v] = __builtin_amdgcn_ballot_w64(!(fabsf(ta) > tol));      // also when not finite
                                fb |= (tb >= 0.f) ? (1u << rsel) : 0u;
                                fb |= !(fabsf(tb) > tol) ? (0x10000u << rsel) : 0u;
                            }
                            const int vs = r16 & 3, sh = 16 * (r16 >> 2);
                            const u64 mf = vs == 0 ? fire_m[0] : vs == 1 ? fire_m[1] : vs == 2 ? fire_m[2] : fire_m[3];
                            const u64 ma = vs == 0 ? amb_m[0] : vs == 1 ? amb_m[1] : vs == 2 ? amb_m[2] : amb_m[3];
                            fa = ((u32)(mf >> sh) & 0xFFFFu) | (((u32)(ma >> sh) & 0xFFFFu) << 16);
                        } else {
                            const float dj = __uint_as_float(key_dist(sm.key[16 * J + r16]));
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                const int rsel = 4 * v + q;
                                const int si = 16 * I + rsel;
                                const double dvwd = sm.nrm[si] + nr[J] - 2.0 * (double)acc[t][v];
                                const float dvw = (float)dvwd;
                                const float di = __uint_as_float(key_dist(sm.key[si]));
                                fa |= (di >= dvw) ? (1u << rsel) : 0u;
                                fb |= (dj >= dvw) ? (1u << rsel) : 0u;
                            }
                        }
                        if constexpr (FAST) {
                            FA[t] = fa;
                        } else {
                            fa |= (u32)__shfl_xor((int)fa, 16);
                            fa |= (u32)__shfl_xor((int)fa, 32);
                            FA[t] = transpose16_bits(fa, lane);
                        }
                        if (I != J) {
                            fb |= (u32)__shfl_xor((int)fb, 16);
                            fb |= (u32)__shfl_xor((int)fb, 32);
                            FB[t] = FAST ? fb : (fb & 0xFFFFu);
                        }
                    }
                }
            }

            // ---- per lane: the rows it owns (slot 16 q + r16 of set 0, slot 64 + 16 q + r16 of set 1) as masks
            // over all column slots, restricted to the pairs Alg. 4 tests
            u32 Fw[NSET][NWD], Ew[NSET][NWD], Bw[NSET][NWD], Aw[NSET][NWD];
            bool valid[NSET];
            int mypos[NSET];
#pragma unroll
            for (int e = 0; e < NSET; ++e) {
                const int rg = 4 * e + q;                 // my row group in this set
                const int s = 16 * rg + r16;
                valid[e] = rg < NRC && s < m;
                mypos[e] = valid[e] ? sm.pos[s] : 0;
                const bool snew = s < n_new;
                const int a = popc_below_w<(NRC <= 4)>(new0, new1, mypos[e]);     // new entries before mine in the list
                const int b = popc_below_w<(NRC <= 4)>(old0, old1, mypos[e]);     // old entries before mine
#pragma unroll
                for (int c = 0; c < NWD; ++c) {
                    // column groups 2c and 2c + 1
                    u32 w = 0, wa = 0;
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        const int Jc = 2 * c + hh;
                        if (Jc >= NRC) continue;
                        u32 w16 = 0;
#pragma unroll
                        for (int Ir = 4 * e; Ir < 4 * e + 4 && Ir < NRC; ++Ir) {
                            const u32 cand = Jc <= Ir ? FA[Ir * (Ir + 1) / 2 + Jc] : FB[Jc * (Jc + 1) / 2 + Ir];
                            w16 = (rg == Ir) ? cand : w16;
                        }
                        w |= (w16 & 0xFFFFu) << (16 * hh);
                        wa |= (w16 >> 16) << (16 * hh);
                    }
                    const u32 bnew = range_word(0, a, c), bold = range_word(n_new, n_new + b, c);
                    Bw[e][c] = bnew | bold;
                    Ew[e][c] = valid[e] ? (snew ? (bnew | bold) : bnew) : 0u;
                    Aw[e][c] = FAST ? (wa & Ew[e][c]) : 0u;
                    Fw[e][c] = w & Ew[e][c] & ~Aw[e][c];
                }
            }

            // ---- single precision only: the undecided pairs get the exact delta(v,w)
            bool defer = false;
            if (FAST) {
                int mine = 0;
#pragma unroll
                for (int e = 0; e < NSET; ++e)
#pragma unroll
                    for (int c = 0; c < NWD; ++c) mine += __popc(Aw[e][c]);
                int incl = mine, total = 0;
                if (__builtin_amdgcn_ballot_w64(mine != 0) != 0ull) {     // most vertices have no undecided pair at all
#pragma unroll
                    for (int o = 1; o < 64; o <<= 1) {
                        const int up = __shfl_up(incl, o);
                        if (lane >= o) incl += up;
                    }
                    total = __shfl(incl, 63);
                }
                if (total > F32_AMB_CAP) {
                    defer = true;
                    if (lane == 0) redo[atomicAdd(n_redo, 1u)] = u;
                } else if (total > 0) {
                    wave_sync();
                    int o = incl - mine;
#pragma unroll
                    for (int e = 0; e < NSET; ++e) {
                        const int s = 16 * (4 * e + q) + r16;
#pragma unroll
                        for (int c = 0; c < NWD; ++c) {
                            u32 bits = Aw[e][c];
                            while (bits) {
                                const int b = __builtin_ctz(bits);
                                bits &= bits - 1u;
                                sm.amb[o++] = (uint16_t)((s << 8) | (32 * c + b));
                            }
                        }
                    }
                    wave_sync();
                    for (int base = 0; base < total; base += 8) {
                        const int p = base + grp;
                        const bool have = p < total;
                        const u32 pair = sm.amb[have ? p : 0];
                        const u32 sv0 = (pair >> 8) & 0x7Fu, sw0 = pair & 0xFFu;
                        const u32 sv = sv0 < 16u * NRC ? sv0 : 0u, sw = sw0 < 16u * NRC ? sw0 : 0u;
                        const int idv = (int)key_id(sm.key[sv]), idw = (int)key_id(sm.key[sw]);
                        u32 db = 0;
                        if (have) db = group8_dist_bits<DT>(X + (size_t)idv * rowbytes, X + (size_t)idw * rowbytes, d, 1, sub);
                        if (have && sub == 0) {
                            const bool fails = __uint_as_float(key_dist(sm.key[sv])) >= __uint_as_float(db);
                            sm.amb[p] = (uint16_t)(pair | (fails ? 0x8000u : 0u));
                        }
                    }
                    wave_sync();
                    o = incl - mine;
#pragma unroll
                    for (int e = 0; e < NSET; ++e)
#pragma unroll
                        for (int c = 0; c < NWD; ++c) {
                            u32 bits = Aw[e][c];
                            while (bits) {
                                const int b = __builtin_ctz(bits);
                                bits &= bits - 1u;
                                if (sm.amb[o++] & 0x8000u) Fw[e][c] |= 1u << b;
                            }
                        }
                }
            }
            if (!defer) {

            // ---- the loop over v: the kept set as the fixed point, all rows at once
            u32 Kw[3] = {0u, 0u, 0u};
            u64 Kset[2] = {0ull, 0ull};       // bit lane of Kset[e]: my row of set e is kept
            {
                const u64 v0 = val0, v1 = val1;     // slots in use: 0 .. m-1 (same masks as positions)
                u64 K0 = v0;
                u32 K1 = (u32)v1;
                for (int sweep = 0; sweep < 16 * NRC + 1; ++sweep) {
                    bool hit0 = false, hit1 = false;
#pragma unroll
                    for (int c = 0; c < NWD; ++c) {
                        const u32 kc = c == 0 ? (u32)K0 : c == 1 ? (u32)(K0 >> 32) : K1;
                        hit0 = hit0 || ((Fw[0][c] & kc) != 0);
                        if (NSET > 1) hit1 = hit1 || ((Fw[NSET - 1][c] & kc) != 0);
                    }
                    const u64 b0 = __builtin_amdgcn_ballot_w64(hit0);
                    const u64 b1 = NSET > 1 ? __builtin_amdgcn_ballot_w64(hit1) : 0ull;
                    const u64 K0n = v0 & ~b0;
                    const u32 K1n = (u32)v1 & ~(u32)b1;
                    if (K0n == K0 && K1n == K1) break;
                    K0 = K0n;
                    K1 = K1n;
                }
                Kw[0] = (u32)K0;
                Kw[1] = (u32)(K0 >> 32);
                Kw[2] = K1;
                Kset[0] = K0;
                Kset[1] = (u64)K1;
            }

            // ---- kept rows go back to the list in list order; pruned rows name their target
            int np_base = 0;
            int nkept = 0;
#pragma unroll
            for (int c = 0; c < 3; ++c) nkept += __popc(Kw[c]);
            wave_sync();
#pragma unroll
            for (int e = 0; e < NSET; ++e) {
                const int s = 16 * (4 * e + q) + r16;
                const bool kept = valid[e] && ((Kset[e] >> lane) & 1ull);
                const bool pruned = valid[e] && !kept;
                int tgt = -1, ev = 0;
                if (valid[e]) {
                    // failing kept columns: the first new one and the first old one are the list-first of their kind
                    int tn = -1, to = -1;
#pragma unroll
                    for (int c = NWD - 1; c >= 0; --c) {
                        const u32 fk = Fw[e][c] & Kw[c];
                        const u32 fn = fk & range_word(0, n_new, c), fo = fk & ~range_word(0, n_new, c);
                        if (fn) tn = 32 * c + __builtin_ctz(fn);
                        if (fo) to = 32 * c + __builtin_ctz(fo);
                    }
                    if (tn >= 0 && to >= 0) tgt = sm.pos[tn] < sm.pos[to] ? tn : to;
                    else tgt = tn >= 0 ? tn : to;
                }
                // the evaluations Alg. 4 makes for this row: tested kept candidates up to and including w, i.e. the
                // slots before w in the list -- the mask the lane that owns slot w holds as its own `before` -- and w
                // (no target: everything that was tested)
                {
                    const int tl = tgt >= 0 ? (tgt & 15) + 16 * ((tgt >> 4) & 3) : lane;
#pragma unroll
                    for (int c = 0; c < NWD; ++c) {
                        u32 upto = (u32)__shfl((int)Bw[0][c], tl);
                        if (NSET > 1) {
                            const u32 hi = (u32)__shfl((int)Bw[NSET - 1][c], tl);
                            upto = (tgt >> 6) ? hi : upto;
                        }
                        if ((tgt >> 5) == c) upto |= 1u << (tgt & 31);
                        if (tgt < 0) upto = 0xFFFFFFFFu;
                        if (valid[e]) ev += __popc(Ew[e][c] & Kw[c] & upto);
                    }
                }
                ev_lane += (u32)ev;
                if (kept) {
                    int rank = 0;
#pragma unroll
                    for (int c = 0; c < NWD; ++c) rank += __popc(Kw[c] & Bw[e][c]);
                    row[rank] = sm.key[s] & ~1ull;      // kept: flag old
                }
                const u64 pm = __builtin_amdgcn_ballot_w64(pruned);
                if (pruned) {
                    const int p = np_base + __popcll(pm & lanes_below(lane));
                    sm.pv[p] = (u32)s;
                    sm.pw[p] = (u32)tgt;
                }
                np_base += __popcll(pm);
            }
            if (lane == 0) {
                deg[u] = nkept;
                nprop[u] = np_base;
            }
            nprops_total += np_base;
            wave_sync();
            // the redirected edges, with delta(v,w) from the routine every stored distance comes from
            for (int b = 0; b < np_base; b += 8) {
                const int p = b + grp;
                const bool have = p < np_base;
                const u32 sv = sm.pv[have ? p : 0], sw0 = sm.pw[have ? p : 0];
                const u32 sw = sw0 < 16u * NRC ? sw0 : 0u;     // a pruned row always has a target
                const int idv = (int)key_id(sm.key[sv]), idw = (int)key_id(sm.key[sw]);
                u32 db = 0;
                if (have) db = group8_dist_bits<DT, (NRC <= 2 ? 5 : 8)>(X + (size_t)idv * rowbytes, X + (size_t)idw * rowbytes, d, 1, sub);
                if (have && sub == 0) emit_redirect(make_key(db, (u32)idv, 1u), (u32)idw, props + (size_t)u * R + p);
            }
            }   // !defer
        }
        cur = nxt;
        nxt = aft;
    }
    u64 evals_algo = ev_lane;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) evals_algo += shfl_xor_u64(evals_algo, o);
    if (lane == 0 && rows) add_round_stats(ctr, evals_algo, tiles * 256ull, rows, nprops_total);
}
