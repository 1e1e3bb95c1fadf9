// delta(a, b) = squared Euclidean distance of two rows of X (Eq. 3 with dist = squared L2),
// computed by a group of 8 consecutive lanes; all 8 receive the result.
//
//   uint8 rows : exact int32, sum of (a-b)^2 through three byte dot products per word.
//   16-bit rows: IEEE binary16 (DT_F16) or bfloat16 (DT_BF16) storage; every coordinate stands for the
//                float it converts to exactly, and the arithmetic is that of float rows (8 coordinates
//                per 16-byte chunk).
//   float rows : each lane accumulates (double)(a-b)^2 over its 16-byte chunks in chunk order,
//                the 8 partial sums are combined in a fixed xor tree, and the double is rounded
//                once to float.  (a-b)^2 == (b-a)^2 exactly, so delta(a,b) and delta(b,a) are the
//                same bits wherever they are computed.
// The result is returned as the 32 "dist_bits" of a key: the int32 value, or the float's bit pattern.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wave_prims.h"

#define DT_U8 0
#define DT_F32 1
#define DT_F16 2
#define DT_BF16 3

// bytes of one coordinate
__host__ __device__ constexpr int dt_size(int dt) { return dt == DT_U8 ? 1 : (dt == DT_F16 || dt == DT_BF16) ? 2 : 4; }

// Sum over the 8 lanes of a group, every lane receiving it: partner 1, then 2, then 4 (a fixed order, so the
// double sums are the same bits wherever they are formed).  The exchanges inside a quad are DPP moves.
__device__ __forceinline__ int group8_sum(int v)
{
    v += (int)xor_lane_u32<1>((uint32_t)v);
    v += (int)xor_lane_u32<2>((uint32_t)v);
    v += (int)xor_lane_u32<4>((uint32_t)v);
    return v;
}
__device__ __forceinline__ double group8_sum(double v)
{
    v += __builtin_bit_cast(double, xor_lane_u64(__builtin_bit_cast(unsigned long long, v), 1));
    v += __builtin_bit_cast(double, xor_lane_u64(__builtin_bit_cast(unsigned long long, v), 2));
    v += __builtin_bit_cast(double, xor_lane_u64(__builtin_bit_cast(unsigned long long, v), 4));
    return v;
}

// a 16-bit stored coordinate as the float it stands for (exact)
template <int DT>
__device__ __forceinline__ float coord16_to_float(unsigned short bits)
{
    if (DT == DT_BF16) return __uint_as_float((uint32_t)bits << 16);
    return (float)__builtin_bit_cast(_Float16, bits);
}

__device__ __forceinline__ int sqdiff_word_u8(uint32_t a, uint32_t b, int acc)
{
    // sum over 4 bytes of (a-b)^2 = a.a + b.b - 2 a.b ; every term fits comfortably in 32 bits
    uint32_t aa = __builtin_amdgcn_udot4(a, a, 0u, false);
    uint32_t bb = __builtin_amdgcn_udot4(b, b, 0u, false);
    uint32_t ab = __builtin_amdgcn_udot4(a, b, 0u, false);
    return acc + (int)(aa + bb - 2u * ab);
}

// UF (float rows): 16-byte chunks per lane whose loads are issued together before the (ordered)
// accumulation; it changes how many loads are in flight, never the order of the arithmetic.  UF >= 2.
template <int DT, int UF = 4>
__device__ __forceinline__ uint32_t group8_dist_bits(const void *pa, const void *pb, int d,
                                                     int vec_ok, int sub)
{
    if (DT == DT_U8) {
        const uint8_t *a = (const uint8_t *)pa, *b = (const uint8_t *)pb;
        int acc = 0;
        if (vec_ok) {
            const int nchunk = d >> 4;
            for (int c = sub; c < nchunk; c += 8) {
                uint4 va = ((const uint4 *)a)[c], vb = ((const uint4 *)b)[c];
                acc = sqdiff_word_u8(va.x, vb.x, acc);
                acc = sqdiff_word_u8(va.y, vb.y, acc);
                acc = sqdiff_word_u8(va.z, vb.z, acc);
                acc = sqdiff_word_u8(va.w, vb.w, acc);
            }
        } else {
            for (int e = sub; e < d; e += 8) {
                int t = (int)a[e] - (int)b[e];
                acc += t * t;
            }
        }
        acc = group8_sum(acc);
        return (uint32_t)acc;
    } else if (DT == DT_F16 || DT == DT_BF16) {
        const unsigned short *a = (const unsigned short *)pa, *b = (const unsigned short *)pb;
        typedef unsigned short us8 __attribute__((ext_vector_type(8)));
        double acc = 0.0;
        if (vec_ok) {
            const int nchunk = d >> 3;
            const us8 *pa8 = (const us8 *)a, *pb8 = (const us8 *)b;
            int c = sub;
            for (; c + 8 * (UF - 1) < nchunk; c += 8 * UF) {
                us8 va[UF], vb[UF];
#pragma unroll
                for (int k = 0; k < UF; ++k) { va[k] = pa8[c + 8 * k]; vb[k] = pb8[c + 8 * k]; }
#pragma unroll
                for (int k = 0; k < UF; ++k)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const double t = (double)coord16_to_float<DT>(va[k][e]) - (double)coord16_to_float<DT>(vb[k][e]);
                        acc = fma(t, t, acc);
                    }
            }
            if (c < nchunk) {
                // the last, shorter trip: its loads are issued together as well; a chunk past the end reads as zeros,
                // and adding the square of 0 - 0 leaves the sum as it is, so the arithmetic is that of the short loop
                us8 va[UF - 1 > 0 ? UF - 1 : 1], vb[UF - 1 > 0 ? UF - 1 : 1];
#pragma unroll
                for (int k = 0; k < UF - 1; ++k) {
                    const bool in = c + 8 * k < nchunk;
                    va[k] = in ? pa8[c + 8 * k] : (us8)(0);
                    vb[k] = in ? pb8[c + 8 * k] : (us8)(0);
                }
#pragma unroll
                for (int k = 0; k < UF - 1; ++k)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const double t = (double)coord16_to_float<DT>(va[k][e]) - (double)coord16_to_float<DT>(vb[k][e]);
                        acc = fma(t, t, acc);
                    }
            }
        } else {
            for (int e = sub; e < d; e += 8) {
                const double t = (double)coord16_to_float<DT>(a[e]) - (double)coord16_to_float<DT>(b[e]);
                acc = fma(t, t, acc);
            }
        }
        acc = group8_sum(acc);
        return __float_as_uint((float)acc);
    } else {
        const float *a = (const float *)pa, *b = (const float *)pb;
        double acc = 0.0;
        if (vec_ok) {
            const int nchunk = d >> 2;
            const float4 *pa4 = (const float4 *)a, *pb4 = (const float4 *)b;
            int c = sub;
            // UF chunks per trip, all 2 UF loads issued before the (ordered) accumulation
            for (; c + 8 * (UF - 1) < nchunk; c += 8 * UF) {
                float4 va[UF], vb[UF];
#pragma unroll
                for (int k = 0; k < UF; ++k) { va[k] = pa4[c + 8 * k]; vb[k] = pb4[c + 8 * k]; }
#pragma unroll
                for (int k = 0; k < UF; ++k) {
                    double t;
                    t = (double)va[k].x - (double)vb[k].x; acc = fma(t, t, acc);
                    t = (double)va[k].y - (double)vb[k].y; acc = fma(t, t, acc);
                    t = (double)va[k].z - (double)vb[k].z; acc = fma(t, t, acc);
                    t = (double)va[k].w - (double)vb[k].w; acc = fma(t, t, acc);
                }
            }
            if (c < nchunk) {
                // the last, shorter trip: its loads are issued together as well; a chunk past the end reads as zeros,
                // and adding the square of 0 - 0 leaves the sum as it is, so the arithmetic is that of the short loop
                float4 va[UF - 1 > 0 ? UF - 1 : 1], vb[UF - 1 > 0 ? UF - 1 : 1];
#pragma unroll
                for (int k = 0; k < UF - 1; ++k) {
                    const bool in = c + 8 * k < nchunk;
                    va[k] = in ? pa4[c + 8 * k] : make_float4(0.f, 0.f, 0.f, 0.f);
                    vb[k] = in ? pb4[c + 8 * k] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int k = 0; k < UF - 1; ++k) {
                    double t;
                    t = (double)va[k].x - (double)vb[k].x; acc = fma(t, t, acc);
                    t = (double)va[k].y - (double)vb[k].y; acc = fma(t, t, acc);
                    t = (double)va[k].z - (double)vb[k].z; acc = fma(t, t, acc);
                    t = (double)va[k].w - (double)vb[k].w; acc = fma(t, t, acc);
                }
            }
        } else {
            for (int e = sub; e < d; e += 8) {
                double t = (double)a[e] - (double)b[e];
                acc = fma(t, t, acc);
            }
        }
        acc = group8_sum(acc);
        return __float_as_uint((float)acc);
    }
}
