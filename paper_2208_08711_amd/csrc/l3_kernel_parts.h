/*
 * Parts shared by the decoder and the encoder kernels of the L3 library, written on the
 * primitives of l3_gfx950.h: the custom Paeth predictor (arxiv 2208.08711 Section 4.2) on
 * packed pairs of 16-bit fields, and the order in which workgroups take work.
 * Device code only; every translation unit gets its own copy.
 */
#ifndef L3_KERNEL_PARTS_H
#define L3_KERNEL_PARTS_H

#include "l3_gfx950.h"

namespace {

/* Section 4.2, custom Paeth filter, on NP registers of two pixels at once (16-bit
 * fields holding 0..255).  Value-wise the nearest of TL, TR, T to TL + TR - T is:
 * with lo = min(TL,TR), hi = max(TL,TR), dl = T - lo, dh = hi - T (signed):
 * lo if dl >= 2*dh, else hi if dh >= 2*dl, else T.  The stated tie order
 * (TL, TR, T) only ever chooses between equal values, except T against a
 * neighbour, where the neighbour wins: that is the ">=" above.
 * `border` has all ones in the fields whose pixel sits in the first or last
 * column of its patch, where the prediction is T.  The registers are worked on
 * in lockstep so that dependent packed instructions are not adjacent. */
template <int NP>
__device__ __forceinline__ void predict_pairs(const uint32_t (&TL)[NP], const uint32_t (&TR)[NP],
                                              const uint32_t (&T)[NP], const uint32_t (&border)[NP],
                                              uint32_t (&pred)[NP]) {
    uint32_t L[NP], H[NP], dl[NP], dh[NP], not_lo[NP], not_hi[NP];
    const uint32_t minus2 = 0xFFFEFFFEu;
#pragma unroll
    for (int j = 0; j < NP; ++j)
        L[j] = __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2, TL[j]),
                                                                      __builtin_bit_cast(u16x2, TR[j])));
#pragma unroll
    for (int j = 0; j < NP; ++j)
        H[j] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, TL[j]),
                                                                      __builtin_bit_cast(u16x2, TR[j])));
#pragma unroll
    for (int j = 0; j < NP; ++j)
        dl[j] = __builtin_bit_cast(uint32_t, (u16x2)(__builtin_bit_cast(u16x2, T[j]) -
                                                     __builtin_bit_cast(u16x2, L[j])));
#pragma unroll
    for (int j = 0; j < NP; ++j)
        dh[j] = __builtin_bit_cast(uint32_t, (u16x2)(__builtin_bit_cast(u16x2, H[j]) -
                                                     __builtin_bit_cast(u16x2, T[j])));
#pragma unroll
    for (int j = 0; j < NP; ++j) not_lo[j] = pk_mad_i16(dh[j], minus2, dl[j]);   /* dl - 2 dh */
#pragma unroll
    for (int j = 0; j < NP; ++j) not_hi[j] = pk_mad_i16(dl[j], minus2, dh[j]);   /* dh - 2 dl */
#pragma unroll
    for (int j = 0; j < NP; ++j)
        not_lo[j] = __builtin_bit_cast(uint32_t, (s16x2)(__builtin_bit_cast(s16x2, not_lo[j]) >> 15));
#pragma unroll
    for (int j = 0; j < NP; ++j)
        not_hi[j] = __builtin_bit_cast(uint32_t, (s16x2)(__builtin_bit_cast(s16x2, not_hi[j]) >> 15));
#pragma unroll
    for (int j = 0; j < NP; ++j) {   /* keep the masks packed */
        L3_OPAQUE_VGPR(not_lo[j]);
        L3_OPAQUE_VGPR(not_hi[j]);
    }
    /* bitop3 0xCA: first ? second : third */
#pragma unroll
    for (int j = 0; j < NP; ++j) pred[j] = __builtin_amdgcn_bitop3_b32(not_hi[j], T[j], H[j], 0xCA);
#pragma unroll
    for (int j = 0; j < NP; ++j) pred[j] = __builtin_amdgcn_bitop3_b32(not_lo[j], pred[j], L[j], 0xCA);
#pragma unroll
    for (int j = 0; j < NP; ++j) pred[j] = __builtin_amdgcn_bitop3_b32(border[j], T[j], pred[j], 0xCA);
}

/* Which (image, unit) a workgroup takes.  The grid is one-dimensional, a multiple of 8
 * long, and the hardware hands consecutive workgroups to the 8 XCDs in turn (workgroup L
 * runs on XCD L mod 8).  Work item number (L mod 8) * grid/8 + L / 8 therefore gives every
 * XCD one contiguous eighth of the (image, unit) sequence: neighbouring strips, whose
 * streams and output rows share cache lines, meet in the same L2. */
__device__ __forceinline__ bool take_work(uint32_t units_per_image, uint32_t images, uint32_t& image,
                                          uint32_t& unit) {
    const uint32_t eighth = gridDim.x >> 3;
    const uint32_t item = (blockIdx.x & 7u) * eighth + (blockIdx.x >> 3);
    image = item / units_per_image;
    unit = item - image * units_per_image;
    return image < images;
}

}  // namespace

#endif
