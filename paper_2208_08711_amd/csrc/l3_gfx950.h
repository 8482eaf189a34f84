/*
 * gfx950 building blocks shared by the decoder and the encoder kernels of the L3
 * library: vector and address-space types, lane shifts, and the custom Paeth
 * predictor (arxiv 2208.08711 Section 4.2) on packed pairs of 16-bit fields.
 * Device code only; every translation unit gets its own copy.
 */
#ifndef L3_GFX950_H
#define L3_GFX950_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef u32x3 u32x3_any __attribute__((aligned(1)));      /* any byte alignment */
typedef uint32_t u32_any __attribute__((aligned(1)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x2 u32x2_any __attribute__((aligned(1)));

typedef __attribute__((address_space(1))) const u32x4 global_const_u32x4;
typedef __attribute__((address_space(1))) const u32_any global_const_u32_any;
typedef __attribute__((address_space(1))) u32x3_any global_u32x3_any;
typedef __attribute__((address_space(1))) u32_any global_u32_any;
typedef __attribute__((address_space(1))) u32x2_any global_u32x2_any;
typedef __attribute__((address_space(1))) uint8_t global_u8;
typedef __attribute__((address_space(1))) uint16_t global_u16;
typedef uint16_t u16_any __attribute__((aligned(1)));
typedef __attribute__((address_space(1))) u16_any global_u16_any;

__device__ __forceinline__ uint32_t dpp_from_lower_lane(uint32_t v) {   /* lane i <- lane i-1, lane 0 <- 0 */
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x138 /* wave_shr:1 */, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t dpp_from_upper_lane(uint32_t v) {   /* lane i <- lane i+1, lane 63 <- 0 */
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x130 /* wave_shl:1 */, 0xF, 0xF, true);
}

__device__ __forceinline__ uint32_t pk_mad_i16(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t d;
    asm("v_pk_mad_i16 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

/* Both 16-bit halves of v shifted right by the low half of `by`. */
__device__ __forceinline__ uint32_t pk_lshr_b16_by_low(uint32_t by, uint32_t v) {
    uint32_t d;
    asm("v_pk_lshrrev_b16 %0, %1, %2 op_sel_hi:[0,1]" : "=v"(d) : "v"(by), "v"(v));
    return d;
}
/* a * (low half of b) + c in both 16-bit halves, modulo 2^16. */
__device__ __forceinline__ uint32_t pk_mad_u16_by_low(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t d;
    asm("v_pk_mad_u16 %0, %1, %2, %3 op_sel_hi:[1,0,1]" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

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
    for (int j = 0; j < NP; ++j) asm("" : "+v"(not_lo[j]), "+v"(not_hi[j]));   /* keep the masks packed */
    /* bitop3 0xCA: first ? second : third */
#pragma unroll
    for (int j = 0; j < NP; ++j) pred[j] = __builtin_amdgcn_bitop3_b32(not_hi[j], T[j], H[j], 0xCA);
#pragma unroll
    for (int j = 0; j < NP; ++j) pred[j] = __builtin_amdgcn_bitop3_b32(not_lo[j], pred[j], L[j], 0xCA);
#pragma unroll
    for (int j = 0; j < NP; ++j) pred[j] = __builtin_amdgcn_bitop3_b32(border[j], T[j], pred[j], 0xCA);
}

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
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
