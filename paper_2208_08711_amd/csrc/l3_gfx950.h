/*
 * gfx950 primitives of the L3 kernels: vector and address-space types, lane shifts, packed
 * 16-bit operations, LDS addressing by 32-bit address, register pinning.  Everything in the
 * decoder that names the target sits here or is an amdgcn builtin; its own logic
 * (l3_kernel_parts.h, l3_device.hip) is written on top of these names.  (A host build of the
 * decode kernels for the sanitizers replaces this file alone: tests/native/kernel_cpu.)
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

/* true in every lane if `mine` is true in any lane of the wave */
__device__ __forceinline__ bool wave_any(bool mine) { return __builtin_amdgcn_ballot_w64(mine) != 0; }

/* ---- LDS by 32-bit address ------------------------------------------------ */

typedef __attribute__((address_space(3))) const uint32_t lds_const_u32;
struct LdsPair { uint32_t lo, hi; };
__device__ __forceinline__ uint32_t lds_address_of(const uint32_t* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const uint32_t*)p;
}
/* the two consecutive words at LDS address `where` (one ds_read2_b32) */
__device__ __forceinline__ LdsPair lds_read_pair(uint32_t where) {
    lds_const_u32* p = reinterpret_cast<lds_const_u32*>(where);
    LdsPair v;
    v.lo = p[0];
    v.hi = p[1];
    return v;
}

__device__ __forceinline__ uint32_t lds_read_u32(uint32_t where) {
    return *reinterpret_cast<lds_const_u32*>(where);
}
__device__ __forceinline__ u32x2 lds_read_u32x2(uint32_t where) {      /* 8-byte aligned */
    return *reinterpret_cast<__attribute__((address_space(3))) const u32x2*>(where);
}
__device__ __forceinline__ u32x4 lds_read_u32x4(uint32_t where) {      /* 16-byte aligned */
    return *reinterpret_cast<__attribute__((address_space(3))) const u32x4*>(where);
}
__device__ __forceinline__ void lds_write_u32x2(uint32_t where, u32x2 v) {
    *reinterpret_cast<__attribute__((address_space(3))) u32x2*>(where) = v;
}
__device__ __forceinline__ void lds_write_u32x4(uint32_t where, u32x4 v) {
    *reinterpret_cast<__attribute__((address_space(3))) u32x4*>(where) = v;
}

/* ---- keeping a value where it is ------------------------------------------ */

/* The value becomes opaque to the optimiser and stays in a vector (scalar) register: used
 * where the compiler would otherwise widen, rematerialise or reload it at a bad place. */
#define L3_KEEP_VGPR(x) asm volatile("" : "+v"(x))
#define L3_KEEP_SGPR(x) asm volatile("" : "+s"(x))
#define L3_OPAQUE_VGPR(x) asm("" : "+v"(x))     /* the same, free to move or vanish with its value */

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace

#endif
