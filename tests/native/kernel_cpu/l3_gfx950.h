/*
 * Host twin of paper_2208_08711_amd/csrc/l3_gfx950.h: the same names, written for host
 * threads (hip/hip_runtime.h beside this file), so that the decode kernels' own logic runs
 * under the sanitizers.  Each primitive states what the GPU instruction does; the kernels'
 * parity with the oracle on the CPU (tests/test_kernel_cpu_build.py) and on the GPU checks
 * that the two agree.  Included ahead of the kernel source, whose own include of the
 * product header then finds the guard set.  Test infrastructure.
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
typedef u32x3 u32x3_any __attribute__((aligned(1)));
typedef uint32_t u32_any __attribute__((aligned(1)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x2 u32x2_any __attribute__((aligned(1)));

/* "global" pointers are host pointers */
typedef const u32x4 global_const_u32x4;
typedef const u32_any global_const_u32_any;
typedef u32x3_any global_u32x3_any;
typedef u32_any global_u32_any;
typedef u32x2_any global_u32x2_any;
typedef uint8_t global_u8;
typedef uint16_t global_u16;
typedef uint16_t u16_any __attribute__((aligned(1)));
typedef u16_any global_u16_any;

/* streaming stores are plain stores here; a vector of three words is stored as three words,
 * as on the GPU (the host compiler would store the padded fourth as well) */
template <class V>
inline void l3cpu_store(V v, void* p) { std::memcpy(p, &v, sizeof v); }   /* at any alignment */
inline void l3cpu_store(u32x3 v, void* p) { std::memcpy(p, &v, 12); }
#define __builtin_nontemporal_store(v, p) l3cpu_store((v), (p))

/* wave_shr:1 / wave_shl:1 with bound_ctrl: the neighbour lane's value, 0 at the wave's end */
inline uint32_t dpp_from_lower_lane(uint32_t v) {
    const uint32_t* all = l3cpu::exchange(v);
    const unsigned l = l3cpu::lane();
    return l > 0 ? all[l - 1] : 0u;
}
inline uint32_t dpp_from_upper_lane(uint32_t v) {
    const uint32_t* all = l3cpu::exchange(v);
    const unsigned l = l3cpu::lane();
    return l < 63 ? all[l + 1] : 0u;
}
inline uint32_t l3cpu_readfirstlane(uint32_t v) { return l3cpu::exchange(v)[0]; }
/* a ballot over the wave: true if any lane's flag is */
inline bool wave_any(bool mine) {
    const uint32_t* all = l3cpu::exchange(mine ? 1u : 0u);
    uint32_t any = 0;
    for (int l = 0; l < 64; ++l) any |= all[l];
    return any != 0;
}

/* v_pk_mad_i16: a * b + c in both 16-bit halves, modulo 2^16 */
inline uint32_t pk_mad_i16(uint32_t a, uint32_t b, uint32_t c) {
    const uint32_t lo = ((a & 0xFFFFu) * (b & 0xFFFFu) + (c & 0xFFFFu)) & 0xFFFFu;
    const uint32_t hi = ((a >> 16) * (b >> 16) + (c >> 16)) & 0xFFFFu;
    return lo | (hi << 16);
}
/* v_pk_lshrrev_b16 with op_sel_hi [0,1]: both halves of v shifted right by the low four
 * bits of the low half of `by` */
inline uint32_t pk_lshr_b16_by_low(uint32_t by, uint32_t v) {
    const uint32_t sh = by & 15u;
    return ((v & 0xFFFFu) >> sh) | (((v >> 16) >> sh) << 16);
}
/* v_pk_mad_u16 with op_sel_hi [1,0,1]: a * (low half of b) + c in both halves, modulo 2^16 */
inline uint32_t pk_mad_u16_by_low(uint32_t a, uint32_t b, uint32_t c) {
    const uint32_t m = b & 0xFFFFu;
    const uint32_t lo = ((a & 0xFFFFu) * m + (c & 0xFFFFu)) & 0xFFFFu;
    const uint32_t hi = ((a >> 16) * m + (c >> 16)) & 0xFFFFu;
    return lo | (hi << 16);
}

/* v_bfe_u32: offset and width taken modulo 32 */
inline uint32_t l3cpu_ubfe(uint32_t x, uint32_t offset, uint32_t width) {
    offset &= 31u;
    width &= 31u;
    return width == 0 ? 0u : (x >> offset) & ((1u << width) - 1u);
}
/* v_alignbit_b32: the low 32 bits of {hi, lo} >> (shift mod 32) */
inline uint32_t l3cpu_alignbit(uint32_t hi, uint32_t lo, uint32_t shift) {
    return (uint32_t)((((uint64_t)hi << 32) | lo) >> (shift & 31u));
}
/* v_perm_b32: each selector byte picks a byte of {s0, s1} (0..3: s1, 4..7: s0), 12 gives
 * 0x00 and 13 and above 0xFF (the sign-replicating selectors 8..11 are not used here) */
inline uint32_t l3cpu_perm(uint32_t s0, uint32_t s1, uint32_t selector) {
    const uint64_t both = ((uint64_t)s0 << 32) | s1;
    uint32_t out = 0;
    for (int i = 0; i < 4; ++i) {
        const uint32_t sel = (selector >> (8 * i)) & 0xFFu;
        uint32_t byte;
        if (sel < 8) byte = (uint32_t)(both >> (8 * sel)) & 0xFFu;
        else if (sel == 12) byte = 0;
        else if (sel >= 13) byte = 0xFF;
        else std::abort();
        out |= byte << (8 * i);
    }
    return out;
}
/* v_bitop3_b32: bit k of the result is bit (a_k << 2 | b_k << 1 | c_k) of the table */
inline uint32_t l3cpu_bitop3(uint32_t a, uint32_t b, uint32_t c, uint32_t table) {
    uint32_t out = 0;
    for (uint32_t m = 0; m < 8; ++m)
        if (table >> m & 1u)
            out |= ((m & 4u) ? a : ~a) & ((m & 2u) ? b : ~b) & ((m & 1u) ? c : ~c);
    return out;
}
#define __builtin_amdgcn_ubfe l3cpu_ubfe
#define __builtin_amdgcn_alignbit l3cpu_alignbit
#define __builtin_amdgcn_perm l3cpu_perm
#define __builtin_amdgcn_bitop3_b32 l3cpu_bitop3
#define __builtin_amdgcn_readfirstlane l3cpu_readfirstlane
#define __builtin_amdgcn_sched_barrier(mask) ((void)0)
#define __builtin_amdgcn_s_setprio(level) ((void)0)

/* LDS is static host memory; its 32-bit addresses are offsets from one of its objects */
struct LdsPair { uint32_t lo, hi; };
inline char* l3cpu_lds_base() {
    static char base;
    return &base;
}
inline uint32_t lds_address_of(const uint32_t* p) {
    return (uint32_t)(int32_t)(reinterpret_cast<const char*>(p) - l3cpu_lds_base());
}
inline LdsPair lds_read_pair(uint32_t where) {
    const uint32_t* p = reinterpret_cast<const uint32_t*>(l3cpu_lds_base() + (int32_t)where);
    LdsPair v;
    v.lo = p[0];
    v.hi = p[1];
    return v;
}

template <class T>
inline T* l3cpu_lds_at(uint32_t where, unsigned alignment) {
    char* p = l3cpu_lds_base() + (int32_t)where;
    if (reinterpret_cast<uintptr_t>(p) % alignment != 0) std::abort();   /* the GPU requires it too */
    return reinterpret_cast<T*>(p);
}
inline uint32_t lds_read_u32(uint32_t where) { return *l3cpu_lds_at<const uint32_t>(where, 4); }
inline u32x2 lds_read_u32x2(uint32_t where) { return *l3cpu_lds_at<const u32x2>(where, 8); }
inline u32x4 lds_read_u32x4(uint32_t where) { return *l3cpu_lds_at<const u32x4>(where, 16); }
inline void lds_write_u32x2(uint32_t where, u32x2 v) { *l3cpu_lds_at<u32x2>(where, 8) = v; }
inline void lds_write_u32x4(uint32_t where, u32x4 v) { *l3cpu_lds_at<u32x4>(where, 16) = v; }

#define L3_KEEP_VGPR(x) asm volatile("" : "+r"(x))
#define L3_KEEP_SGPR(x) asm volatile("" : "+r"(x))
#define L3_OPAQUE_VGPR(x) asm("" : "+r"(x))

/* the lanes of a wave, which are threads here, meet: what one wrote to LDS the others see */
inline void wave_lds_fence() { l3cpu::wave_barrier(); }

}  // namespace

#endif
