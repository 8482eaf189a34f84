/*
 * gfx950 kernels and launch planning of the L3 batch decoder.
 *
 * What is computed (arxiv 2208.08711): Section 4.2, decoding direction -- per
 * patch, per row: read the 4-bit width and the 8-bit base, extract one delta
 * per pixel and add the base (base-delta decoding), then add the selected upper
 * neighbour (custom Paeth filter: nearest of top-left, top, top-right to
 * TL + TR - T; the first row is raw).  Section 4.4: patches are independent and
 * all of them are decoded in parallel; within a row every pixel is independent.
 *
 * How it is mapped to CDNA4 (this differs from the paper's one-block-per-patch,
 * one-thread-per-pixel CUDA decoder):
 *   - A workgroup of three waves owns TPW horizontally adjacent patches; wave c
 *     decodes colour channel c of all of them.  A group of LPT = N/4 lanes owns
 *     one patch; every lane owns 4 adjacent pixels of the current row, held as
 *     two packed pairs of 16-bit fields so that one v_pk_* instruction works on
 *     two pixels.
 *   - The compressed stream of each (patch, channel) is pulled from HBM in
 *     16-byte-aligned chunks (global_load_dwordx4 per lane, contiguous over the
 *     group) into a private LDS ring; the next chunk waits in registers.
 *   - Rows are handled in periods of P = 3: rings are topped up once per period
 *     for the P rows ahead; the P decoded rows of a period are parked in LDS (one
 *     word of 4 pixels per lane and channel), and after one workgroup barrier
 *     per period wave c interleaves the three channels of row c of the period
 *     and writes it to HBM (12 contiguous bytes per lane, 768 per wave row).
 *     Loads and stores share one in-order counter on this hardware, so waiting
 *     for a prefetched chunk also waits for every earlier store: the period
 *     keeps rows of decode work between issuing either and waiting for them.
 *   - The row-start chain (row r+1 begins where row r ends, and row r's length
 *     is known only from its own width field) is walked in LDS by all lanes of
 *     the group redundantly (broadcast reads), one row ahead of the arithmetic.
 *   - The upper-row neighbours come from registers: in-lane for the inner pixels,
 *     DPP wave shifts for the two pixels at the lane's edges.
 */
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>
#include <new>

#include "l3_internal.h"

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

constexpr int kBlockThreads = 192;   /* three waves: one per colour channel */

template <int N>
struct Geom {
    static_assert(N == 32 || N == 64 || N == 128, "patch sizes of the GPU path");
    static constexpr int PPL = 4;                 /* pixels per lane */
    static constexpr int LPT = N / PPL;           /* lanes per patch */
    static constexpr int TPW = 64 / LPT;          /* patches per wave */
    static constexpr int GPL = 2;                 /* 16-byte granules per lane per refill */
    static constexpr int CHUNK = LPT * 16 * GPL;  /* bytes per refill of one stream (8N) */
    static constexpr int RING = 16 * N;           /* ring bytes per stream */
    static constexpr int RING_WORDS = RING / 4 + 4; /* + 16-byte mirror of the ring start */
    static constexpr int P = 3;                   /* rows per period = waves per workgroup */
    static constexpr int ROW_MAX = N + 3;         /* bytes a row can span: ceil((12 + 8N)/8) + 1 */
    static constexpr int AHEAD = P * ROW_MAX + 12; /* bytes a period may touch past its first row */
    /* one refill per period suffices, the first refill covers the first period
     * from any start alignment, and a refill never overwrites bytes still needed */
    static_assert(CHUNK >= P * ROW_MAX, "refill keeps up with the longest rows");
    static_assert(CHUNK >= 15 + AHEAD, "first refill covers the first period");
    static_assert(RING >= AHEAD + CHUNK + ROW_MAX + 8, "ring holds a row, a period ahead and a refill");
};

/* ---- small device helpers ------------------------------------------------ */

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

/* Section 4.2, custom Paeth filter, on 2 x 2 pixels at once (two registers of
 * two 16-bit fields holding 0..255).  Value-wise the nearest of TL, TR, T to
 * TL + TR - T is: with lo = min(TL,TR), hi = max(TL,TR), dl = T - lo,
 * dh = hi - T (signed): lo if dl >= 2*dh, else hi if dh >= 2*dl, else T.  The
 * stated tie order (TL, TR, T) only ever chooses between equal values, except T
 * against a neighbour, where the neighbour wins: that is the ">=" above.
 * `border` has all ones in the fields whose pixel sits in the first or last
 * column of its patch, where the prediction is T.  The two registers are
 * worked on in lockstep so that dependent packed instructions are not adjacent. */
struct Pred2 { uint32_t p0, p1; };
__device__ __forceinline__ Pred2 predict4(uint32_t TL0, uint32_t TR0, uint32_t T0, uint32_t border0,
                                          uint32_t TL1, uint32_t TR1, uint32_t T1, uint32_t border1) {
    const u16x2 a0 = __builtin_bit_cast(u16x2, TL0), b0 = __builtin_bit_cast(u16x2, TR0),
                c0 = __builtin_bit_cast(u16x2, T0);
    const u16x2 a1 = __builtin_bit_cast(u16x2, TL1), b1 = __builtin_bit_cast(u16x2, TR1),
                c1 = __builtin_bit_cast(u16x2, T1);
    const u16x2 lo0 = __builtin_elementwise_min(a0, b0), lo1 = __builtin_elementwise_min(a1, b1);
    const u16x2 hi0 = __builtin_elementwise_max(a0, b0), hi1 = __builtin_elementwise_max(a1, b1);
    const uint32_t dl0 = __builtin_bit_cast(uint32_t, (u16x2)(c0 - lo0));
    const uint32_t dl1 = __builtin_bit_cast(uint32_t, (u16x2)(c1 - lo1));
    const uint32_t dh0 = __builtin_bit_cast(uint32_t, (u16x2)(hi0 - c0));
    const uint32_t dh1 = __builtin_bit_cast(uint32_t, (u16x2)(hi1 - c1));
    const uint32_t minus2 = 0xFFFEFFFEu;
    const s16x2 tl0 = __builtin_bit_cast(s16x2, pk_mad_i16(dh0, minus2, dl0));   /* dl - 2 dh */
    const s16x2 tl1 = __builtin_bit_cast(s16x2, pk_mad_i16(dh1, minus2, dl1));
    const s16x2 th0 = __builtin_bit_cast(s16x2, pk_mad_i16(dl0, minus2, dh0));   /* dh - 2 dl */
    const s16x2 th1 = __builtin_bit_cast(s16x2, pk_mad_i16(dl1, minus2, dh1));
    uint32_t not_lo0 = __builtin_bit_cast(uint32_t, (s16x2)(tl0 >> 15));
    uint32_t not_lo1 = __builtin_bit_cast(uint32_t, (s16x2)(tl1 >> 15));
    uint32_t not_hi0 = __builtin_bit_cast(uint32_t, (s16x2)(th0 >> 15));
    uint32_t not_hi1 = __builtin_bit_cast(uint32_t, (s16x2)(th1 >> 15));
    asm("" : "+v"(not_lo0), "+v"(not_lo1), "+v"(not_hi0), "+v"(not_hi1));   /* keep the masks packed */
    const uint32_t H0 = __builtin_bit_cast(uint32_t, hi0), L0 = __builtin_bit_cast(uint32_t, lo0);
    const uint32_t H1 = __builtin_bit_cast(uint32_t, hi1), L1 = __builtin_bit_cast(uint32_t, lo1);
    /* bitop3 0xCA: first ? second : third */
    const uint32_t r0 = __builtin_amdgcn_bitop3_b32(not_hi0, T0, H0, 0xCA);
    const uint32_t r1 = __builtin_amdgcn_bitop3_b32(not_hi1, T1, H1, 0xCA);
    const uint32_t q0 = __builtin_amdgcn_bitop3_b32(not_lo0, r0, L0, 0xCA);
    const uint32_t q1 = __builtin_amdgcn_bitop3_b32(not_lo1, r1, L1, 0xCA);
    Pred2 out;
    out.p0 = __builtin_amdgcn_bitop3_b32(border0, T0, q0, 0xCA);
    out.p1 = __builtin_amdgcn_bitop3_b32(border1, T1, q1, 0xCA);
    return out;
}

/* The 32 stream bits starting at bit `bit` of a ring live in two aligned words
 * (bit counts from the ring's aligned origin; the ring holds the stream modulo
 * RING bytes).  Three steps, so that the LDS address can be computed one row
 * ahead and the read issued long before its result is needed.  Rings are
 * addressed by their 32-bit LDS byte address. */
typedef __attribute__((address_space(3))) const uint32_t lds_const_u32;
struct RingWords { uint32_t lo, hi; };
template <int RING>
__device__ __forceinline__ uint32_t ring_where(uint32_t ring_lds, uint32_t bit) {
    static_assert((RING & (RING - 1)) == 0, "ring size is a power of two");
    uint32_t word = __builtin_amdgcn_ubfe(bit, 5, __builtin_ctz(RING / 4));
    asm("" : "+v"(word));            /* keep bfe + shift-add: two instructions, not three */
    return (word << 2) + ring_lds;
}
__device__ __forceinline__ RingWords ring_fetch(uint32_t where) {
    lds_const_u32* p = reinterpret_cast<lds_const_u32*>(where);
    RingWords v;
    v.lo = p[0];
    v.hi = p[1];   /* may be the mirror word behind the ring */
    return v;
}
__device__ __forceinline__ uint32_t ring_align(RingWords v, uint32_t bit) {
    return __builtin_amdgcn_alignbit(v.hi, v.lo, bit);   /* ({hi,lo} >> (bit & 31)) */
}

__device__ __forceinline__ u32x4 load_granule(const uint8_t* p, const uint8_t* file_end16) {
    u32x4 v = {0, 0, 0, 0};
    if (p < file_end16) v = *reinterpret_cast<global_const_u32x4*>((uintptr_t)p);
    return v;
}

__device__ __forceinline__ uint32_t load_u32_any_alignment(const uint8_t* p) {
    return *reinterpret_cast<global_const_u32_any*>((uintptr_t)p);
}

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

/* ---- the decode kernel ---------------------------------------------------- */

template <int N, int MODE>
__device__ __forceinline__ void decode_unit(const L3ImageDesc& d, uint32_t* __restrict__ status,
                                            uint32_t crop_w, uint32_t crop_h,
                                            const uint16_t* __restrict__ lut) {
    using G = Geom<N>;
    constexpr int PPL = G::PPL, LPT = G::LPT, TPW = G::TPW, GPL = G::GPL;
    constexpr int CHUNK = G::CHUNK, RING = G::RING, P = G::P;

    __shared__ __attribute__((aligned(16))) uint32_t rings[3][TPW][G::RING_WORDS];
    __shared__ uint32_t parked[2][P][3][64];   /* [buffer][row of period][channel][lane] */
    __shared__ uint16_t s_lut[MODE == L3_MODE_TENSOR ? 768 : 2];

    if (MODE == L3_MODE_TENSOR) {
        for (uint32_t i = threadIdx.x; i < 768; i += kBlockThreads) s_lut[i] = lut[i];
        __syncthreads();
    }

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t c = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   /* this wave's channel */
    const uint32_t unit = blockIdx.x;
    if (unit >= d.units) return;                                           /* whole workgroup */

    const uint32_t g = lane / LPT, xl = lane % LPT;
    const uint32_t trow = unit / d.groups_x, gx = unit - trow * d.groups_x;
    const uint32_t ty = d.tile_y_first + trow;
    const uint32_t txr = gx * TPW + g;
    const bool active = txr < d.tile_x_count;
    const uint32_t tx = d.tile_x_first + (active ? txr : d.tile_x_count - 1);
    const uint32_t x0 = tx * N, y0 = ty * N;
    const uint32_t pw = min((uint32_t)N, d.width - x0);
    uint32_t ph = min((uint32_t)N, d.height - y0);           /* same for the whole workgroup */
    if (MODE == L3_MODE_TENSOR)                              /* rows below the window are not needed */
        ph = min(ph, (uint32_t)d.crop_y0 + crop_h - y0);
    const uint32_t patches = d.tiles_x * d.tiles_y;
    const uint32_t data_len = (uint32_t)(d.file_len - d.header_bytes);
    const uint8_t* file_end16 =
        reinterpret_cast<const uint8_t*>(((uintptr_t)d.file + d.file_len + 15) & ~(uintptr_t)15);

    /* locate this lane group's stream: Section 4.3, offset array of channel c */
    uint32_t flags = 0;
    uint32_t bitpos, endbit, fill;
    const uint8_t* gaddr;
    u32x4 pf[GPL];
    uint32_t* const ring = rings[c][g];
    {
        const uint32_t flat = c * patches + ty * d.tiles_x + tx;
        const uint8_t* otab = d.file + 13 + 4 * (size_t)flat;
        uint32_t off = load_u32_any_alignment(otab);
        uint32_t end = flat + 1 < 3 * patches ? load_u32_any_alignment(otab + 4) : data_len;
        if (off > data_len || end > data_len || end < off) {
            flags |= L3_STATUS_BAD_OFFSET;
            off = min(off, data_len);
            end = min(max(end, off), data_len);
        }
        const uintptr_t a = (uintptr_t)(d.file + d.header_bytes + off);
        const uintptr_t ab = a & ~(uintptr_t)15;
        bitpos = (uint32_t)(a - ab) * 8;
        endbit = bitpos + (end - off) * 8;
        gaddr = reinterpret_cast<const uint8_t*>(ab) + xl * 16;
        /* first chunk into the ring (covers the first period), second into registers */
#pragma unroll
        for (int t = 0; t < GPL; ++t) pf[t] = load_granule(gaddr + t * LPT * 16, file_end16);
#pragma unroll
        for (int t = 0; t < GPL; ++t) {
            const uint32_t idx = (t * LPT + xl) * 16;
            *reinterpret_cast<u32x4*>(reinterpret_cast<uint8_t*>(ring) + idx) = pf[t];
            if (idx == 0) *reinterpret_cast<u32x4*>(reinterpret_cast<uint8_t*>(ring) + RING) = pf[t];
        }
        fill = CHUNK;
#pragma unroll
        for (int t = 0; t < GPL; ++t) pf[t] = load_granule(gaddr + CHUNK + t * LPT * 16, file_end16);
    }
    wave_lds_fence();

    /* per-lane constants of the row loop */
    const uint32_t xpix = xl * PPL;                         /* first pixel column of this lane */
    /* The lane's 4 pixels sit in two registers of two 16-bit fields: register 0 holds
     * pixels (0, 2), register 1 pixels (1, 3).  Then the top-right neighbours of
     * register 0 are register 1 itself and the top-left neighbours of register 1 are
     * register 0; only the two outer neighbours need a lane shift. */
    uint32_t border[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint32_t xa = xpix + j, xb = xa + 2;
        border[j] = ((xa == 0 || xa + 1 == pw) ? 0x0000FFFFu : 0u) |
                    ((xb == 0 || xb + 1 == pw) ? 0xFFFF0000u : 0u);
    }
    const uint32_t nvalid = !active ? 0u : (xpix >= pw ? 0u : min((uint32_t)PPL, pw - xpix));

    /* what the arithmetic of a row needs from its base-delta record */
    uint32_t w, w2, w3, base2, xbit, wmax = 0;
    uint32_t xwhere;   /* LDS address of the words holding this lane's deltas of the open row */
    uint32_t hwhere;   /* LDS address of the words holding the record after the open row */
    const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint32_t*)ring;

    /* Opens the row whose record (4-bit width, 8-bit base) is at bitpos: works out
     * where this lane's 4 deltas are (4w <= 32 contiguous bits) and advances bitpos
     * to the next record.  A width above 8 (damaged stream) is not clamped: ring
     * indices are masked and global loads are bounded by the file, so it can only
     * produce wrong pixels. */
    auto open_row = [&](RingWords hw) {
        const uint32_t hdr = ring_align(hw, bitpos);
        const uint32_t wr = hdr & 15u;
        const uint32_t base = __builtin_amdgcn_ubfe(hdr, 4, 8);
        const uint32_t dbit = bitpos + 12;
        bitpos = dbit + pw * wr;
        xbit = dbit + xpix * wr;
        xwhere = ring_where<RING>(ring_lds, xbit);
        hwhere = ring_where<RING>(ring_lds, bitpos);
        w = wr;
        w2 = wr + wr;
        w3 = w2 + wr;
        base2 = base | (base << 16);
    };

    /* After the workgroup barrier: this wave writes row c of the period whose rows
     * are parked in buffer `buf` (rows first .. first+count-1 of the patch). */
    auto flush = [&](uint32_t buf, uint32_t first, uint32_t count) {
        if (c >= count) return;
        const uint32_t y = y0 + first + c;
        const uint32_t* src = &parked[buf][c][0][lane];
        const uint32_t pr = src[0], pg = src[64], pb = src[128];   /* 4 pixels of R, G, B */
        if (MODE == L3_MODE_HWC) {
            uint8_t* dst = d.out + (size_t)y * d.row_stride + (size_t)(x0 + xpix) * 3;
            /* R0 G0 B0 R1 | G1 B1 R2 G2 | B2 R3 G3 B3 */
            const uint32_t t0 = __builtin_amdgcn_perm(pg, pr, 0x010c0400u);
            const uint32_t o0 = __builtin_amdgcn_perm(pb, t0, 0x03040100u);
            const uint32_t t1 = __builtin_amdgcn_perm(pb, pg, 0x020c0501u);
            const uint32_t o1 = __builtin_amdgcn_perm(pr, t1, 0x03060100u);
            const uint32_t t2 = __builtin_amdgcn_perm(pr, pb, 0x030c0702u);
            const uint32_t o2 = __builtin_amdgcn_perm(pg, t2, 0x03070100u);
            if (nvalid == PPL) {
                const u32x3 v = {o0, o1, o2};
                *reinterpret_cast<global_u32x3_any*>((uintptr_t)dst) = v;
            } else if (nvalid) {
                global_u8* b = reinterpret_cast<global_u8*>((uintptr_t)dst);
#pragma unroll
                for (int k = 0; k < 9; ++k) {
                    const uint32_t word = k < 4 ? o0 : (k < 8 ? o1 : o2);
                    if ((uint32_t)k < 3 * nvalid) b[k] = (uint8_t)(word >> (8 * (k & 3)));
                }
            }
        } else if (MODE == L3_MODE_CHW) {
#pragma unroll
            for (int ch = 0; ch < 3; ++ch) {
                const uint32_t word = ch == 0 ? pr : (ch == 1 ? pg : pb);
                uint8_t* dst = d.out + (size_t)ch * d.plane_stride + (size_t)y * d.row_stride + x0 + xpix;
                if (nvalid == PPL) {
                    *reinterpret_cast<global_u32_any*>((uintptr_t)dst) = word;
                } else if (nvalid) {
                    global_u8* b = reinterpret_cast<global_u8*>((uintptr_t)dst);
#pragma unroll
                    for (int k = 0; k < 3; ++k)
                        if ((uint32_t)k < nvalid) b[k] = (uint8_t)(word >> (8 * k));
                }
            }
        } else {
            /* tensor mode: window test, optional mirror, table of the 256 normalised
             * values.  A lane whose 4 pixels all lie inside the window writes 4 elements
             * (8 bytes) per channel at once, mirrored or not; edge lanes go element by
             * element. */
            const int32_t row = (int32_t)y - d.crop_y0;
            if (row >= 0 && row < (int32_t)crop_h && nvalid) {
                const int32_t col0 = (int32_t)(x0 + xpix) - d.crop_x0;   /* window column of pixel 0 */
                const bool whole = nvalid == PPL && col0 >= 0 && col0 + PPL <= (int32_t)crop_w;
#pragma unroll
                for (int ch = 0; ch < 3; ++ch) {
                    const uint32_t word = ch == 0 ? pr : (ch == 1 ? pg : pb);
                    const uint32_t e0 = s_lut[ch * 256 + (word & 0xFFu)];
                    const uint32_t e1 = s_lut[ch * 256 + ((word >> 8) & 0xFFu)];
                    const uint32_t e2 = s_lut[ch * 256 + ((word >> 16) & 0xFFu)];
                    const uint32_t e3 = s_lut[ch * 256 + (word >> 24)];
                    uint8_t* base = d.out + (((size_t)ch * crop_h + row) * crop_w) * 2;
                    if (whole) {
                        u32x2 v;
                        int32_t col;
                        if (d.flip) {
                            col = (int32_t)crop_w - PPL - col0;
                            v.x = e3 | (e2 << 16);
                            v.y = e1 | (e0 << 16);
                        } else {
                            col = col0;
                            v.x = e0 | (e1 << 16);
                            v.y = e2 | (e3 << 16);
                        }
                        *reinterpret_cast<global_u32x2_any*>((uintptr_t)(base + (size_t)col * 2)) = v;
                    } else {
                        global_u16* out16 = reinterpret_cast<global_u16*>((uintptr_t)base);
#pragma unroll
                        for (int k = 0; k < PPL; ++k) {
                            int32_t col = col0 + k;
                            if ((uint32_t)k < nvalid && col >= 0 && col < (int32_t)crop_w) {
                                if (d.flip) col = (int32_t)crop_w - 1 - col;
                                out16[col] = (uint16_t)(k == 0 ? e0 : (k == 1 ? e1 : (k == 2 ? e2 : e3)));
                            }
                        }
                    }
                }
            }
        }
    };

    uint32_t prev0 = 0, prev1 = 0;   /* an all-zero row above predicts 0: row 0 is raw */
    open_row(ring_fetch(ring_where<RING>(ring_lds, bitpos)));

    /* One row: no branch inside.  The deltas of the row and the record of the next
     * row travel from LDS while part 1 is computed; after the last row the record
     * read does not exist, which is harmless.  `park` is where this wave parks the
     * row (one word p0 p1 p2 p3). */
    auto do_row = [&](uint32_t* park) {
        const RingWords xw = ring_fetch(xwhere);
        const RingWords hdr_next = ring_fetch(hwhere);
        __builtin_amdgcn_sched_barrier(0);

        /* inverse filter, part 1: the prediction depends only on the row above
         * (registers + lane neighbours) */
        const uint32_t from_left = dpp_from_lower_lane(prev1);    /* pixels (1,3) of the lane below */
        const uint32_t from_right = dpp_from_upper_lane(prev0);   /* pixels (0,2) of the lane above */
        /* pixels (0,2): top-left = (3 of the lower lane, 1), top-right = (1,3);
         * pixels (1,3): top-left = (0,2), top-right = (2, 0 of the upper lane) */
        const Pred2 pr = predict4(__builtin_amdgcn_alignbit(prev1, from_left, 16), prev1, prev0, border[0],
                                  prev0, __builtin_amdgcn_alignbit(from_right, prev0, 16), prev1, border[1]);
        const uint32_t pred0 = pr.p0, pred1 = pr.p1;
        __builtin_amdgcn_sched_barrier(0);

        /* base-delta: value = base + delta; part 2 of the filter: pixel = prediction
         * + value (both mod 256, one mask at the end) */
        wmax = max(wmax, w);
        const uint32_t x = ring_align(xw, xbit);
        const uint32_t d0 = __builtin_amdgcn_ubfe(x, 0, w);
        const uint32_t d1 = __builtin_amdgcn_ubfe(x, w, w);
        const uint32_t d2 = __builtin_amdgcn_ubfe(x, w2, w);
        const uint32_t d3 = __builtin_amdgcn_ubfe(x, w3, w);
        prev0 = (pred0 + (d0 | (d2 << 16)) + base2) & 0x00FF00FFu;
        prev1 = (pred1 + (d1 | (d3 << 16)) + base2) & 0x00FF00FFu;
        *park = __builtin_amdgcn_perm(prev1, prev0, 0x06020400u);   /* p0 p1 p2 p3 */

        __builtin_amdgcn_sched_barrier(0);
        open_row(hdr_next);
    };

    /* Periods of P = 3 rows, unrolled so that the row's place in the period is a
     * constant: the previous period is written out before row 0, the ring is topped
     * up before row 2.  Only the last period can be shorter. */
    /* Waves that are ahead yield to waves that are behind (the hardware otherwise
     * favours the oldest wave, and the youngest ones would finish the kernel alone):
     * the wave's issue priority drops by one in each quarter of its rows. */
    const uint32_t quarter = (ph + 3) / 4;
    uint32_t next_drop = quarter, stage = 0;
    __builtin_amdgcn_s_setprio(3);

    uint32_t buf = 0;
    for (uint32_t r = 0; r < ph; r += P) {
        const uint32_t rows = min((uint32_t)P, ph - r);
        if (r >= next_drop) {
            next_drop += quarter;
            ++stage;
            if (stage == 1) __builtin_amdgcn_s_setprio(2);
            else if (stage == 2) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        if (r > 0) {
            /* all three channels of the previous period are parked: write them out */
            __syncthreads();
            flush(buf ^ 1u, r - P, P);
        }
        uint32_t* park = &parked[buf][0][c][lane];
        do_row(park);
        if (rows > 1) do_row(park + 3 * 64);
        if (rows > 2) {
            if (r + P < ph) {
                /* top the ring up for rows r+3 .. r+5; bitpos is the record of row r+3 */
                const uint32_t need = (bitpos >> 3) + G::AHEAD;
                if (fill < need) {
#pragma unroll
                    for (int t = 0; t < GPL; ++t) {
                        const uint32_t idx = (fill + (t * LPT + xl) * 16) & (RING - 1);
                        *reinterpret_cast<u32x4*>(reinterpret_cast<uint8_t*>(ring) + idx) = pf[t];
                        if (t == 0 && idx == 0)
                            *reinterpret_cast<u32x4*>(reinterpret_cast<uint8_t*>(ring) + RING) = pf[t];
                    }
                    fill += CHUNK;
#pragma unroll
                    for (int t = 0; t < GPL; ++t)
                        pf[t] = load_granule(gaddr + fill + t * LPT * 16, file_end16);
                }
                wave_lds_fence();
            }
            do_row(park + 2 * 3 * 64);
        }
        buf ^= 1u;
    }
    {
        const uint32_t first = ((ph - 1) / P) * P;
        __syncthreads();
        flush(buf ^ 1u, first, ph - first);
    }

    if (wmax > 8) flags |= L3_STATUS_BAD_WIDTH;
    /* bitpos is one (non-existent) row past the end: step back over it */
    if (bitpos - 12 - pw * w > endbit) flags |= L3_STATUS_OVERRUN;
    if (flags && active && status) atomicOr(&status[d.status_index], flags);
}

/* Descriptors in a device table (any batch size)... */
template <int N, int MODE>
__global__ __launch_bounds__(kBlockThreads) void l3_decode_kernel(
    const L3ImageDesc* __restrict__ descs, uint32_t* __restrict__ status, uint32_t crop_w,
    uint32_t crop_h, const uint16_t* __restrict__ lut) {
    decode_unit<N, MODE>(descs[blockIdx.y], status, crop_w, crop_h, lut);
}

/* ...or, for small batches, inside the kernel arguments: no upload, no dependency
 * on a copy, so consecutive calls run back to back. */
constexpr int kArgDescs = 32;
struct DescPack { L3ImageDesc d[kArgDescs]; };
static_assert(sizeof(DescPack) + 64 <= 4096, "kernel argument segment");

template <int N, int MODE>
__global__ __launch_bounds__(kBlockThreads) void l3_decode_kernel_args(
    const DescPack pack, uint32_t* __restrict__ status, uint32_t crop_w, uint32_t crop_h,
    const uint16_t* __restrict__ lut) {
    decode_unit<N, MODE>(pack.d[blockIdx.y], status, crop_w, crop_h, lut);
}

/* y = (x/255 - mean) / stdv for all 256 byte values of each channel, IEEE
 * binary32 without contraction, rounded to nearest-even to the 16-bit type. */
__global__ void l3_build_table_kernel(float m0, float m1, float m2, float s0, float s1, float s2,
                                      int dtype, uint16_t* __restrict__ table) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= 768) return;
    const uint32_t c = i >> 8, v = i & 255u;
    const float mean = c == 0 ? m0 : (c == 1 ? m1 : m2);
    const float stdv = c == 0 ? s0 : (c == 1 ? s1 : s2);
    const float y = __fdiv_rn(__fsub_rn(__fdiv_rn((float)v, 255.0f), mean), stdv);
    uint16_t bits;
    if (dtype == L3_BF16) {
        uint32_t u = __float_as_uint(y);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) {
            bits = (uint16_t)((u >> 16) | 0x0040u);
        } else {
            u += 0x7FFFu + ((u >> 16) & 1u);
            bits = (uint16_t)(u >> 16);
        }
    } else {
        const _Float16 h = (_Float16)y;
        bits = __builtin_bit_cast(uint16_t, h);
    }
    table[i] = bits;
}

__global__ void l3_fill_u32_kernel(uint32_t* p, uint32_t n, uint32_t value) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

/* Pulls the descriptor table from pinned host memory into device memory (words of
 * 8 bytes) and clears the status words: one small kernel on the caller's stream, so
 * that the decode kernel behind it depends on nothing but its predecessor. */
__global__ void l3_prepare_kernel(const uint64_t* __restrict__ pinned_src, uint64_t* __restrict__ dst,
                                  uint32_t words, uint32_t* status, uint32_t n_status) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) dst[i] = pinned_src[i];
    if (status && i < n_status) status[i] = 0;
}

/* ---- host side: context, planning, launch ------------------------------- */

constexpr int kSlots = 4;   /* descriptor staging slots: calls in flight before the host waits */

typedef void (*decode_kernel_t)(const L3ImageDesc*, uint32_t*, uint32_t, uint32_t, const uint16_t*);

template <int N>
decode_kernel_t kernel_for_mode(int mode) {
    switch (mode) {
        case L3_MODE_HWC: return l3_decode_kernel<N, L3_MODE_HWC>;
        case L3_MODE_CHW: return l3_decode_kernel<N, L3_MODE_CHW>;
        default: return l3_decode_kernel<N, L3_MODE_TENSOR>;
    }
}

typedef void (*decode_kernel_args_t)(const DescPack, uint32_t*, uint32_t, uint32_t, const uint16_t*);

template <int N>
decode_kernel_args_t kernel_args_for_mode(int mode) {
    switch (mode) {
        case L3_MODE_HWC: return l3_decode_kernel_args<N, L3_MODE_HWC>;
        case L3_MODE_CHW: return l3_decode_kernel_args<N, L3_MODE_CHW>;
        default: return l3_decode_kernel_args<N, L3_MODE_TENSOR>;
    }
}

decode_kernel_args_t pick_kernel_args(int n, int mode) {
    if (n == 32) return kernel_args_for_mode<32>(mode);
    if (n == 64) return kernel_args_for_mode<64>(mode);
    return kernel_args_for_mode<128>(mode);
}

decode_kernel_t pick_kernel(int n, int mode, int* tiles_per_wave) {
    if (n == 32) { *tiles_per_wave = Geom<32>::TPW; return kernel_for_mode<32>(mode); }
    if (n == 64) { *tiles_per_wave = Geom<64>::TPW; return kernel_for_mode<64>(mode); }
    *tiles_per_wave = Geom<128>::TPW; return kernel_for_mode<128>(mode);
}

}  // namespace

struct l3_ctx {
    int device = 0;
    L3ImageDesc* scratch = nullptr;       /* host: descriptors of the call being planned */
    size_t scratch_cap = 0;
    size_t cap = 0;                       /* descriptors per slot */
    L3ImageDesc* h_stage[kSlots] = {};    /* pinned host */
    L3ImageDesc* d_descs[kSlots] = {};    /* device */
    uint16_t* d_table[kSlots] = {};       /* device: 768-entry normalisation table */
    hipEvent_t done[kSlots] = {};         /* the slot's kernels have finished */
    bool pending[kSlots] = {};
    int next = 0;
};

namespace {

void release_slots(l3_ctx* ctx) {
    for (int s = 0; s < kSlots; ++s) {
        if (ctx->h_stage[s]) (void)hipHostFree(ctx->h_stage[s]);
        if (ctx->d_descs[s]) (void)hipFree(ctx->d_descs[s]);
        ctx->h_stage[s] = nullptr;
        ctx->d_descs[s] = nullptr;
    }
    ctx->cap = 0;
}

l3_status ensure_capacity(l3_ctx* ctx, size_t n) {
    if (n <= ctx->cap) return L3_OK;
    for (int s = 0; s < kSlots; ++s)
        if (ctx->pending[s]) {
            if (hipEventSynchronize(ctx->done[s]) != hipSuccess) return L3_ERR_DEVICE;
            ctx->pending[s] = false;
        }
    release_slots(ctx);
    size_t cap = 256;
    while (cap < n) cap *= 2;
    for (int s = 0; s < kSlots; ++s) {
        if (hipHostMalloc(reinterpret_cast<void**>(&ctx->h_stage[s]), cap * sizeof(L3ImageDesc),
                          hipHostMallocDefault) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&ctx->d_descs[s]), cap * sizeof(L3ImageDesc)) !=
                hipSuccess) {
            release_slots(ctx);
            return L3_ERR_DEVICE;
        }
    }
    ctx->cap = cap;
    return L3_OK;
}

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int device) {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = prev == device || hipSetDevice(device) == hipSuccess;
    }
    ~DeviceGuard() {
        int now = -1;
        if (prev >= 0 && hipGetDevice(&now) == hipSuccess && now != prev) (void)hipSetDevice(prev);
    }
};

/* Checks one item against what the GPU path needs; fills the mode-independent
 * part of its descriptor. */
l3_status check_item(const l3_item& it, L3ImageDesc* d) {
    const l3_info& f = it.info;
    if (!it.d_file || f.width == 0 || f.height == 0 || f.patch == 0) return L3_ERR_INVALID_ARG;
    const uint64_t tx = (f.width + f.patch - 1) / f.patch, ty = (f.height + f.patch - 1) / f.patch;
    if (f.patches_per_channel != tx * ty || f.header_bytes != 13 + 12 * tx * ty ||
        it.file_len < f.header_bytes || it.file_len - f.header_bytes > 0xFFFFFFFFull)
        return L3_ERR_INVALID_ARG;
    if (f.patch != 32 && f.patch != 64 && f.patch != 128) return L3_ERR_UNSUPPORTED;
    if (f.width > (1u << 24) || f.height > (1u << 24)) return L3_ERR_UNSUPPORTED;
    std::memset(d, 0, sizeof *d);
    d->file = it.d_file;
    d->file_len = it.file_len;
    d->width = f.width;
    d->height = f.height;
    d->tiles_x = (uint32_t)tx;
    d->tiles_y = (uint32_t)ty;
    d->header_bytes = (uint32_t)f.header_bytes;
    return L3_OK;
}

l3_status run_batch(l3_ctx* ctx, const l3_item* items, const l3_crop* crops, int n, int mode,
                    uint32_t crop_w, uint32_t crop_h, const float* mean, const float* stdv,
                    int dtype, void* d_out_tensor, uint32_t* d_status, void* stream_v) {
    if (!ctx || n < 0 || (n > 0 && !items)) return L3_ERR_INVALID_ARG;
    if (n == 0) return L3_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);

    DeviceGuard guard(ctx->device);
    if (!guard.ok) return L3_ERR_DEVICE;
    l3_status st = L3_OK;
    if ((size_t)n > ctx->scratch_cap) {
        size_t cap = 256;
        while (cap < (size_t)n) cap *= 2;
        L3ImageDesc* grown = static_cast<L3ImageDesc*>(std::realloc(ctx->scratch, cap * sizeof(L3ImageDesc)));
        if (!grown) return L3_ERR_DEVICE;
        ctx->scratch = grown;
        ctx->scratch_cap = cap;
    }
    L3ImageDesc* stage = ctx->scratch;

    /* descriptors grouped by patch size: classes 32, 64, 128 in this order */
    static const int kClasses[3] = {32, 64, 128};
    int class_begin[4] = {0, 0, 0, 0};
    int filled = 0;
    uint32_t max_units[3] = {0, 0, 0};
    for (int k = 0; k < 3; ++k) {
        class_begin[k] = filled;
        int tpw = 1;
        (void)pick_kernel(kClasses[k], mode, &tpw);
        for (int i = 0; i < n; ++i) {
            if (k == 0) {   /* validate everything before anything is enqueued */
                L3ImageDesc probe;
                st = check_item(items[i], &probe);
                if (st != L3_OK) return st;
                const l3_info& f = items[i].info;
                if (mode == L3_MODE_HWC &&
                    (!items[i].d_out || items[i].out_row_stride < (size_t)f.width * 3))
                    return L3_ERR_INVALID_ARG;
                if (mode == L3_MODE_CHW && (!items[i].d_out || items[i].out_row_stride < f.width))
                    return L3_ERR_INVALID_ARG;
                if (mode == L3_MODE_TENSOR) {
                    const l3_crop& cr = crops[i];
                    if (cr.x0 < 0 || cr.y0 < 0 || (uint64_t)cr.x0 + crop_w > f.width ||
                        (uint64_t)cr.y0 + crop_h > f.height)
                        return L3_ERR_INVALID_ARG;
                }
            }
            if (items[i].info.patch != kClasses[k]) continue;
            L3ImageDesc* d = &stage[filled++];
            (void)check_item(items[i], d);
            const uint32_t np = kClasses[k];
            d->status_index = (uint32_t)i;
            if (mode == L3_MODE_TENSOR) {
                const l3_crop& cr = crops[i];
                d->out = static_cast<uint8_t*>(d_out_tensor) + (size_t)i * 3 * crop_w * crop_h * 2;
                d->crop_x0 = cr.x0;
                d->crop_y0 = cr.y0;
                d->flip = cr.flip ? 1u : 0u;
                d->tile_x_first = (uint32_t)cr.x0 / np;
                d->tile_y_first = (uint32_t)cr.y0 / np;
                d->tile_x_count = ((uint32_t)cr.x0 + crop_w - 1) / np - d->tile_x_first + 1;
                const uint32_t rows = ((uint32_t)cr.y0 + crop_h - 1) / np - d->tile_y_first + 1;
                d->groups_x = (d->tile_x_count + tpw - 1) / tpw;
                d->units = d->groups_x * rows;
            } else {
                d->out = items[i].d_out;
                d->row_stride = items[i].out_row_stride;
                d->plane_stride = (uint64_t)items[i].out_row_stride * d->height;
                d->tile_x_first = d->tile_y_first = 0;
                d->tile_x_count = d->tiles_x;
                d->groups_x = (d->tiles_x + tpw - 1) / tpw;
                d->units = d->groups_x * d->tiles_y;
            }
            if (d->units > max_units[k]) max_units[k] = d->units;
        }
    }
    class_begin[3] = filled;

    /* Small batches travel inside the kernel arguments; larger ones through a device
     * table that a small kernel on the caller's stream pulls from pinned host memory. */
    bool in_args = true;
    for (int k = 0; k < 3; ++k)
        if (class_begin[k + 1] - class_begin[k] > kArgDescs) in_args = false;

    int slot = -1;
    L3ImageDesc* d_descs = nullptr;
    if (!in_args || mode == L3_MODE_TENSOR) {
        st = ensure_capacity(ctx, (size_t)n);
        if (st != L3_OK) return st;
        slot = ctx->next;
        if (ctx->pending[slot]) {
            if (hipEventSynchronize(ctx->done[slot]) != hipSuccess) return L3_ERR_DEVICE;
            ctx->pending[slot] = false;
        }
    }
    if (!in_args) {
        static_assert(sizeof(L3ImageDesc) % 8 == 0, "descriptor table is copied in 8-byte words");
        std::memcpy(ctx->h_stage[slot], stage, (size_t)n * sizeof(L3ImageDesc));
        d_descs = ctx->d_descs[slot];
        const uint32_t words = (uint32_t)((size_t)n * sizeof(L3ImageDesc) / 8);
        const uint32_t threads = words > (uint32_t)n ? words : (uint32_t)n;
        hipLaunchKernelGGL(l3_prepare_kernel, dim3((threads + 255) / 256), dim3(256), 0, stream,
                           reinterpret_cast<const uint64_t*>(ctx->h_stage[slot]),
                           reinterpret_cast<uint64_t*>(d_descs), words, d_status, (uint32_t)n);
    } else if (d_status) {
        hipLaunchKernelGGL(l3_fill_u32_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, d_status,
                           (uint32_t)n, 0u);
    }
    const uint16_t* table = nullptr;
    if (mode == L3_MODE_TENSOR) {
        hipLaunchKernelGGL(l3_build_table_kernel, dim3(3), dim3(256), 0, stream, mean[0], mean[1],
                           mean[2], stdv[0], stdv[1], stdv[2], dtype, ctx->d_table[slot]);
        table = ctx->d_table[slot];
    }
    for (int k = 0; k < 3; ++k) {
        const int count = class_begin[k + 1] - class_begin[k];
        if (count == 0 || max_units[k] == 0) continue;
        const uint32_t gx = max_units[k];
        if (in_args) {
            DescPack pack;
            std::memcpy(pack.d, stage + class_begin[k], (size_t)count * sizeof(L3ImageDesc));
            hipLaunchKernelGGL(pick_kernel_args(kClasses[k], mode), dim3(gx, (uint32_t)count),
                               dim3(kBlockThreads), 0, stream, pack, d_status, crop_w, crop_h, table);
            continue;
        }
        int tpw = 1;
        decode_kernel_t kern = pick_kernel(kClasses[k], mode, &tpw);
        for (int first = 0; first < count; first += 65535) {
            const int m = count - first < 65535 ? count - first : 65535;
            hipLaunchKernelGGL(kern, dim3(gx, (uint32_t)m), dim3(kBlockThreads), 0, stream,
                               d_descs + class_begin[k] + first, d_status, crop_w, crop_h, table);
        }
    }
    if (hipGetLastError() != hipSuccess) return L3_ERR_DEVICE;
    if (slot >= 0) {
        if (hipEventRecord(ctx->done[slot], stream) != hipSuccess) return L3_ERR_DEVICE;
        ctx->pending[slot] = true;
        ctx->next = (slot + 1) % kSlots;
    }
    return L3_OK;
}

}  // namespace

extern "C" {

l3_status l3_ctx_create(l3_ctx** out, int device) {
    if (!out || device < 0) return L3_ERR_INVALID_ARG;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device >= count) return L3_ERR_DEVICE;
    DeviceGuard guard(device);
    if (!guard.ok) return L3_ERR_DEVICE;
    l3_ctx* ctx = new (std::nothrow) l3_ctx;
    if (!ctx) return L3_ERR_DEVICE;
    ctx->device = device;
    for (int s = 0; s < kSlots; ++s) {
        if (hipEventCreateWithFlags(&ctx->done[s], hipEventDisableTiming) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&ctx->d_table[s]), 768 * sizeof(uint16_t)) !=
                hipSuccess) {
            l3_ctx_destroy(ctx);
            return L3_ERR_DEVICE;
        }
    }
    *out = ctx;
    return L3_OK;
}

void l3_ctx_destroy(l3_ctx* ctx) {
    if (!ctx) return;
    DeviceGuard guard(ctx->device);
    for (int s = 0; s < kSlots; ++s) {
        if (ctx->pending[s]) (void)hipEventSynchronize(ctx->done[s]);
        if (ctx->done[s]) (void)hipEventDestroy(ctx->done[s]);
        if (ctx->d_table[s]) (void)hipFree(ctx->d_table[s]);
    }
    release_slots(ctx);
    std::free(ctx->scratch);
    delete ctx;
}

l3_status l3_decode_batch(l3_ctx* ctx, const l3_item* items, int n, l3_layout layout,
                          uint32_t* d_status, void* stream) {
    if (layout != L3_LAYOUT_HWC && layout != L3_LAYOUT_CHW) return L3_ERR_INVALID_ARG;
    return run_batch(ctx, items, nullptr, n, layout == L3_LAYOUT_HWC ? L3_MODE_HWC : L3_MODE_CHW, 0,
                     0, nullptr, nullptr, 0, nullptr, d_status, stream);
}

l3_status l3_decode_crop_normalize_batch(l3_ctx* ctx, const l3_item* items, const l3_crop* crops,
                                         int n, uint32_t crop_w, uint32_t crop_h,
                                         const float mean[3], const float stdv[3], l3_dtype dtype,
                                         void* d_out_nchw, uint32_t* d_status, void* stream) {
    if (n > 0 && (!crops || !mean || !stdv || !d_out_nchw || crop_w == 0 || crop_h == 0))
        return L3_ERR_INVALID_ARG;
    if (dtype != L3_BF16 && dtype != L3_FP16) return L3_ERR_INVALID_ARG;
    if (n > 0 && (stdv[0] == 0.0f || stdv[1] == 0.0f || stdv[2] == 0.0f)) return L3_ERR_INVALID_ARG;
    return run_batch(ctx, items, crops, n, L3_MODE_TENSOR, crop_w, crop_h, mean, stdv, (int)dtype,
                     d_out_nchw, d_status, stream);
}

}  // extern "C"
