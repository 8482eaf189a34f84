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
 *   - The grid is one-dimensional; every XCD takes a contiguous eighth of the
 *     (image, strip) sequence, so that strips which share cache lines share an L2.
 *   - Where TPW does not divide the patches of a row, the host numbers an image's
 *     units in flat order: consecutive patches in row-major order, across the ends
 *     of patch rows (all of equal height within a unit), so that lane groups idle
 *     only in the last unit of the image.
 */
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "l3_internal.h"
#include "l3_ctx.h"
#include "l3_gfx950.h"
#include "l3_kernel_parts.h"

namespace {

constexpr int kBlockThreads = 192;   /* three waves: one per colour channel */

template <int N, int PPL_>
struct Geom {
    static_assert(N == 32 || N == 64 || N == 128, "patch sizes of the GPU path");
    static_assert(PPL_ == 4 || PPL_ == 8, "pixels per lane");
    static constexpr int PPL = PPL_;              /* pixels per lane */
    static constexpr int NW = PPL / 4;            /* 4-pixel words (32-bit delta windows) per lane */
    static constexpr int NP = PPL / 2;            /* packed registers per lane */
    static constexpr int LPT = N / PPL;           /* lanes per patch */
    static constexpr int TPW = 64 / LPT;          /* patches per wave */
    static constexpr int CHUNK = 8 * N;           /* bytes per refill of one stream */
    static constexpr int GPL = CHUNK / (LPT * 16); /* 16-byte granules per lane per refill */
    static constexpr int RING = 16 * N;           /* ring bytes per stream */
    static constexpr int RING_WORDS = RING / 4 + 4; /* + 16-byte mirror of the ring start */
    static constexpr int P = 3;                   /* rows per period = waves per workgroup */
    static constexpr int QW = 64 * NW;            /* 4-pixel words per wave row */
    static constexpr int ROW_MAX = N + 3;         /* bytes a row can span: ceil((12 + 8N)/8) + 1 */
    static constexpr int AHEAD = P * ROW_MAX + 12; /* bytes a period may touch past its first row */
    /* one refill per period suffices, the first refill covers the first period
     * from any start alignment, and a refill never overwrites bytes still needed */
    static_assert(GPL * LPT * 16 == CHUNK && GPL >= 1, "chunk is a whole number of granule rounds");
    static_assert(CHUNK >= P * ROW_MAX, "refill keeps up with the longest rows");
    static_assert(CHUNK >= 15 + AHEAD, "first refill covers the first period");
    static_assert(CHUNK >= 15 + P * ROW_MAX + AHEAD, "no refill is due in the first period");
    static_assert(RING >= AHEAD + CHUNK + ROW_MAX + 8, "ring holds a row, a period ahead and a refill");
    /* how much sooner than it must a stream may take its next chunk: the chunk goes CHUNK
     * bytes behind the fill level modulo the ring, which has to stay behind the row being
     * decoded (its start is at most ROW_MAX + 8 bytes before the record of the next period) */
    static constexpr int EARLY = RING - CHUNK - ROW_MAX - 8 - AHEAD;
    static_assert(EARLY >= 1, "a refill that is due is also allowed");
    static_assert(GPL == 2 && RING == 2 * CHUNK, "two granules per lane and refill, which never wrap inside one");
};

/* The 32 stream bits starting at bit `bit` of a ring live in two aligned words
 * (bit counts from the ring's aligned origin; the ring holds the stream modulo
 * RING bytes).  Three steps, so that the LDS address can be computed one row
 * ahead and the read issued long before its result is needed.  Rings are
 * addressed by their 32-bit LDS byte address. */
typedef LdsPair RingWords;
template <int RING>
__device__ __forceinline__ uint32_t ring_where(uint32_t ring_lds, uint32_t bit) {
    static_assert((RING & (RING - 1)) == 0, "ring size is a power of two");
    uint32_t word = __builtin_amdgcn_ubfe(bit, 5, __builtin_ctz(RING / 4));
    L3_OPAQUE_VGPR(word);            /* keep bfe + shift-add: two instructions, not three */
    return (word << 2) + ring_lds;
}
__device__ __forceinline__ RingWords ring_fetch(uint32_t where) {
    return lds_read_pair(where);   /* the second word may be the mirror word behind the ring */
}
__device__ __forceinline__ uint32_t ring_align(RingWords v, uint32_t bit) {
    return __builtin_amdgcn_alignbit(v.hi, v.lo, bit);   /* ({hi,lo} >> (bit & 31)) */
}

/* One 16-byte granule of a patch stream, zeros at and beyond `limit` (byte offsets from
 * the stream's aligned origin): nothing is fetched past the granule that holds the
 * stream's last byte. */
__device__ __forceinline__ u32x4 load_granule(const uint8_t* origin, uint32_t at, uint32_t limit) {
    u32x4 v = {0, 0, 0, 0};
    if (at < limit) v = *reinterpret_cast<global_const_u32x4*>((uintptr_t)(origin + at));
    return v;
}

__device__ __forceinline__ uint32_t load_u32_any_alignment(const uint8_t* p) {
    return *reinterpret_cast<global_const_u32_any*>((uintptr_t)p);
}

/* ---- the fused epilogue's table ------------------------------------------- */

/* The 256 normalised values per channel as 16-bit patterns, [channel][byte value]: what
 * the fused kernels look pixels up in.  It travels inside the kernel arguments. */
struct L3Table {
    uint16_t bits[768];
};
struct L3NoTable {};
template <int MODE> struct TailFor { typedef L3NoTable type; };
template <> struct TailFor<L3_MODE_TENSOR> { typedef L3Table type; };

/* y = (v/255 - mean) / stdv in IEEE binary32 without contraction, rounded to nearest-even
 * to the 16-bit type; returns its bits.  (The host works the same values out in
 * l3_normalized_values; the call that keeps its table in device memory uses this one.) */
__device__ __forceinline__ uint16_t normalised_bits(uint32_t v, float mean, float stdv, int dtype) {
    const float y = __fdiv_rn(__fsub_rn(__fdiv_rn((float)v, 255.0f), mean), stdv);
    if (dtype == L3_BF16) {
        uint32_t u = __float_as_uint(y);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
    const _Float16 h = (_Float16)y;
    return __builtin_bit_cast(uint16_t, h);
}

/* ---- the decode kernel ---------------------------------------------------- */

template <int N, int PPL, int MODE>
__device__ __forceinline__ void decode_unit(const L3ImageDesc& d, const uint32_t unit,
                                            uint32_t* __restrict__ status, uint32_t crop_w,
                                            uint32_t crop_h, const bool keeps_priority,
                                            const uint32_t age_rank,
                                            const uint16_t* __restrict__ lut) {
    using G = Geom<N, PPL>;
    constexpr int LPT = G::LPT, TPW = G::TPW, GPL = G::GPL, NW = G::NW, NP = G::NP, QW = G::QW;
    constexpr int CHUNK = G::CHUNK, RING = G::RING, P = G::P;

    __shared__ __attribute__((aligned(16))) uint32_t rings[3][TPW][G::RING_WORDS];
    /* Where the period's barrier sits (see the period loop): behind row 0 for the
     * small-patch pixel modes, where it measured 3 % faster; in front of row 0 otherwise
     * (no gain at N = 128, and the third parking buffer it needs costs the fused path a
     * workgroup per CU). */
    constexpr bool LATE_BARRIER = N == 32 && MODE != L3_MODE_TENSOR;
    /* Planar output needs nothing from the other channels: a wave can write its rows
     * itself as it decodes them, 4 pixels per lane, 256 contiguous bytes per wave row, with
     * no parking and no barrier.  That measured 4 to 5 % faster than the parked route for
     * N = 128 and slower for N = 64 and 32 (three times as many store instructions for
     * the same bytes), so only N = 128 takes it. */
    constexpr bool DIRECT = MODE == L3_MODE_CHW && PPL == 4 && N == 128;
    constexpr int PARKS = LATE_BARRIER ? 3 : 2;
    __shared__ __attribute__((aligned(8))) uint32_t parked[PARKS][P][3][QW]; /* [buffer][row of period][channel][word] */
    __shared__ uint16_t s_lut[MODE == L3_MODE_TENSOR ? 768 : 2];

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t c = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   /* this wave's channel */
    if (unit >= d.units) return;                                           /* whole workgroup */
    /* the table of normalised values (first needed by the first write-out) is requested
     * first and put into LDS behind the stream's first chunk, so that it costs no round
     * trip of its own */
    uint16_t lut_part[4] = {0, 0, 0, 0};
    if (MODE == L3_MODE_TENSOR) {
#pragma unroll
        for (int k = 0; k < 4; ++k) lut_part[k] = lut[threadIdx.x + k * kBlockThreads];
    }

    const uint32_t g = lane / LPT, xl = lane % LPT;
    /* Which patch this lane group decodes: (tx, ty); ty_base is the patch row of the
     * unit's first group, the same for the whole workgroup. */
    uint32_t tx, ty, ty_base, strip_x0 = 0;
    bool active;
    const bool flat_order = MODE != L3_MODE_TENSOR && PPL == 4 && d.groups_x == 0;
    if (flat_order) {
        const bool upper = unit < d.flat_upper_units;
        const uint32_t first = (upper ? unit : unit - d.flat_upper_units) * TPW;
        const uint32_t count = upper ? d.tiles_x * d.flat_upper_rows : d.tiles_x;
        const uint32_t row_off = upper ? 0u : d.flat_upper_rows;
        const uint32_t fl = first + g;
        active = fl < count;
        const uint32_t flc = active ? fl : count - 1;
        const uint32_t qrow = flc / d.tiles_x;
        ty = row_off + qrow;
        tx = flc - qrow * d.tiles_x;
        ty_base = row_off + first / d.tiles_x;
    } else {
        const uint32_t trow = unit / d.groups_x, gx = unit - trow * d.groups_x;
        const uint32_t txr = gx * TPW + g;
        active = txr < d.tile_x_count;
        tx = d.tile_x_first + (active ? txr : d.tile_x_count - 1);
        ty = ty_base = d.tile_y_first + trow;
        strip_x0 = (d.tile_x_first + gx * TPW) * N;   /* first column of the wave's strip */
    }
    const uint32_t x0 = tx * N, y0 = ty_base * N;     /* y0: first image row of the unit's first patch */
    const uint32_t pw = min((uint32_t)N, d.width - x0);
    uint32_t ph = min((uint32_t)N, d.height - y0);           /* same for the whole workgroup */
    if (MODE == L3_MODE_TENSOR)                              /* rows below the window are not needed */
        ph = min(ph, (uint32_t)d.crop_y0 + crop_h - y0);
    const uint32_t patches = d.tiles_x * d.tiles_y;
    const uint32_t data_len = (uint32_t)(d.file_len - d.header_bytes);

    /* locate this lane group's stream: Section 4.3, offset array of channel c */
    uint32_t flags = 0;
    uint32_t bitpos, endbit, fill, limit;
    const uint8_t* origin;
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
        origin = reinterpret_cast<const uint8_t*>(ab);
        limit = ((endbit >> 3) + 15u) & ~15u;     /* the stream's granules end here; inside the file's last one */
        /* first chunk into the ring (covers the first period), second into registers */
#pragma unroll
        for (int t = 0; t < GPL; ++t) pf[t] = load_granule(origin, (t * LPT + xl) * 16, limit);
#pragma unroll
        for (int t = 0; t < GPL; ++t) {
            const uint32_t idx = (t * LPT + xl) * 16;
            *reinterpret_cast<u32x4*>(reinterpret_cast<uint8_t*>(ring) + idx) = pf[t];
            if (idx == 0) *reinterpret_cast<u32x4*>(reinterpret_cast<uint8_t*>(ring) + RING) = pf[t];
        }
        fill = CHUNK + xl * 16;   /* this lane's first granule of the chunk in pf: see the ring top-up */
        /* the second chunk is asked for in the first period, not here, where every workgroup
         * of the launch waits for its first one */
#pragma unroll
        for (int t = 0; t < GPL; ++t) pf[t] = u32x4{0, 0, 0, 0};
    }
    if (MODE == L3_MODE_TENSOR) {
#pragma unroll
        for (int k = 0; k < 4; ++k) s_lut[threadIdx.x + k * kBlockThreads] = lut_part[k];
        __syncthreads();
    }
    wave_lds_fence();

    /* The lane's pixels, 4 per word k (pixels 4k .. 4k+3 of the lane), sit in registers
     * of two 16-bit fields: register 2k holds pixels (4k, 4k+2), register 2k+1 pixels
     * (4k+1, 4k+3).  Then the top-right neighbours of an even register are the odd
     * register beside it and the top-left neighbours of an odd register the even one;
     * the other neighbours take one alignbit, the two outermost a lane shift. */
    const uint32_t xpix = xl * PPL;                         /* first pixel column of this lane */
    uint32_t border[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        const uint32_t xa = xpix + 4 * (j / 2) + (j & 1), xb = xa + 2;
        border[j] = ((xa == 0 || xa + 1 == pw) ? 0x0000FFFFu : 0u) |
                    ((xb == 0 || xb + 1 == pw) ? 0xFFFF0000u : 0u);
    }

    /* what the arithmetic of a row needs from its base-delta record */
    uint32_t w, w2, K, base2, xbit[NW], wmax = 0;
    uint32_t xwhere[NW];   /* LDS addresses of the words holding this lane's deltas of the open row */
    uint32_t hwhere;       /* LDS address of the words holding the record after the open row */
    const uint32_t ring_lds = lds_address_of(ring);

    /* Opens the row whose record (4-bit width, 8-bit base) is at bitpos: works out
     * where this lane's deltas are (4w <= 32 contiguous bits per word of 4 pixels) and
     * advances bitpos to the next record.  A width above 8 (damaged stream) is not
     * clamped: ring indices are masked and global loads are bounded by the file, so it
     * can only produce wrong pixels. */
    auto open_row = [&](RingWords hw) {
        const uint32_t hdr = ring_align(hw, bitpos);
        const uint32_t wr = hdr & 15u;
        const uint32_t base = __builtin_amdgcn_ubfe(hdr, 4, 8);
        const uint32_t dbit = bitpos + 12;
        bitpos = dbit + pw * wr;
        xbit[0] = dbit + xpix * wr;
#pragma unroll
        for (int k = 1; k < NW; ++k) xbit[k] = xbit[k - 1] + 4 * wr;
#pragma unroll
        for (int k = 0; k < NW; ++k) xwhere[k] = ring_where<RING>(ring_lds, xbit[k]);
        hwhere = ring_where<RING>(ring_lds, bitpos);
        w = wr;
        w2 = wr + wr;
        K = 0xFFFFFFFFu << wr;
        base2 = base | (base << 16);
    };

    /* What the write-out needs from the descriptor, pinned in registers: left to
     * itself the compiler reloads these from the argument segment after every
     * barrier, and the wave waits for the scalar load each period. */
    uint64_t out_base = (uint64_t)(uintptr_t)d.out, out_row_stride = d.row_stride,
             out_plane_stride = d.plane_stride;
    uint32_t img_width = d.width;
    int32_t win_x0 = d.crop_x0, win_y0 = d.crop_y0;
    uint32_t win_flip = d.flip;
    L3_KEEP_SGPR(out_base);
    L3_KEEP_SGPR(out_row_stride);
    L3_KEEP_SGPR(out_plane_stride);
    L3_KEEP_SGPR(img_width);
    L3_KEEP_SGPR(win_x0);
    L3_KEEP_SGPR(win_y0);
    L3_KEEP_SGPR(win_flip);
    /* lane l takes the 4-pixel words l, l + 64, ... of the wave's strip; how many of
     * their pixels exist does not change from row to row */
    uint32_t word_x[NW], word_valid[NW], word_off[NW];
#pragma unroll
    for (int pass = 0; pass < NW; ++pass) {
        /* in flat order (NW = 1) the word is the lane's own four pixels; a group that
         * only shadows the block's last patch writes nothing */
        word_x[pass] = flat_order ? x0 + 4 * xl : strip_x0 + 4 * (lane + 64 * pass);
        word_valid[pass] = (word_x[pass] >= img_width || (flat_order && !active)) ? 0u : min(4u, img_width - word_x[pass]);
        /* byte offset of the word from the start of the output row that the unit's
         * first patch row writes: column bytes, plus the rows by which this group's
         * patch row lies below it (flat order; the host checked that this fits 32 bits) */
        word_off[pass] = (MODE == L3_MODE_HWC ? 3u : 1u) * word_x[pass] +
                         (ty - ty_base) * (uint32_t)N * (uint32_t)out_row_stride;
    }
    /* tensor mode: whether the word's 4 pixels all lie inside the window, and the byte offset
     * of its 4 elements in a row of the window (mirrored or not): the same for every row */
    bool tensor_whole[NW];
    uint32_t tensor_at[NW];
#pragma unroll
    for (int pass = 0; pass < NW; ++pass) {
        const int32_t col0 = (int32_t)word_x[pass] - win_x0;
        tensor_whole[pass] = MODE == L3_MODE_TENSOR && word_valid[pass] == 4 && col0 >= 0 &&
                             col0 + 4 <= (int32_t)crop_w;
        tensor_at[pass] = 2u * (uint32_t)(win_flip ? (int32_t)crop_w - 4 - col0 : col0);
    }

    /* After the workgroup barrier: this wave writes row c of the period whose rows
     * are parked in buffer `buf` (rows first .. first+count-1 of the patch).  Lane l
     * takes the 4-pixel words l, l + 64, ... of the wave's strip: 12 contiguous
     * output bytes each, contiguous over the lanes. */
    auto flush = [&](uint32_t buf, uint32_t first, uint32_t count) {
        if (c >= count) return;
        const uint32_t y = y0 + first + c;
#pragma unroll
        for (int pass = 0; pass < NW; ++pass) {
            const uint32_t q = lane + 64 * pass;
            const uint32_t x = word_x[pass];                           /* image column of the word */
            const uint32_t nvalid = word_valid[pass];
            const uint32_t* src = &parked[buf][c][0][0];
            /* interleaved mode: 12 bytes R0 G0 B0 R1 G1 B1 R2 G2 B2 R3 G3 B3 per word q;
             * planar modes: one word of 4 pixels per channel */
            const uint32_t pr = MODE == L3_MODE_HWC ? src[3 * q] : src[q];
            const uint32_t pg = MODE == L3_MODE_HWC ? src[3 * q + 1] : src[QW + q];
            const uint32_t pb = MODE == L3_MODE_HWC ? src[3 * q + 2] : src[2 * QW + q];
            if (MODE == L3_MODE_HWC) {
                /* row start: scalar arithmetic; the lane's 32-bit column offset goes into the
                 * store's offset register (kept opaque here so that it is not widened and
                 * added with vector instructions ahead of time) */
                uint32_t column = word_off[pass];
                L3_KEEP_VGPR(column);
                global_u8* row = reinterpret_cast<global_u8*>((uintptr_t)(out_base + (uint64_t)y * out_row_stride));
                const uint32_t o0 = pr, o1 = pg, o2 = pb;
                if (nvalid == 4) {
                    const u32x3 v = {o0, o1, o2};
                    __builtin_nontemporal_store(v, reinterpret_cast<global_u32x3_any*>(row + column));
                } else if (nvalid) {
                    /* the last word of an image row: 3, 6 or 9 bytes in two stores */
                    global_u8* b = row + column;
                    if (nvalid == 3) {
                        const u32x2 v = {o0, o1};
                        *reinterpret_cast<global_u32x2_any*>(b) = v;
                        b[8] = (uint8_t)o2;
                    } else if (nvalid == 2) {
                        *reinterpret_cast<global_u32_any*>(b) = o0;
                        *reinterpret_cast<global_u16_any*>(b + 4) = (uint16_t)o1;
                    } else {
                        *reinterpret_cast<global_u16_any*>(b) = (uint16_t)o0;
                        b[2] = (uint8_t)(o0 >> 16);
                    }
                }
            } else if (MODE == L3_MODE_CHW) {
#pragma unroll
                for (int ch = 0; ch < 3; ++ch) {
                    const uint32_t word = ch == 0 ? pr : (ch == 1 ? pg : pb);
                    global_u8* row = reinterpret_cast<global_u8*>(
                        (uintptr_t)(out_base + (uint64_t)ch * out_plane_stride + (uint64_t)y * out_row_stride));
                    uint32_t column = word_off[pass];
                    L3_KEEP_VGPR(column);
                    if (nvalid == 4) {
                        __builtin_nontemporal_store(word, reinterpret_cast<global_u32_any*>(row + column));
                    } else if (nvalid) {
                        global_u8* b = row + column;
#pragma unroll
                        for (int k = 0; k < 3; ++k)
                            if ((uint32_t)k < nvalid) b[k] = (uint8_t)(word >> (8 * k));
                    }
                }
            } else {
                /* tensor mode: window test, optional mirror, table of the 256 normalised
                 * values.  A word whose 4 pixels all lie inside the window is written as 4
                 * elements (8 bytes) per channel at once, mirrored or not; words on the
                 * window's edge go element by element. */
                const int32_t row = (int32_t)y - win_y0;
                if (row >= 0 && row < (int32_t)crop_h && nvalid) {
                    /* all twelve table reads first, so that they travel together */
                    uint16_t e[3][4];
#pragma unroll
                    for (int ch = 0; ch < 3; ++ch) {
                        const uint32_t word = ch == 0 ? pr : (ch == 1 ? pg : pb);
#pragma unroll
                        for (int k = 0; k < 4; ++k) e[ch][k] = s_lut[ch * 256 + ((word >> (8 * k)) & 0xFFu)];
                    }
                    /* element (ch, row, 0) of this image; planes are crop_h * crop_w apart: the
                     * planes' rows start at scalar addresses, the lane adds its byte offset */
                    const size_t plane = (size_t)crop_h * crop_w;
                    if (tensor_whole[pass]) {
                        if (win_flip) {        /* the same for the whole image: elements 3 2 | 1 0 */
#pragma unroll
                            for (int ch = 0; ch < 3; ++ch) {
                                uint64_t line_at = out_base + 2 * ((uint64_t)row * crop_w + ch * plane);
                                L3_KEEP_SGPR(line_at);
                                global_u8* line = reinterpret_cast<global_u8*>((uintptr_t)line_at);
                                uint32_t at = tensor_at[pass];
                                L3_KEEP_VGPR(at);      /* stays the store's 32-bit offset */
                                const u16x2 lo = {e[ch][3], e[ch][2]}, hi = {e[ch][1], e[ch][0]};
                                const u32x2 v = {__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
                                __builtin_nontemporal_store(v, reinterpret_cast<global_u32x2_any*>(line + at));
                            }
                        } else {
#pragma unroll
                            for (int ch = 0; ch < 3; ++ch) {
                                uint64_t line_at = out_base + 2 * ((uint64_t)row * crop_w + ch * plane);
                                L3_KEEP_SGPR(line_at);
                                global_u8* line = reinterpret_cast<global_u8*>((uintptr_t)line_at);
                                uint32_t at = tensor_at[pass];
                                L3_KEEP_VGPR(at);      /* stays the store's 32-bit offset */
                                const u16x2 lo = {e[ch][0], e[ch][1]}, hi = {e[ch][2], e[ch][3]};
                                const u32x2 v = {__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
                                __builtin_nontemporal_store(v, reinterpret_cast<global_u32x2_any*>(line + at));
                            }
                        }
                    } else {
                        const int32_t col0 = (int32_t)x - win_x0;   /* window column of pixel 0 */
                        global_u16* line = reinterpret_cast<global_u16*>((uintptr_t)out_base) + (size_t)row * crop_w;
#pragma unroll
                        for (int ch = 0; ch < 3; ++ch) {
                            global_u16* out16 = line + ch * plane;
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                int32_t col = col0 + k;
                                if ((uint32_t)k < nvalid && col >= 0 && col < (int32_t)crop_w) {
                                    if (win_flip) col = (int32_t)crop_w - 1 - col;
                                    out16[col] = e[ch][k];
                                }
                            }
                        }
                    }
                }
            }
        }
    };

    uint32_t prev[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) prev[j] = 0;   /* an all-zero row above predicts 0: row 0 is raw */
    open_row(ring_fetch(ring_where<RING>(ring_lds, bitpos)));

    /* One row: no branch inside.  The deltas of the row and the record of the next
     * row travel from LDS while part 1 is computed; after the last row the record
     * read does not exist, which is harmless.  `park` is where this lane parks its
     * NW words (p0 p1 p2 p3 each). */
    auto do_row = [&](uint32_t* park, uint32_t y) {
        RingWords xw[NW];
#pragma unroll
        for (int k = 0; k < NW; ++k) xw[k] = ring_fetch(xwhere[k]);
        const RingWords hdr_next = ring_fetch(hwhere);
        __builtin_amdgcn_sched_barrier(0);

        /* inverse filter, part 1: the prediction depends only on the row above
         * (registers + lane neighbours) */
        const uint32_t from_left = dpp_from_lower_lane(prev[NP - 1]);   /* pixels (PPL-3, PPL-1) of the lane below */
        const uint32_t from_right = dpp_from_upper_lane(prev[0]);       /* pixels (0, 2) of the lane above */
        uint32_t TL[NP], TR[NP], pred[NP];
#pragma unroll
        for (int k = 0; k < NW; ++k) {
            const uint32_t E = prev[2 * k], O = prev[2 * k + 1];
            /* pixels (4k, 4k+2): top-left = (4k-1, 4k+1), top-right = (4k+1, 4k+3) */
            TL[2 * k] = __builtin_amdgcn_alignbit(O, k > 0 ? prev[2 * k - 1] : from_left, 16);
            TR[2 * k] = O;
            /* pixels (4k+1, 4k+3): top-left = (4k, 4k+2), top-right = (4k+2, 4k+4) */
            TL[2 * k + 1] = E;
            TR[2 * k + 1] = __builtin_amdgcn_alignbit(k < NW - 1 ? prev[2 * k + 2] : from_right, E, 16);
        }
        predict_pairs<NP>(TL, TR, prev, border, pred);
        __builtin_amdgcn_sched_barrier(0);

        /* base-delta: value = base + delta; part 2 of the filter: pixel = prediction
         * + value (both mod 256, one mask at the end) */
        wmax = max(wmax, w);
        uint32_t word[NW];
#pragma unroll
        for (int k = 0; k < NW; ++k) {
            /* The lane's four deltas d0..d3 sit in the low 4w bits of x.  Y holds the two
             * halves of that field in its 16-bit halves: (d0 | d1 << w, d2 | d3 << w).  A
             * packed shift by w leaves (d1, d3); taking that, times 2^w, off Y leaves
             * (d0, d2): K = -(2^w) mod 2^16 turns it into one packed multiply-add. */
            const uint32_t x = ring_align(xw[k], xbit[k]);
            const uint32_t f01 = __builtin_amdgcn_ubfe(x, 0, w2);
            const uint32_t f23 = __builtin_amdgcn_ubfe(x, w2, w2);
            const uint32_t Y = f01 | (f23 << 16);
            const uint32_t B = pk_lshr_b16_by_low(w, Y);
            const uint32_t A = pk_mad_u16_by_low(B, K, Y);   /* before the 32-bit sums: Y's halves are full */
            prev[2 * k] = (A + pred[2 * k] + base2) & 0x00FF00FFu;
            prev[2 * k + 1] = (B + pred[2 * k + 1] + base2) & 0x00FF00FFu;
            if (MODE != L3_MODE_HWC)
                word[k] = __builtin_amdgcn_perm(prev[2 * k + 1], prev[2 * k], 0x06020400u);   /* p0 p1 p2 p3 */
        }
        if (MODE == L3_MODE_HWC) {
            /* interleave through LDS byte writes (no vector-ALU work): channel c of
             * pixel i of word k goes to byte 12k + 3i + c of the lane's 12 NW bytes */
            uint8_t* pb = reinterpret_cast<uint8_t*>(park);
#pragma unroll
            for (int k = 0; k < NW; ++k) {
                pb[12 * k + 0] = (uint8_t)prev[2 * k];
                pb[12 * k + 3] = (uint8_t)prev[2 * k + 1];
                pb[12 * k + 6] = (uint8_t)(prev[2 * k] >> 16);
                pb[12 * k + 9] = (uint8_t)(prev[2 * k + 1] >> 16);
            }
        } else if (DIRECT) {
            global_u8* row = reinterpret_cast<global_u8*>(
                (uintptr_t)(out_base + (uint64_t)c * out_plane_stride + (uint64_t)y * out_row_stride));
            uint32_t column = word_off[0];
            L3_KEEP_VGPR(column);
            if (word_valid[0] == 4) {
                __builtin_nontemporal_store(word[0], reinterpret_cast<global_u32_any*>(row + column));
            } else if (word_valid[0]) {
                global_u8* b = row + column;
#pragma unroll
                for (int k = 0; k < 3; ++k)
                    if ((uint32_t)k < word_valid[0]) b[k] = (uint8_t)(word[0] >> (8 * k));
            }
        } else {
#pragma unroll
            for (int k = 0; k < NW; ++k) park[k] = word[k];
        }

        __builtin_amdgcn_sched_barrier(0);
        open_row(hdr_next);
    };

    /* Waves that are ahead yield to waves that are behind (the hardware otherwise
     * favours the oldest wave, and the youngest ones would finish the kernel alone):
     * the wave's issue priority drops by one in each quarter of its rows.  Among waves of
     * equal priority the oldest still wins, so an older workgroup drops a little sooner
     * than a younger one: after (8 k + age_rank) / 32 of its rows, k = 1, 2, 3, where
     * age_rank is 0 for the oldest of the (up to eight) workgroups of a CU and 7 for the
     * youngest.  That is for the workgroups that are resident when the launch ends.  A
     * launch of several rounds of workgroups leaves the earlier ones at the top priority
     * (keeps_priority): with the hardware's preference for the oldest wave they end one
     * after the other instead of together, so their successors do not all wait for their
     * first chunks at the same time. */
    const uint32_t drop_at[3] = {keeps_priority ? 0x7FFFFFFFu : (ph * (8u + age_rank) + 31u) / 32u,
                                 (ph * (16u + age_rank) + 31u) / 32u, (ph * (24u + age_rank) + 31u) / 32u};
    uint32_t next_drop = drop_at[0], stage = 0;
    __builtin_amdgcn_s_setprio(3);

    /* Periods of P = 3 rows, unrolled so that the row's place in the period is a
     * constant: the workgroup barrier and the write-out of the previous period, rows 0
     * and 1, the ring top-up, row 2.  Only the last period can be shorter.
     * With LATE_BARRIER the barrier and the write-out come behind row 0, so that a wave
     * that arrives early has a row to do before it waits.  Three parking buffers in turn
     * make that safe: a wave that parks period k has passed the barrier of period k-1,
     * which every wave reaches only after it has written out period k-3, the previous
     * tenant of the buffer.  (With two buffers a wave could still be writing out period
     * k-2 when an early one starts to park period k.) */
    uint32_t buf = 0, prev_buf = 0;
    /* see the ring top-up: the bit position up to which the record of the next period may
     * lie before this lane's stream must take its next chunk, 8 * (fill - AHEAD - 16 xl) */
    uint32_t reach = (fill - (G::AHEAD + xl * 16)) * 8;
    for (uint32_t r = 0; r < ph; r += P) {
        const uint32_t rows = min((uint32_t)P, ph - r);
        if (r >= next_drop) {
            ++stage;
            next_drop = stage == 1 ? drop_at[1] : (stage == 2 ? drop_at[2] : 0x7FFFFFFFu);
            if (stage == 1) __builtin_amdgcn_s_setprio(2);
            else if (stage == 2) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        if (!DIRECT && !LATE_BARRIER && r > 0) {
            /* all three channels of the previous period are parked: write them out */
            __syncthreads();
            flush(prev_buf, r - P, P);
        }
        /* interleaved mode: this lane's 12 NW bytes of the row, channel c first at byte c;
         * planar modes: this lane's NW words of channel c */
        uint32_t* park = MODE == L3_MODE_HWC
                             ? reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(&parked[buf][0][0][0]) +
                                                           lane * (12 * NW) + c)
                             : &parked[buf][0][c][lane * NW];
        do_row(park, y0 + r);
        if (!DIRECT && LATE_BARRIER && r > 0) {
            __syncthreads();
            flush(prev_buf, r - P, P);
        }
        if (rows > 1) do_row(park + 3 * QW, y0 + r + 1);
        if (rows > 2) {
            if (r + P < ph) {
                /* top the ring up for rows r+3 .. r+5; bitpos is the record of row r+3.  `fill`
                 * counts this lane's own first granule of the chunk held in pf (the stream's
                 * fill level plus 16 bytes per lane of the group), so that ring place and load
                 * address follow from it directly.  A chunk is half the ring and starts at a
                 * multiple of its size, so its granules never wrap inside one refill: the
                 * lane's second granule sits CHUNK / 2 behind its first, in the ring and in
                 * the stream.  What pf holds beyond the stream's last granule is left as it
                 * was: nothing that is decoded reads it. */
                /* A stream must be topped up once its fill level is less than AHEAD beyond the
                 * record of row r+3 (bitpos beyond `reach`; the comparison in bits asks for it
                 * up to 7 bits sooner than one in bytes would), and may be up to EARLY bytes
                 * sooner (the chunk then still lands behind everything that is unread; one
                 * byte of that is given away to the comparison in bits).  When any stream of
                 * the wave must, all that may do: the streams of a wave then take their chunks
                 * in the same periods instead of each in its own, and the other periods skip
                 * all this.  The first period instead asks for the chunk behind the first one:
                 * its top-up is never due (the first chunk reaches AHEAD beyond the record of
                 * row 3 from any start alignment, see Geom). */
                if (r == 0) {
#pragma unroll
                    for (int t = 0; t < GPL; ++t) pf[t] = load_granule(origin, CHUNK + (t * LPT + xl) * 16, limit);
                } else if (wave_any(reach < bitpos) && reach < bitpos + 8 * (G::EARLY - 1)) {
                    const uint32_t idx = fill & (RING - 1);
                    uint8_t* at = reinterpret_cast<uint8_t*>(ring) + idx;
                    *reinterpret_cast<u32x4*>(at) = pf[0];
                    *reinterpret_cast<u32x4*>(at + CHUNK / 2) = pf[1];
                    if (idx == 0) *reinterpret_cast<u32x4*>(at + RING) = pf[0];
                    fill += CHUNK;
                    reach += 8 * CHUNK;
                    if (fill < limit)
                        pf[0] = *reinterpret_cast<global_const_u32x4*>((uintptr_t)(origin + fill));
                    if (fill + CHUNK / 2 < limit)
                        pf[1] = *reinterpret_cast<global_const_u32x4*>((uintptr_t)(origin + fill + CHUNK / 2));
                }
                wave_lds_fence();
            }
            do_row(park + 2 * 3 * QW, y0 + r + 2);
        }
        prev_buf = buf;
        buf = buf == PARKS - 1 ? 0u : buf + 1u;
    }
    if (!DIRECT) {
        const uint32_t first = ((ph - 1) / P) * P;
        __syncthreads();
        flush(prev_buf, first, ph - first);
    }

    if (wmax > 8) flags |= L3_STATUS_BAD_WIDTH;
    /* bitpos is one (non-existent) row past the end: step back over it */
    if (bitpos - 12 - pw * w > endbit) flags |= L3_STATUS_OVERRUN;
    if (flags && active && status) atomicOr(&status[d.status_index], flags);
}

/* How old a workgroup of the launch's last round is among the workgroups of its CU, 0 (oldest)
 * to 7: workgroups are handed out in the order of their numbers, to the XCDs in turn and inside
 * an XCD to its 32 CUs in turn, so the n-th workgroup of an XCD is about the (n / 32)-th of
 * its CU.  Only steers issue priorities. */
__device__ __forceinline__ uint32_t age_rank_of(uint32_t top_priority_below) {
    const uint32_t nth = (blockIdx.x - min(blockIdx.x, top_priority_below)) >> 3;
    return min(7u, nth / 32u);
}

/* Where a fused kernel reads its table: in device memory if the call gave one, else in its
 * own arguments (the argument segment is ordinary device memory). */
template <int MODE>
__device__ __forceinline__ const uint16_t* table_of(const uint16_t* lut, const L3NoTable&) { return lut; }
template <int MODE>
__device__ __forceinline__ const uint16_t* table_of(const uint16_t* lut, const L3Table& tail) {
    return lut ? lut : tail.bits;
}

/* Descriptors in a device table (any batch size)... */
template <int N, int PPL, int MODE>
__global__ __launch_bounds__(kBlockThreads) void l3_decode_kernel(
    const L3ImageDesc* __restrict__ descs, uint32_t units_per_image, uint32_t images,
    uint32_t* __restrict__ status, uint32_t crop_w, uint32_t crop_h, uint32_t top_priority_below,
    const uint16_t* __restrict__ lut, const typename TailFor<MODE>::type tail) {
    uint32_t image, unit;
    if (!take_work(units_per_image, images, image, unit)) return;
    decode_unit<N, PPL, MODE>(descs[image], unit, status, crop_w, crop_h, blockIdx.x < top_priority_below,
                              age_rank_of(top_priority_below), table_of<MODE>(lut, tail));
}

/* ...or inside the kernel arguments: no upload, no dependency on a copy, so consecutive
 * calls run back to back.  Two capacities, so that small batches do not carry a large
 * argument block (the runtime accepts argument blocks of at least 64 KB). */
constexpr int kArgDescsSmall = 32, kArgDescs = 256;
template <int CAP>
struct DescPack { L3ImageDesc d[CAP]; };
static_assert(sizeof(DescPack<kArgDescs>) + sizeof(L3Table) + 64 <= 32768, "kernel argument segment");

template <int N, int PPL, int MODE, int CAP>
__global__ __launch_bounds__(kBlockThreads) void l3_decode_kernel_args(
    const DescPack<CAP> pack, uint32_t units_per_image, uint32_t images, uint32_t* __restrict__ status,
    uint32_t crop_w, uint32_t crop_h, uint32_t top_priority_below, const uint16_t* __restrict__ lut,
    const typename TailFor<MODE>::type tail) {
    uint32_t image, unit;
    if (!take_work(units_per_image, images, image, unit)) return;
    decode_unit<N, PPL, MODE>(pack.d[image], unit, status, crop_w, crop_h, blockIdx.x < top_priority_below,
                              age_rank_of(top_priority_below), table_of<MODE>(lut, tail));
}

/* The table in device memory, for the call that keeps one there. */
__global__ void l3_build_table_kernel(float m0, float m1, float m2, float s0, float s1, float s2,
                                      int dtype, uint16_t* __restrict__ table) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= 768) return;
    const uint32_t c = i >> 8;
    const float mean = c == 0 ? m0 : (c == 1 ? m1 : m2);
    const float stdv = c == 0 ? s0 : (c == 1 ? s1 : s2);
    table[i] = normalised_bits(i & 255u, mean, stdv, dtype);
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

/* The table of normalised values of l3_decode_crop_normalize_batch_noalloc: memory that exists
 * from the moment the library is loaded, one copy per GPU, so that the call itself allocates
 * nothing.  Host code never uses this name as an address: l3_ctx_create asks the runtime for the
 * address of the current device's copy once and keeps it (static_table_of). */
constexpr int kStaticTableEntries = 768;
static __device__ __align__(256) uint16_t scratch[kStaticTableEntries];

/* ---- host side: context, planning, launch ------------------------------- */

constexpr int kMaxDevices = 64;
std::mutex g_static_table_mutex;
uint16_t* g_static_table[kMaxDevices] = {};

/* Address of the current device's copy of `scratch`; asked for once per device, with that
 * device current.  NULL if the runtime refuses. */
uint16_t* static_table_of(int device) {
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_static_table_mutex);
    if (!g_static_table[device]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        g_static_table[device] = static_cast<uint16_t*>(ptr);
    }
    return g_static_table[device];
}


/* The kernels are launched through argument arrays (hipLaunchKernel): the fused ones take one
 * argument more than the others, the table. */
typedef const void* decode_kernel_t;
typedef const void* decode_kernel_args_small_t;
typedef const void* decode_kernel_args_t;

struct KernelChoice {
    decode_kernel_t table;        /* descriptors in a device table */
    decode_kernel_args_small_t args_small;   /* descriptors in the kernel arguments, up to 32 */
    decode_kernel_args_t args;               /* up to 256 */
    int tiles_per_wave;
};

template <int N, int PPL>
KernelChoice choice_for_mode(int mode) {
    KernelChoice k;
    k.tiles_per_wave = Geom<N, PPL>::TPW;
    switch (mode) {
        case L3_MODE_HWC:
            k.table = reinterpret_cast<const void*>(&l3_decode_kernel<N, PPL, L3_MODE_HWC>);
            k.args_small = reinterpret_cast<const void*>(&l3_decode_kernel_args<N, PPL, L3_MODE_HWC, kArgDescsSmall>);
            k.args = reinterpret_cast<const void*>(&l3_decode_kernel_args<N, PPL, L3_MODE_HWC, kArgDescs>);
            break;
        case L3_MODE_CHW:
            k.table = reinterpret_cast<const void*>(&l3_decode_kernel<N, PPL, L3_MODE_CHW>);
            k.args_small = reinterpret_cast<const void*>(&l3_decode_kernel_args<N, PPL, L3_MODE_CHW, kArgDescsSmall>);
            k.args = reinterpret_cast<const void*>(&l3_decode_kernel_args<N, PPL, L3_MODE_CHW, kArgDescs>);
            break;
        default:
            k.table = reinterpret_cast<const void*>(&l3_decode_kernel<N, PPL, L3_MODE_TENSOR>);
            k.args_small = reinterpret_cast<const void*>(&l3_decode_kernel_args<N, PPL, L3_MODE_TENSOR, kArgDescsSmall>);
            k.args = reinterpret_cast<const void*>(&l3_decode_kernel_args<N, PPL, L3_MODE_TENSOR, kArgDescs>);
            break;
    }
    return k;
}

/* The kernels are written for NW = PPL / 4 words of four pixels per lane; the library is
 * built with PPL = 4 (one word): 8 pixels per lane issue 12 % fewer vector instructions but
 * halve the number of waves, and measured slower on every workload. */
constexpr int kPixelsPerLane = 4;

KernelChoice pick_kernel(int n, int mode) {
    if (n == 32) return choice_for_mode<32, kPixelsPerLane>(mode);
    if (n == 64) return choice_for_mode<64, kPixelsPerLane>(mode);
    return choice_for_mode<128, kPixelsPerLane>(mode);
}

}  // namespace

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
                    int dtype, void* d_out_tensor, uint32_t* d_status, void* stream_v,
                    bool no_alloc = false) {
    if (!ctx || n < 0 || (n > 0 && !items)) return L3_ERR_INVALID_ARG;
    if (n == 0) return L3_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);

    DeviceGuard guard(ctx->device);
    if (!guard.ok) return L3_ERR_DEVICE;
    l3_status st = L3_OK;
    if (no_alloc && (size_t)n > ctx->scratch_cap) return L3_ERR_LIMIT;   /* cannot happen: n <= 256 */
    if ((size_t)n > ctx->scratch_cap) {
        size_t cap = 256;
        while (cap < (size_t)n) cap *= 2;
        /* kArgDescs spare entries: a launch may read a whole argument block from any descriptor on */
        L3ImageDesc* grown = static_cast<L3ImageDesc*>(
            std::realloc(ctx->scratch, (cap + kArgDescs) * sizeof(L3ImageDesc)));
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
        const int tpw = pick_kernel(kClasses[k], mode).tiles_per_wave;
        const bool flat_ok = ctx->flat_order;
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
                l3_plan_units(d, np, (uint32_t)tpw, flat_ok);
            }
            if (d->units > max_units[k]) max_units[k] = d->units;
        }
    }
    class_begin[3] = filled;

    /* Small batches travel inside the kernel arguments; larger ones through a device
     * table that a small kernel on the caller's stream pulls from pinned host memory. */
    bool in_args = true;
    for (int k = 0; k < 3; ++k) {
        const uint64_t count = (uint64_t)(class_begin[k + 1] - class_begin[k]);
        if (count > (uint64_t)kArgDescs || count * max_units[k] > 0x7FFFFF00ull) in_args = false;
    }

    if (no_alloc && !in_args) return L3_ERR_LIMIT;
    int slot = -1;
    L3ImageDesc* d_descs = nullptr;
    if (!in_args) {
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
    /* The table of normalised values travels inside the arguments of the fused kernels: the
     * host works it out (and remembers the last one), so a call depends on no table in device
     * memory and on no kernel ahead of it, and records the same work under stream capture as
     * outside it.  Only the call that allocates nothing keeps its table in device memory (the
     * library's static one, rebuilt by a small kernel ahead of every launch). */
    const uint16_t* table = nullptr;
    L3NoTable no_tail;
    void* tail = &no_tail;
    if (mode == L3_MODE_TENSOR) {
        if (no_alloc) {
            hipLaunchKernelGGL(l3_build_table_kernel, dim3(3), dim3(256), 0, stream, mean[0], mean[1],
                               mean[2], stdv[0], stdv[1], stdv[2], dtype, ctx->static_table);
            table = ctx->static_table;
        } else {
            const float key[7] = {mean[0], mean[1], mean[2], stdv[0], stdv[1], stdv[2], (float)dtype};
            if (!ctx->table_valid || std::memcmp(ctx->table_key, key, sizeof key) != 0) {
                if (l3_normalized_values(mean, stdv, (l3_dtype)dtype, ctx->table_bits) != L3_OK)
                    return L3_ERR_INVALID_ARG;
                std::memcpy(ctx->table_key, key, sizeof key);
                ctx->table_valid = true;
            }
        }
        static_assert(sizeof(L3Table) == sizeof ctx->table_bits, "the context's copy is the argument");
        tail = ctx->table_bits;
    }
    for (int k = 0; k < 3; ++k) {
        const int count = class_begin[k + 1] - class_begin[k];
        if (count == 0 || max_units[k] == 0) continue;
        const uint32_t gx = max_units[k];
        /* one-dimensional grid, rounded up to a multiple of 8 (see take_work) */
        const auto grid_for = [gx](uint64_t images) { return (uint32_t)((gx * images + 7) / 8 * 8); };
        uint32_t gx_arg = gx;
        /* the workgroups ahead of the launch's last round (see decode_unit's priorities) */
        const uint32_t last_round = ctx->resident_workgroups;
        const auto top_below = [last_round](uint32_t grid) { return grid > last_round ? grid - last_round : 0u; };
        if (in_args && count <= kArgDescsSmall) {
            DescPack<kArgDescsSmall> pack;
            std::memcpy(pack.d, stage + class_begin[k], (size_t)count * sizeof(L3ImageDesc));
            uint32_t count_arg = (uint32_t)count;
            uint32_t top_arg = top_below(grid_for((uint64_t)count));
            void* kernel_args[9] = {&pack, &gx_arg, &count_arg, &d_status, &crop_w, &crop_h, &top_arg, &table, tail};
            if (hipLaunchKernel(pick_kernel(kClasses[k], mode).args_small, dim3(grid_for((uint64_t)count)),
                                dim3(kBlockThreads), kernel_args, 0, stream) != hipSuccess)
                return L3_ERR_DEVICE;
            continue;
        }
        if (in_args) {
            /* 28 KB of arguments: handed over by address, straight from the staging array
             * (which has kArgDescs spare entries behind the last descriptor), so that the
             * block is copied once, by the launch, and never sits on the stack */
            uint32_t count_arg = (uint32_t)count;
            uint32_t top_arg = top_below(grid_for((uint64_t)count));
            void* kernel_args[9] = {stage + class_begin[k], &gx_arg, &count_arg, &d_status,
                                    &crop_w, &crop_h, &top_arg, &table, tail};
            if (hipLaunchKernel(pick_kernel(kClasses[k], mode).args, dim3(grid_for((uint64_t)count)),
                                dim3(kBlockThreads), kernel_args, 0, stream) != hipSuccess)
                return L3_ERR_DEVICE;
            continue;
        }
        decode_kernel_t kern = pick_kernel(kClasses[k], mode).table;
        if (gx > 0x7FFFFF00u) return L3_ERR_UNSUPPORTED;     /* more units in one image than a grid holds */
        const int per_launch = (int)std::min<uint64_t>((uint64_t)count, 0x7FFFFF00ull / gx);
        for (int first = 0; first < count; first += per_launch) {
            const int m = count - first < per_launch ? count - first : per_launch;
            const L3ImageDesc* first_desc = d_descs + class_begin[k] + first;
            uint32_t m_arg = (uint32_t)m;
            uint32_t top_arg = top_below(grid_for((uint64_t)m));
            void* kernel_args[9] = {&first_desc, &gx_arg, &m_arg, &d_status, &crop_w, &crop_h, &top_arg, &table, tail};
            if (hipLaunchKernel(kern, dim3(grid_for((uint64_t)m)), dim3(kBlockThreads), kernel_args, 0,
                                stream) != hipSuccess)
                return L3_ERR_DEVICE;
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
    {
        /* L3_FLAT_ORDER=0 in the environment at creation keeps every image on the per-row order
         * of work units (for comparisons; the flat order is never slower in measurements) */
        const char* e = std::getenv("L3_FLAT_ORDER");
        ctx->flat_order = !(e && e[0] == '0' && e[1] == 0);
    }
    ctx->static_table = static_table_of(device);
    {
        /* how many workgroups the launch's last round holds: eight per CU (what the local
         * memory of the smallest-patch kernels allows; the others hold one or two more, which
         * makes no difference to what the number is used for) */
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0)
            cus = 256;
        ctx->resident_workgroups = 8u * (uint32_t)cus;
    }
    /* host staging for up to three full argument blocks, so that batches of that size never
     * make a call allocate */
    ctx->scratch_cap = 3 * kArgDescs;
    ctx->scratch = static_cast<L3ImageDesc*>(std::malloc((ctx->scratch_cap + kArgDescs) * sizeof(L3ImageDesc)));
    bool ok = ctx->static_table && ctx->scratch;
    for (int s = 0; s < kSlots && ok; ++s)
        ok = hipEventCreateWithFlags(&ctx->done[s], hipEventDisableTiming) == hipSuccess;
    if (!ok) {
        l3_ctx_destroy(ctx);
        return L3_ERR_DEVICE;
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
    }
    release_slots(ctx);
    std::free(ctx->scratch);
    l3_encode_state_free(ctx->enc);
    l3_ablation_state_free(ctx->abl);
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

l3_status l3_decode_crop_normalize_batch_noalloc(l3_ctx* ctx, const l3_item* items,
                                                 const l3_crop* crops, int n, uint32_t crop_w,
                                                 uint32_t crop_h, const float mean[3],
                                                 const float stdv[3], l3_dtype dtype,
                                                 void* d_out_nchw, uint32_t* d_status, void* stream) {
    if (n > L3_NOALLOC_MAX_IMAGES) return L3_ERR_LIMIT;
    if (n > 0 && (!crops || !mean || !stdv || !d_out_nchw || crop_w == 0 || crop_h == 0))
        return L3_ERR_INVALID_ARG;
    if (dtype != L3_BF16 && dtype != L3_FP16) return L3_ERR_INVALID_ARG;
    if (n > 0 && (stdv[0] == 0.0f || stdv[1] == 0.0f || stdv[2] == 0.0f)) return L3_ERR_INVALID_ARG;
    return run_batch(ctx, items, crops, n, L3_MODE_TENSOR, crop_w, crop_h, mean, stdv, (int)dtype,
                     d_out_nchw, d_status, stream, true);
}

}  // extern "C"
