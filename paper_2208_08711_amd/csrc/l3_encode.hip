/*
 * gfx950 encoder of the L3 format: interleaved 8-bit RGB in device memory ->
 * L3 files in device memory, byte for byte what l3_encode_cpu produces.
 *
 * arxiv 2208.08711, Section 4.2, encoding direction: per patch and channel, the
 * custom Paeth filter (rows after the first: pixel minus the nearest of the three
 * upper neighbours to TL + TR - T, taken from the ORIGINAL row above, so every
 * pixel of the patch is independent), then row-wise base-delta (row minimum as
 * base, minimal width, deltas packed).  Section 4.3: patches concatenated, their
 * offsets recorded in three arrays behind a 13-byte header.
 *
 * Patch sizes 32, 64 and 128 (the ones the paper's rule picks) take three kernels:
 *   strip    a workgroup of three waves (one per channel) owns a strip of adjacent
 *            patches, 4 pixels per lane as two packed pairs of 16-bit fields: per
 *            row it filters, reduces min and max over the patch's lanes, packs the
 *            deltas with LDS atomic OR into a small ring per patch and streams the
 *            finished 16-byte granules to a fixed-size slot of a workspace; the
 *            patch's byte size goes to a table;
 *   layout   one workgroup per image: exclusive prefix sum of the patch sizes ->
 *            header, offset arrays, file length (this is where a scan belongs: the
 *            addends are all known);
 *   compact  copies every slot to its place in the file.
 * Any other patch size up to 128 takes the plain route: measure (one wave per patch
 * and channel walks the rows for the sizes), layout, pack (walks them again and
 * writes the bits).  The forward filter needs no row recurrence: the row above is
 * the original one, kept in registers, with lane shifts for the neighbours.
 */
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>
#include <new>

#include "l3_ctx.h"
#include "l3_gfx950.h"
#include "l3_kernel_parts.h"

namespace {

constexpr int kMaxPatch = 128;                       /* two pixels per lane */

struct L3EncodeDesc {
    const uint8_t* rgb;
    uint8_t* file;
    uint64_t row_stride;
    uint64_t file_cap;
    uint32_t width, height;
    uint32_t tiles_x, tiles_y;
    uint32_t patch;
    uint32_t sizes_base;     /* first entry of this image in the sizes scratch */
    uint32_t status_index;
    uint32_t strips_x;       /* strip route: wave strips per patch row */
    uint64_t slots_base;     /* strip route: byte offset of this image's first slot in the workspace */
};

typedef __attribute__((address_space(1))) uint32_t global_u32_unaligned __attribute__((aligned(1)));

__device__ __forceinline__ int nearest_upper(int tl, int t, int tr) {
    /* distances to TL + TR - T: |TR - T| for TL, |TL - T| for TR, |TL + TR - 2T| for T;
     * ties: TL, then TR, then T */
    const int d_tl = abs(tr - t), d_tr = abs(tl - t), d_t = abs(tl + tr - 2 * t);
    if (d_tl <= d_tr && d_tl <= d_t) return tl;
    return d_tr <= d_t ? tr : t;
}

__device__ __forceinline__ int wave_min(int v) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v = min(v, __shfl_xor(v, s));
    return v;
}
__device__ __forceinline__ int wave_max(int v) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v = max(v, __shfl_xor(v, s));
    return v;
}

/* Walks the rows of patch (c, ty, tx).  PACK = false: returns the patch's size in
 * bits.  PACK = true: also ORs every field into `bits` (LDS, zeroed by the caller). */
template <bool PACK>
__device__ uint32_t walk_patch(const L3EncodeDesc& d, uint32_t c, uint32_t tx, uint32_t ty,
                               uint32_t* bits) {
    const uint32_t lane = threadIdx.x;
    const uint32_t n = d.patch;
    const uint32_t x0 = tx * n, y0 = ty * n;
    const uint32_t pw = min(n, d.width - x0), ph = min(n, d.height - y0);
    const bool has0 = lane < pw, has1 = lane + 64 < pw;          /* pixels lane and lane + 64 */
    const uint8_t* src = d.rgb + (size_t)y0 * d.row_stride + (size_t)x0 * 3 + c;

    int up0 = 0, up1 = 0;           /* the original row above */
    uint32_t pos = 0;               /* bit position of the current row's record */
    int next0 = has0 ? src[3 * (size_t)lane] : 0;             /* the row after, already travelling */
    int next1 = has1 ? src[3 * (size_t)(lane + 64)] : 0;
    for (uint32_t r = 0; r < ph; ++r) {
        const int cur0 = next0, cur1 = next1;
        if (r + 1 < ph) {
            const uint8_t* row = src + (size_t)(r + 1) * d.row_stride;
            next0 = has0 ? row[3 * (size_t)lane] : 0;
            next1 = has1 ? row[3 * (size_t)(lane + 64)] : 0;
        }
        int v0, v1;
        if (r == 0) {
            v0 = cur0;              /* first row raw, taken as unsigned */
            v1 = cur1;
        } else {
            /* neighbours of pixel `lane`: lanes -1/+1; of pixel `lane + 64`: the same
             * lanes' second pixels, with lanes 63 and 0 joining the halves */
            const int l0 = __shfl_up(up0, 1), r0 = __shfl_down(up0, 1);
            const int l1 = __shfl_up(up1, 1), r1 = __shfl_down(up1, 1);
            const int first1 = __shfl(up1, 0), last0 = __shfl(up0, 63);
            const int tl0 = l0, tr0 = lane == 63 ? first1 : r0;
            const int tl1 = lane == 0 ? last0 : l1, tr1 = r1;
            const bool edge0 = lane == 0 || lane + 1 == pw;
            const bool edge1 = lane + 64 + 1 == pw;
            const int p0 = edge0 ? up0 : nearest_upper(tl0, up0, tr0);
            const int p1 = edge1 ? up1 : nearest_upper(tl1, up1, tr1);
            v0 = (int)(int8_t)(uint8_t)(cur0 - p0);   /* later rows taken as signed bytes */
            v1 = (int)(int8_t)(uint8_t)(cur1 - p1);
        }
        int lo = 1 << 20, hi = -(1 << 20);
        if (has0) { lo = v0; hi = v0; }
        if (has1) { lo = min(lo, v1); hi = max(hi, v1); }
        lo = wave_min(lo);
        hi = wave_max(hi);
        const uint32_t range = (uint32_t)(hi - lo);
        const uint32_t width = range ? 32u - (uint32_t)__builtin_clz(range) : 0u;
        if (PACK) {
            if (lane == 0) {
                const uint32_t rec = width | (((uint32_t)lo & 0xFFu) << 4);
                const uint32_t sh = pos & 31u;
                atomicOr(&bits[pos >> 5], rec << sh);
                if (sh > 20) atomicOr(&bits[(pos >> 5) + 1], rec >> (32u - sh));
            }
            if (width) {
                if (has0) {
                    const uint32_t b = pos + 12 + lane * width, sh = b & 31u;
                    const uint32_t dlt = (uint32_t)(v0 - lo);
                    atomicOr(&bits[b >> 5], dlt << sh);
                    if (sh + width > 32) atomicOr(&bits[(b >> 5) + 1], dlt >> (32u - sh));
                }
                if (has1) {
                    const uint32_t b = pos + 12 + (lane + 64) * width, sh = b & 31u;
                    const uint32_t dlt = (uint32_t)(v1 - lo);
                    atomicOr(&bits[b >> 5], dlt << sh);
                    if (sh + width > 32) atomicOr(&bits[(b >> 5) + 1], dlt >> (32u - sh));
                }
            }
        }
        pos += 12 + pw * width;
        up0 = cur0;
        up1 = cur1;
    }
    return pos;
}


/* ---- the strip route: N in {32, 64, 128} ------------------------------------ */

template <int N>
struct StripGeom {
    static constexpr int LPT = N / 4;              /* lanes per patch, 4 pixels each */
    static constexpr int TPW = 64 / LPT;           /* patches per wave */
    static constexpr int P = 3;                    /* rows between two flushes of the rings */
    static constexpr int ROW_MAX = N + 3;          /* bytes a row can touch: ceil((12 + 8N)/8) + 1 */
    static constexpr int RING = 8 * N;             /* ring bytes per patch and channel */
    static constexpr int RING_WORDS = RING / 4 + 4; /* + a word that stands for word 0 of the next lap (and padding to 16 bytes) */
    /* the longest patch stream, rounded up to whole 16-byte granules */
    static constexpr uint32_t SLOT = ((uint32_t)N * (12 + 8 * N) / 8 + 1 + 15) / 16 * 16;
    /* one flush round (a granule per lane of the patch) takes everything that P rows
     * and a pending partial granule can have completed, and the ring holds it */
    static_assert(LPT * 16 >= P * ROW_MAX + 15, "a flush round empties a period");
    static_assert(RING >= 2 * (P * ROW_MAX + 16), "ring holds a period beside the granules being cleared");
    static_assert((RING & (RING - 1)) == 0, "ring size is a power of two");
};

__host__ __device__ constexpr uint32_t strip_slot_bytes(uint32_t n) {
    return n == 32 ? StripGeom<32>::SLOT : n == 64 ? StripGeom<64>::SLOT : StripGeom<128>::SLOT;
}

typedef __attribute__((address_space(1))) const u32x3_any global_const_u32x3_any;
typedef __attribute__((address_space(1))) u32x4 global_u32x4;

__device__ __forceinline__ uint32_t pk_sub_u16_sat(uint32_t a, uint32_t b) {   /* max(a - b, 0) per field */
    uint32_t d;
    asm("v_pk_sub_u16 %0, %1, %2 clamp" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2, a),
                                                                  __builtin_bit_cast(u16x2, b)));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move(uint32_t v) {
    /* every lane has a source lane under these controls, so the "old" value is never used */
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}

/* Minimum of both 16-bit fields, separately, over the LPT lanes of a patch; every
 * lane gets the result.  Butterfly: lane ^ 1, ^ 2 inside quads, then mirrors inside 8
 * and 16 lanes, then the swap of neighbouring 16-lane rows. */
template <int LPT>
__device__ __forceinline__ uint32_t patch_min_u16x2(uint32_t v) {
    v = pk_min_u16(v, dpp_move<0xB1>(v));    /* quad_perm [1,0,3,2] */
    v = pk_min_u16(v, dpp_move<0x4E>(v));    /* quad_perm [2,3,0,1] */
    v = pk_min_u16(v, dpp_move<0x141>(v));   /* row_half_mirror */
    if (LPT >= 16) v = pk_min_u16(v, dpp_move<0x140>(v));   /* row_mirror */
    if (LPT >= 32) {
        const auto both = __builtin_amdgcn_permlane16_swap(v, v, false, false);
        v = pk_min_u16((uint32_t)both[0], (uint32_t)both[1]);
    }
    return v;
}

/* One strip: TPW adjacent patches of one patch row, channel C. */
template <int N, int C>
__device__ __forceinline__ void encode_strip(const L3EncodeDesc& d, uint32_t* __restrict__ sizes,
                                             uint8_t* __restrict__ slots, uint32_t* ring_words) {
    using G = StripGeom<N>;
    constexpr int LPT = G::LPT, TPW = G::TPW, P = G::P, RING = G::RING;

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t g = lane / LPT, xl = lane % LPT;
    const uint32_t ty = blockIdx.x / d.strips_x, strip = blockIdx.x - ty * d.strips_x;
    const uint32_t tx = strip * TPW + g;
    const bool active = tx < d.tiles_x;
    const uint32_t x0 = tx * N, y0 = ty * N;
    const uint32_t pw = active ? min((uint32_t)N, d.width - x0) : 0u;
    const uint32_t ph = min((uint32_t)N, d.height - y0);
    const uint32_t patches = d.tiles_x * d.tiles_y;
    const uint32_t k = C * patches + ty * d.tiles_x + tx;               /* index in the offset arrays */
    uint8_t* const slot = slots + d.slots_base + (uint64_t)k * G::SLOT;

    /* this lane's 4 pixels: columns 4 xl .. 4 xl + 3 of the patch, nvalid of them exist */
    const uint32_t xpix = 4 * xl;
    const uint32_t nvalid = pw > xpix ? min(4u, pw - xpix) : 0u;
    const uint8_t* src = d.rgb + (size_t)y0 * d.row_stride + ((size_t)x0 + xpix) * 3;   /* walks down the rows */

    /* registers of two 16-bit fields: E = pixels (0, 2), O = pixels (1, 3) */
    const uint32_t validE = (nvalid > 0 ? 0x0000FFFFu : 0u) | (nvalid > 2 ? 0xFFFF0000u : 0u);
    const uint32_t validO = (nvalid > 1 ? 0x0000FFFFu : 0u) | (nvalid > 3 ? 0xFFFF0000u : 0u);
    uint32_t border[2];
    border[0] = ((xpix == 0 || xpix + 1 == pw) ? 0x0000FFFFu : 0u) | ((xpix + 3 == pw) ? 0xFFFF0000u : 0u);
    border[1] = ((xpix + 2 == pw) ? 0x0000FFFFu : 0u) | ((xpix + 4 == pw) ? 0xFFFF0000u : 0u);
    const uint32_t keepE = validE & 0x00FF00FFu, keepO = validO & 0x00FF00FFu;

    /* The residual byte r is looked at as t = r ^ K, K = 0 in the first row (raw,
     * unsigned) and 0x80 after it (signed byte + 128), so that the unsigned minimum of t
     * is the row minimum of Section 4.2; u = t ^ 0xFF turns the maximum into a minimum
     * too.  Fields of pixels that do not exist read 0xFFFF in both. */
    uint32_t kminE = ~validE, kminO = ~validO;                          /* K = 0 */
    uint32_t kmaxE = ~validE | keepE, kmaxO = ~validO | keepO;          /* K ^ 0xFF = 0xFF */
    uint32_t krow = 0;

    uint64_t row_stride = d.row_stride;
    asm volatile("" : "+s"(row_stride));    /* kept in registers, not reloaded every row */
    /* The lane's 12 bytes of a row.  A lane at the right edge of the image owns fewer than
     * 4 pixels and must not read past the row: it reads the 12 bytes that END at its last
     * pixel and shifts them down (what then sits above the valid bytes is masked later).
     * Only waves with such a lane take that path; images narrower than 4 pixels go byte by
     * byte. */
    const bool ragged_wave = __builtin_amdgcn_ballot_w64(nvalid != 0 && nvalid != 4) != 0;
    const bool wide = d.width >= 4;
    const uint32_t back = nvalid ? 3 * (4 - nvalid) : 0;              /* bytes to step back: 0, 3, 6, 9 */
    auto load_row = [&](const uint8_t* p) -> u32x3 {
        u32x3 v = {0, 0, 0};
        if (!ragged_wave) {
            if (nvalid == 4) v = *reinterpret_cast<global_const_u32x3_any*>((uintptr_t)p);
        } else if (wide) {
            if (nvalid) {
                const u32x3 q = *reinterpret_cast<global_const_u32x3_any*>((uintptr_t)(p - back));
                const uint32_t words = back >> 2, bits = (back & 3u) * 8;
                const uint32_t a0 = words == 0 ? q.x : (words == 1 ? q.y : q.z);
                const uint32_t a1 = words == 0 ? q.y : (words == 1 ? q.z : 0u);
                const uint32_t a2 = words == 0 ? q.z : 0u;
                v.x = __builtin_amdgcn_alignbit(a1, a0, bits);
                v.y = __builtin_amdgcn_alignbit(a2, a1, bits);
                v.z = a2 >> bits;
            }
        } else if (nvalid) {
            uint32_t b[9];
#pragma unroll
            for (int i = 0; i < 9; ++i) b[i] = (uint32_t)((uint32_t)i < 3 * nvalid ? p[i] : 0);
            v.x = b[0] | (b[1] << 8) | (b[2] << 16) | (b[3] << 24);
            v.y = b[4] | (b[5] << 8) | (b[6] << 16) | (b[7] << 24);
            v.z = b[8];
        }
        return v;
    };

    uint32_t* const ring = ring_words + g * G::RING_WORDS;
    const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint32_t*)ring;
    typedef __attribute__((address_space(3))) uint32_t lds_u32;
    {
        u32x4 zero = {0, 0, 0, 0};
        for (uint32_t i = xl; i < G::RING_WORDS / 4; i += LPT) reinterpret_cast<u32x4*>(ring)[i] = zero;
    }
    wave_lds_fence();

    /* ORs `value` (at most 32 bits) into the ring at bit `pos`.  The upper part may land in
     * the word behind the ring, which stands for word 0 of the next lap: the flush folds
     * it in. */
    auto put = [&](uint32_t value, uint32_t pos) {
        const uint32_t w0 = __builtin_amdgcn_ubfe(pos, 5, __builtin_ctz(RING / 4));
        const uint32_t lo = value << (pos & 31u);
        const uint32_t hi = (value >> 1) >> (~pos & 31u);
        lds_u32* cell = reinterpret_cast<lds_u32*>(ring_lds + 4 * w0);
        __hip_atomic_fetch_or(cell, lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
        __hip_atomic_fetch_or(cell + 1, hi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    };

    uint32_t rowpos = 0;       /* bit position of the next row record in the patch stream */
    uint32_t flushed = 0;      /* granules already in the slot */
    /* writes granules [flushed, upto) of the stream to the slot and clears them in the ring */
    auto flush = [&](uint32_t upto) {
        wave_lds_fence();
        const uint32_t gi = flushed + xl;
        if (active && gi < upto) {
            const uint32_t at = (gi * 16) & (RING - 1);
            u32x4* cell = reinterpret_cast<u32x4*>(reinterpret_cast<uint8_t*>(ring) + at);
            u32x4 v = *cell;
            const u32x4 zero = {0, 0, 0, 0};
            *cell = zero;
            if (at == 0) {                  /* what the previous lap left for this granule's first word */
                v.x |= ring[RING / 4];
                ring[RING / 4] = 0;
            }
            *reinterpret_cast<global_u32x4*>((uintptr_t)(slot + (size_t)gi * 16)) = v;
        }
        flushed = max(flushed, upto);
        wave_lds_fence();
    };

    uint32_t up[2] = {0, 0};   /* the original row above; zeros above the first row predict 0 */

    /* One row: filter, row minimum and maximum, the lane's deltas into the ring.  Returns
     * the row's 12-bit record; its place is the value of rowpos on entry. */
    auto do_row = [&](const u32x3 raw) -> uint32_t {
        /* channel C of pixel i is byte 3 i + C of the lane's 12 bytes */
        uint32_t cur[2];
        if (C == 0) {
            cur[0] = __builtin_amdgcn_perm(raw.y, raw.x, 0x0C060C00u);   /* bytes 0, 6 */
            cur[1] = __builtin_amdgcn_perm(raw.z, raw.x, 0x0C050C03u);   /* bytes 3, 9 */
        } else if (C == 1) {
            cur[0] = __builtin_amdgcn_perm(raw.y, raw.x, 0x0C070C01u);   /* bytes 1, 7 */
            cur[1] = __builtin_amdgcn_perm(raw.z, raw.y, 0x0C060C00u);   /* bytes 4, 10 */
        } else {
            cur[0] = __builtin_amdgcn_perm(raw.z, raw.x, 0x0C040C02u);   /* bytes 2, 8 */
            cur[1] = __builtin_amdgcn_perm(raw.z, raw.y, 0x0C070C01u);   /* bytes 5, 11 */
        }

        /* Section 4.2 stage 1 on the original row above */
        const uint32_t from_left = dpp_from_lower_lane(up[1]);
        const uint32_t from_right = dpp_from_upper_lane(up[0]);
        uint32_t TL[2], TR[2], pred[2];
        TL[0] = __builtin_amdgcn_alignbit(up[1], from_left, 16);
        TR[0] = up[1];
        TL[1] = up[0];
        TR[1] = __builtin_amdgcn_alignbit(from_right, up[0], 16);
        predict_pairs<2>(TL, TR, up, border, pred);
        const uint32_t rE = __builtin_bit_cast(uint32_t, (u16x2)(__builtin_bit_cast(u16x2, cur[0]) -
                                                                 __builtin_bit_cast(u16x2, pred[0])));
        const uint32_t rO = __builtin_bit_cast(uint32_t, (u16x2)(__builtin_bit_cast(u16x2, cur[1]) -
                                                                 __builtin_bit_cast(u16x2, pred[1])));
        /* (r & keep) ^ k */
        const uint32_t tE = __builtin_amdgcn_bitop3_b32(rE, keepE, kminE, 0x6A);
        const uint32_t tO = __builtin_amdgcn_bitop3_b32(rO, keepO, kminO, 0x6A);
        const uint32_t uE = __builtin_amdgcn_bitop3_b32(rE, keepE, kmaxE, 0x6A);
        const uint32_t uO = __builtin_amdgcn_bitop3_b32(rO, keepO, kmaxO, 0x6A);

        /* stage 2, steps 1-2: row minimum and maximum over the patch */
        const uint32_t a = pk_min_u16(tE, tO), b = pk_min_u16(uE, uO);
        uint32_t mm = pk_min_u16(__builtin_amdgcn_perm(b, a, 0x05040100u),    /* (a.lo, b.lo) */
                                 __builtin_amdgcn_perm(b, a, 0x07060302u));   /* (a.hi, b.hi) */
        mm = patch_min_u16x2<LPT>(mm);
        const uint32_t tmin = mm & 0xFFFFu, umin = mm >> 16;     /* min t, 255 - max t */
        const uint32_t range = (255u - (tmin + umin)) & 0xFFu;   /* masked: lanes without a patch hold no minimum */
        const uint32_t w = 31u - (uint32_t)__builtin_clz(2u * range + 1u);
        const uint32_t rec = w | (((tmin ^ krow) & 0xFFu) << 4);

        /* steps 3-4: deltas t - tmin = (255 - tmin) - u, 0 where no pixel exists; the
         * lane's four deltas as one field of 4 w bits */
        const uint32_t top1 = (tmin ^ 0xFFu) & 0xFFu, top = top1 | (top1 << 16);
        const uint32_t dE = pk_sub_u16_sat(top, uE), dO = pk_sub_u16_sat(top, uO);
        const uint32_t pair = dE | (dO << w);                   /* (d0 | d1 << w, d2 | d3 << w) */
        const uint32_t group = (pair & 0xFFFFu) | ((pair >> 16) << (2 * w));
        if (active) put(group, rowpos + 12 + xpix * w);
        rowpos += 12 + pw * w;
        up[0] = cur[0];
        up[1] = cur[1];
        return rec;
    };

    /* Periods of P rows.  The rows of the next period are already travelling from memory
     * while this one is worked on; the granules the previous period completed are written
     * out right after those loads were issued, so that neither is waited for before a
     * whole period of arithmetic has passed. */
    u32x3 ahead[P];
#pragma unroll
    for (int i = 0; i < P; ++i) {
        const u32x3 zero = {0, 0, 0};
        ahead[i] = (uint32_t)i < ph ? load_row(src + i * row_stride) : zero;
    }
    /* issue priorities as in the decoder: lowered by quarters of the rows, an older
     * workgroup of a CU a little sooner; workgroups ahead of the launch's last round keep
     * the top priority */
    const uint32_t wg = blockIdx.y * gridDim.x + blockIdx.x, wgs = gridDim.x * gridDim.y;
    const uint32_t last_round_from = wgs > 2048u ? wgs - 2048u : 0u;
    const uint32_t age_rank = min(7u, ((wg - min(wg, last_round_from)) >> 3) / 32u);
    const uint32_t drop_at[3] = {wg < last_round_from ? 0x7FFFFFFFu : (ph * (8u + age_rank) + 31u) / 32u,
                                 (ph * (16u + age_rank) + 31u) / 32u, (ph * (24u + age_rank) + 31u) / 32u};
    uint32_t next_drop = drop_at[0], stage = 0;
    __builtin_amdgcn_s_setprio(3);
    for (uint32_t r = 0; r < ph; r += P) {
        const uint32_t rows = min((uint32_t)P, ph - r);
        if (r >= next_drop) {
            ++stage;
            next_drop = stage == 1 ? drop_at[1] : (stage == 2 ? drop_at[2] : 0x7FFFFFFFu);
            if (stage == 1) __builtin_amdgcn_s_setprio(2);
            else if (stage == 2) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        u32x3 raw[P];
#pragma unroll
        for (int i = 0; i < P; ++i) raw[i] = ahead[i];
        src += P * row_stride;
        if (r + P < ph) {
#pragma unroll
            for (int i = 0; i < P; ++i)
                if (r + P + i < ph) ahead[i] = load_row(src + i * row_stride);
        }
        if (r > 0) flush(rowpos >> 7);

        uint32_t rec[P], at[P];
        at[0] = rowpos;
        rec[0] = do_row(raw[0]);
        if (r == 0) {            /* rows after the first are looked at as signed bytes */
            krow = 0x80u;
            kminE = ~validE | (keepE & 0x00800080u);
            kminO = ~validO | (keepO & 0x00800080u);
            kmaxE = ~validE | (keepE & 0x007F007Fu);
            kmaxO = ~validO | (keepO & 0x007F007Fu);
        }
        at[1] = rowpos;
        rec[1] = rows > 1 ? do_row(raw[1]) : 0u;
        at[2] = rowpos;
        rec[2] = rows > 2 ? do_row(raw[2]) : 0u;
        /* the records of the period: lane i of the patch writes the one of row i */
        static_assert(P == 3 && LPT >= P, "one lane per record of a period");
        const uint32_t my_rec = xl == 0 ? rec[0] : (xl == 1 ? rec[1] : rec[2]);
        const uint32_t my_at = xl == 0 ? at[0] : (xl == 1 ? at[1] : at[2]);
        if (active && xl < rows) put(my_rec, my_at);
    }
    const uint32_t bytes = (rowpos + 7) / 8;
    flush((bytes + 15) / 16);
    if (active && xl == 0) sizes[d.sizes_base + k] = bytes;
}

template <int N>
__device__ __forceinline__ void strip_block(const L3EncodeDesc& d, uint32_t* __restrict__ sizes,
                                            uint8_t* __restrict__ slots) {
    __shared__ __attribute__((aligned(16))) uint32_t rings[3][StripGeom<N>::TPW * StripGeom<N>::RING_WORDS];
    if (d.patch != N || blockIdx.x >= d.strips_x * d.tiles_y) return;
    const uint32_t c = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (c == 0) encode_strip<N, 0>(d, sizes, slots, rings[0]);
    else if (c == 1) encode_strip<N, 1>(d, sizes, slots, rings[1]);
    else encode_strip<N, 2>(d, sizes, slots, rings[2]);
}

/* Descriptors either in a device table (any batch size) or, for small batches, inside
 * the kernel arguments: no upload to wait for, so consecutive calls run back to back. */
constexpr int kArgDescs = 32;
struct EncodePack { L3EncodeDesc d[kArgDescs]; };
static_assert(sizeof(EncodePack) + 64 <= 4096, "kernel argument segment");

template <int N>
__global__ __launch_bounds__(192) void l3_encode_strip_kernel(const L3EncodeDesc* __restrict__ descs,
                                                              uint32_t* __restrict__ sizes,
                                                              uint8_t* __restrict__ slots) {
    strip_block<N>(descs[blockIdx.y], sizes, slots);
}
template <int N>
__global__ __launch_bounds__(192) void l3_encode_strip_kernel_args(const EncodePack pack,
                                                                   uint32_t* __restrict__ sizes,
                                                                   uint8_t* __restrict__ slots) {
    strip_block<N>(pack.d[blockIdx.y], sizes, slots);
}

/* Copies one slot of the strip route to its place in the file (one workgroup per slot). */
template <int THREADS>
__device__ __forceinline__ void compact_block(const L3EncodeDesc& d, const uint32_t* __restrict__ sizes,
                                              const uint8_t* __restrict__ slots,
                                              const uint64_t* __restrict__ file_len) {
    const uint32_t patches = d.tiles_x * d.tiles_y;
    const uint32_t k = blockIdx.x;
    if ((d.patch != 32 && d.patch != 64 && d.patch != 128) || k >= 3 * patches) return;
    const uint64_t need = file_len[d.status_index];
    if (need > d.file_cap || need - (13 + 12ull * patches) > 0xFFFFFFFFull) return;
    const uint32_t bytes = sizes[d.sizes_base + k];
    const uint32_t offset = *reinterpret_cast<const global_u32_unaligned*>((uintptr_t)(d.file + 13 + 4 * (size_t)k));
    const uint8_t* from = slots + d.slots_base + (uint64_t)k * strip_slot_bytes(d.patch);
    uint8_t* to = d.file + 13 + 12 * (size_t)patches + offset;
    typedef __attribute__((address_space(1))) u32x4 global_u32x4_any __attribute__((aligned(1)));
    const uint32_t whole = bytes / 16;
    for (uint32_t i = threadIdx.x; i < whole; i += THREADS)
        *reinterpret_cast<global_u32x4_any*>((uintptr_t)(to + 16 * (size_t)i)) =
            *reinterpret_cast<const global_const_u32x4*>((uintptr_t)(from + 16 * (size_t)i));
    const uint32_t tail = bytes - 16 * whole;
    if (threadIdx.x < tail) to[16 * (size_t)whole + threadIdx.x] = from[16 * (size_t)whole + threadIdx.x];
}
template <int THREADS>
__global__ __launch_bounds__(THREADS) void l3_encode_compact_kernel(const L3EncodeDesc* __restrict__ descs,
                                                                    const uint32_t* __restrict__ sizes,
                                                                    const uint8_t* __restrict__ slots,
                                                                    const uint64_t* __restrict__ file_len) {
    compact_block<THREADS>(descs[blockIdx.y], sizes, slots, file_len);
}
template <int THREADS>
__global__ __launch_bounds__(THREADS) void l3_encode_compact_kernel_args(const EncodePack pack,
                                                                         const uint32_t* __restrict__ sizes,
                                                                         const uint8_t* __restrict__ slots,
                                                                         const uint64_t* __restrict__ file_len) {
    compact_block<THREADS>(pack.d[blockIdx.y], sizes, slots, file_len);
}

/* ---- the plain route: any other N up to 128 -------------------------------- */

__global__ __launch_bounds__(64) void l3_encode_measure_kernel(const L3EncodeDesc* __restrict__ descs,
                                                               uint32_t* __restrict__ sizes) {
    const L3EncodeDesc& d = descs[blockIdx.y];
    const uint32_t patches = d.tiles_x * d.tiles_y;
    const uint32_t k = blockIdx.x;
    if (k >= 3 * patches || d.patch == 32 || d.patch == 64 || d.patch == 128) return;
    const uint32_t c = k / patches, i = k - c * patches;
    const uint32_t bits = walk_patch<false>(d, c, i % d.tiles_x, i / d.tiles_x, nullptr);
    if (threadIdx.x == 0) sizes[d.sizes_base + k] = (bits + 7) / 8;
}

/* One workgroup per image: offsets = exclusive prefix sum of the patch sizes. */
__device__ __forceinline__ void layout_block(const L3EncodeDesc& d, const uint32_t* __restrict__ sizes,
                                             uint64_t* __restrict__ file_len,
                                             uint32_t* __restrict__ status) {
    const uint32_t patches = d.tiles_x * d.tiles_y, total = 3 * patches;
    const uint64_t header = 13 + 12ull * patches;
    const bool header_fits = header <= d.file_cap;
    __shared__ uint64_t scan[256];
    __shared__ uint64_t carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (uint32_t first = 0; first < total; first += 256) {
        const uint32_t k = first + threadIdx.x;
        const uint64_t mine = k < total ? sizes[d.sizes_base + k] : 0;
        scan[threadIdx.x] = mine;
        __syncthreads();
        for (uint32_t step = 1; step < 256; step <<= 1) {       /* inclusive scan of the chunk */
            const uint64_t add = threadIdx.x >= step ? scan[threadIdx.x - step] : 0;
            __syncthreads();
            scan[threadIdx.x] += add;
            __syncthreads();
        }
        const uint64_t offset = carry + scan[threadIdx.x] - mine;
        if (k < total && header_fits && offset <= 0xFFFFFFFFull)
            *reinterpret_cast<global_u32_unaligned*>((uintptr_t)(d.file + 13 + 4 * (size_t)k)) = (uint32_t)offset;
        __syncthreads();
        if (threadIdx.x == 255) carry += scan[255];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const uint64_t need = header + carry;
        file_len[d.status_index] = need;
        uint32_t st = 0;
        if (need > d.file_cap) st |= 1u;                 /* output capacity too small: nothing packed */
        if (carry > 0xFFFFFFFFull) st |= 2u;             /* data section beyond 32-bit offsets */
        if (status) status[d.status_index] = st;
        if (header_fits) {
            uint8_t* f = d.file;
            f[0] = 0x4C; f[1] = 0x33; f[2] = 0x00; f[3] = 0x01;
            for (int b = 0; b < 4; ++b) {
                f[4 + b] = (uint8_t)(d.width >> (8 * b));
                f[8 + b] = (uint8_t)(d.height >> (8 * b));
            }
            f[12] = (uint8_t)d.patch;
        }
    }
}
__global__ __launch_bounds__(256) void l3_encode_layout_kernel(const L3EncodeDesc* __restrict__ descs,
                                                               const uint32_t* __restrict__ sizes,
                                                               uint64_t* __restrict__ file_len,
                                                               uint32_t* __restrict__ status) {
    layout_block(descs[blockIdx.x], sizes, file_len, status);
}
__global__ __launch_bounds__(256) void l3_encode_layout_kernel_args(const EncodePack pack,
                                                                    const uint32_t* __restrict__ sizes,
                                                                    uint64_t* __restrict__ file_len,
                                                                    uint32_t* __restrict__ status) {
    layout_block(pack.d[blockIdx.x], sizes, file_len, status);
}

__global__ __launch_bounds__(64) void l3_encode_pack_kernel(const L3EncodeDesc* __restrict__ descs,
                                                            const uint32_t* __restrict__ sizes,
                                                            const uint64_t* __restrict__ file_len) {
    const L3EncodeDesc& d = descs[blockIdx.y];
    const uint32_t patches = d.tiles_x * d.tiles_y;
    const uint32_t k = blockIdx.x;
    if (k >= 3 * patches || d.patch == 32 || d.patch == 64 || d.patch == 128) return;
    const uint64_t need = file_len[d.status_index];
    if (need > d.file_cap || need - (13 + 12ull * patches) > 0xFFFFFFFFull) return;

    extern __shared__ uint32_t bits[];   /* sized by the host for the largest patch of the launch */
    const uint32_t bytes = sizes[d.sizes_base + k];
    const uint32_t words = (bytes + 3) / 4 + 1;
    for (uint32_t i = threadIdx.x; i < words; i += 64) bits[i] = 0;
    __syncthreads();
    const uint32_t c = k / patches, i = k - c * patches;
    (void)walk_patch<true>(d, c, i % d.tiles_x, i / d.tiles_x, bits);
    __syncthreads();

    const uint32_t offset = *reinterpret_cast<const global_u32_unaligned*>((uintptr_t)(d.file + 13 + 4 * (size_t)k));
    uint8_t* dst = d.file + 13 + 12 * (size_t)patches + offset;
    const uint32_t whole = bytes / 4;
    for (uint32_t w = threadIdx.x; w < whole; w += 64)
        *reinterpret_cast<global_u32_unaligned*>((uintptr_t)(dst + 4 * (size_t)w)) = bits[w];
    const uint32_t tail = bytes - 4 * whole;
    if (threadIdx.x < tail) dst[4 * (size_t)whole + threadIdx.x] = (uint8_t)(bits[whole] >> (8 * threadIdx.x));
}

}  // namespace

/* Workspace of l3_encode_batch: descriptor table (pinned + device) and patch sizes. */
struct L3EncodeState {
    L3EncodeDesc* h_descs = nullptr;  /* pinned: kStage staging tables of desc_cap entries each */
    hipEvent_t staged[4] = {};        /* the upload from staging table i has left it */
    bool staged_pending[4] = {};
    int next_stage = 0;
    L3EncodeDesc* d_descs = nullptr;
    size_t desc_cap = 0;
    uint32_t* d_sizes = nullptr;
    size_t sizes_cap = 0;
    uint8_t* d_slots = nullptr;      /* strip route: one fixed-size slot per patch and channel */
    size_t slots_cap = 0;
    hipEvent_t done = nullptr;       /* the last call's kernels have finished */
    bool pending = false;
    hipStream_t last_stream = nullptr;
};

void l3_encode_state_free(L3EncodeState* s) {
    if (!s) return;
    if (s->pending) (void)hipEventSynchronize(s->done);
    if (s->done) (void)hipEventDestroy(s->done);
    for (int i = 0; i < 4; ++i)
        if (s->staged[i]) (void)hipEventDestroy(s->staged[i]);
    if (s->h_descs) (void)hipHostFree(s->h_descs);
    if (s->d_descs) (void)hipFree(s->d_descs);
    if (s->d_sizes) (void)hipFree(s->d_sizes);
    if (s->d_slots) (void)hipFree(s->d_slots);
    delete s;
}

extern "C" l3_status l3_encode_batch(l3_ctx* ctx, const l3_encode_item* items, int n,
                                     uint64_t* d_file_len, uint32_t* d_status, void* stream_v) {
    if (!ctx || n < 0 || (n > 0 && (!items || !d_file_len))) return L3_ERR_INVALID_ARG;
    if (n == 0) return L3_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return L3_ERR_DEVICE;

    size_t total_patches = 0, slot_bytes = 0;
    uint32_t max_patches = 0, max_n = 1;
    uint32_t strip_units[3] = {0, 0, 0};   /* largest grid of the strip route per N = 32, 64, 128 */
    bool any_plain = false;
    for (int i = 0; i < n; ++i) {
        const l3_encode_item& it = items[i];
        if (!it.d_rgb || !it.d_file || it.width == 0 || it.height == 0 ||
            it.row_stride < (size_t)it.width * 3)
            return L3_ERR_INVALID_ARG;
        const uint32_t np = it.patch ? it.patch : l3_default_patch(it.width, it.height);
        if (np > kMaxPatch) return L3_ERR_UNSUPPORTED;
        if (np > max_n) max_n = np;
        if (it.width > (1u << 24) || it.height > (1u << 24)) return L3_ERR_UNSUPPORTED;
        const uint64_t p = (uint64_t)((it.width + np - 1) / np) * ((it.height + np - 1) / np);
        if (3 * p > 0x7FFFFFFFull) return L3_ERR_UNSUPPORTED;
        total_patches += (size_t)(3 * p);
        if (3 * p > max_patches) max_patches = (uint32_t)(3 * p);
        if (np == 32 || np == 64 || np == 128) {
            const uint32_t cls = np == 32 ? 0 : np == 64 ? 1 : 2;
            const uint32_t tpw = 256 / np, tiles_x = (it.width + np - 1) / np;
            const uint64_t units = (uint64_t)((tiles_x + tpw - 1) / tpw) * ((it.height + np - 1) / np);
            if (units > strip_units[cls]) strip_units[cls] = (uint32_t)units;
            slot_bytes += (size_t)(3 * p) * strip_slot_bytes(np);
        } else {
            any_plain = true;
        }
    }
    if (total_patches > 0xFFFFFFFFull) return L3_ERR_UNSUPPORTED;

    if (!ctx->enc) {
        ctx->enc = new (std::nothrow) L3EncodeState;
        if (!ctx->enc) return L3_ERR_DEVICE;
        if (hipEventCreateWithFlags(&ctx->enc->done, hipEventDisableTiming) != hipSuccess) return L3_ERR_DEVICE;
    }
    L3EncodeState* st = ctx->enc;
    /* The workspace (size table, slots, descriptor table) is shared by consecutive calls.
     * On the device a call is ordered after the previous one; the host waits for the
     * previous call only before it frees or overwrites something that call still reads. */
    auto wait_previous = [&]() -> bool {
        if (st->pending && hipEventSynchronize(st->done) != hipSuccess) return false;
        st->pending = false;
        return true;
    };
    if (st->pending && stream != st->last_stream &&
        hipStreamWaitEvent(stream, st->done, 0) != hipSuccess)
        return L3_ERR_DEVICE;
    const bool by_args = n <= kArgDescs && !any_plain;
    constexpr int kStage = 4;
    int stage = 0;
    if (!by_args) {
        if ((size_t)n > st->desc_cap) {
            if (!wait_previous()) return L3_ERR_DEVICE;      /* its uploads and kernels read the old tables */
            size_t cap = 64;
            while (cap < (size_t)n) cap *= 2;
            if (st->h_descs) (void)hipHostFree(st->h_descs);
            if (st->d_descs) (void)hipFree(st->d_descs);
            st->h_descs = nullptr;
            st->d_descs = nullptr;
            st->desc_cap = 0;
            for (int i = 0; i < kStage; ++i) st->staged_pending[i] = false;
            if (hipHostMalloc(reinterpret_cast<void**>(&st->h_descs), kStage * cap * sizeof(L3EncodeDesc),
                              hipHostMallocDefault) != hipSuccess ||
                hipMalloc(reinterpret_cast<void**>(&st->d_descs), cap * sizeof(L3EncodeDesc)) != hipSuccess)
                return L3_ERR_DEVICE;
            st->desc_cap = cap;
        }
        /* the staging table about to be rewritten: its last upload must have left it */
        stage = st->next_stage;
        st->next_stage = (stage + 1) % kStage;
        if (!st->staged[stage] &&
            hipEventCreateWithFlags(&st->staged[stage], hipEventDisableTiming) != hipSuccess)
            return L3_ERR_DEVICE;
        if (st->staged_pending[stage] && hipEventSynchronize(st->staged[stage]) != hipSuccess)
            return L3_ERR_DEVICE;
        st->staged_pending[stage] = false;
    }
    if (total_patches > st->sizes_cap) {
        if (!wait_previous()) return L3_ERR_DEVICE;
        size_t cap = 4096;
        while (cap < total_patches) cap *= 2;
        if (st->d_sizes) (void)hipFree(st->d_sizes);
        st->d_sizes = nullptr;
        st->sizes_cap = 0;
        if (hipMalloc(reinterpret_cast<void**>(&st->d_sizes), cap * sizeof(uint32_t)) != hipSuccess)
            return L3_ERR_DEVICE;
        st->sizes_cap = cap;
    }
    if (slot_bytes > st->slots_cap) {
        if (!wait_previous()) return L3_ERR_DEVICE;
        if (st->d_slots) (void)hipFree(st->d_slots);
        st->d_slots = nullptr;
        st->slots_cap = 0;
        if (hipMalloc(reinterpret_cast<void**>(&st->d_slots), slot_bytes) != hipSuccess)
            return L3_ERR_DEVICE;
        st->slots_cap = slot_bytes;
    }

    EncodePack pack;
    L3EncodeDesc* const table = by_args ? pack.d : st->h_descs + (size_t)stage * st->desc_cap;
    size_t base = 0, slots_base = 0;
    for (int i = 0; i < n; ++i) {
        const l3_encode_item& it = items[i];
        L3EncodeDesc& d = table[i];
        const uint32_t np = it.patch ? it.patch : l3_default_patch(it.width, it.height);
        d.rgb = it.d_rgb;
        d.file = it.d_file;
        d.row_stride = it.row_stride;
        d.file_cap = it.file_cap;
        d.width = it.width;
        d.height = it.height;
        d.tiles_x = (it.width + np - 1) / np;
        d.tiles_y = (it.height + np - 1) / np;
        d.patch = np;
        d.sizes_base = (uint32_t)base;
        d.status_index = (uint32_t)i;
        d.strips_x = 0;
        d.slots_base = 0;
        if (np == 32 || np == 64 || np == 128) {
            const uint32_t tpw = 256 / np;
            d.strips_x = (d.tiles_x + tpw - 1) / tpw;
            d.slots_base = slots_base;
            slots_base += 3 * (size_t)d.tiles_x * d.tiles_y * strip_slot_bytes(np);
        }
        base += 3 * (size_t)d.tiles_x * d.tiles_y;
    }
    if (by_args) {
        for (int i = n; i < kArgDescs; ++i) std::memset(&pack.d[i], 0, sizeof(L3EncodeDesc));
        const uint32_t m = (uint32_t)n;
        if (strip_units[0])
            hipLaunchKernelGGL(l3_encode_strip_kernel_args<32>, dim3(strip_units[0], m), dim3(192), 0, stream,
                               pack, st->d_sizes, st->d_slots);
        if (strip_units[1])
            hipLaunchKernelGGL(l3_encode_strip_kernel_args<64>, dim3(strip_units[1], m), dim3(192), 0, stream,
                               pack, st->d_sizes, st->d_slots);
        if (strip_units[2])
            hipLaunchKernelGGL(l3_encode_strip_kernel_args<128>, dim3(strip_units[2], m), dim3(192), 0, stream,
                               pack, st->d_sizes, st->d_slots);
        hipLaunchKernelGGL(l3_encode_layout_kernel_args, dim3(m), dim3(256), 0, stream, pack, st->d_sizes,
                           d_file_len, d_status);
        /* a slot of a 128-pixel patch is up to 16.6 KB: four waves; smaller ones: one */
        if (strip_units[2])
            hipLaunchKernelGGL(l3_encode_compact_kernel_args<256>, dim3(max_patches, m), dim3(256), 0, stream,
                               pack, st->d_sizes, st->d_slots, d_file_len);
        else
            hipLaunchKernelGGL(l3_encode_compact_kernel_args<64>, dim3(max_patches, m), dim3(64), 0, stream,
                               pack, st->d_sizes, st->d_slots, d_file_len);
    } else {
        if (hipMemcpyAsync(st->d_descs, table, (size_t)n * sizeof(L3EncodeDesc), hipMemcpyHostToDevice,
                           stream) != hipSuccess ||
            hipEventRecord(st->staged[stage], stream) != hipSuccess)
            return L3_ERR_DEVICE;
        st->staged_pending[stage] = true;
        const bool any_strip = strip_units[0] || strip_units[1] || strip_units[2];
        const size_t lds_bytes = ((size_t)max_n * (12 + 8 * (size_t)max_n) + 31) / 32 * 4 + 8;
        for (int first = 0; first < n; first += 65535) {
            const uint32_t m = (uint32_t)(n - first < 65535 ? n - first : 65535);
            const L3EncodeDesc* dd = st->d_descs + first;
            if (strip_units[0])
                hipLaunchKernelGGL(l3_encode_strip_kernel<32>, dim3(strip_units[0], m), dim3(192), 0, stream,
                                   dd, st->d_sizes, st->d_slots);
            if (strip_units[1])
                hipLaunchKernelGGL(l3_encode_strip_kernel<64>, dim3(strip_units[1], m), dim3(192), 0, stream,
                                   dd, st->d_sizes, st->d_slots);
            if (strip_units[2])
                hipLaunchKernelGGL(l3_encode_strip_kernel<128>, dim3(strip_units[2], m), dim3(192), 0, stream,
                                   dd, st->d_sizes, st->d_slots);
            if (any_plain)
                hipLaunchKernelGGL(l3_encode_measure_kernel, dim3(max_patches, m), dim3(64), 0, stream, dd,
                                   st->d_sizes);
        }
        hipLaunchKernelGGL(l3_encode_layout_kernel, dim3((uint32_t)n), dim3(256), 0, stream, st->d_descs,
                           st->d_sizes, d_file_len, d_status);
        for (int first = 0; first < n; first += 65535) {
            const uint32_t m = (uint32_t)(n - first < 65535 ? n - first : 65535);
            const L3EncodeDesc* dd = st->d_descs + first;
            if (any_strip && strip_units[2])
                hipLaunchKernelGGL(l3_encode_compact_kernel<256>, dim3(max_patches, m), dim3(256), 0, stream,
                                   dd, st->d_sizes, st->d_slots, d_file_len);
            else if (any_strip)
                hipLaunchKernelGGL(l3_encode_compact_kernel<64>, dim3(max_patches, m), dim3(64), 0, stream,
                                   dd, st->d_sizes, st->d_slots, d_file_len);
            if (any_plain)
                hipLaunchKernelGGL(l3_encode_pack_kernel, dim3(max_patches, m), dim3(64), lds_bytes, stream,
                                   dd, st->d_sizes, d_file_len);
        }
    }
    if (hipGetLastError() != hipSuccess) return L3_ERR_DEVICE;
    if (hipEventRecord(st->done, stream) != hipSuccess) return L3_ERR_DEVICE;
    st->pending = true;
    st->last_stream = stream;
    return L3_OK;
}
