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
 *   - A wave (64 lanes) owns TPW horizontally adjacent patches, all three colour
 *     channels of each.  A group of LPT = N/PPL lanes owns one patch; every lane
 *     owns PPL adjacent pixels of the current row in all three channels, held as
 *     packed pairs of 16-bit fields so that one v_pk_* instruction works on two
 *     pixels.  Waves never synchronise with each other.
 *   - The compressed stream of each (patch, channel) is pulled from HBM in
 *     16-byte-aligned chunks of LPT*16 bytes (one global_load_dwordx4 per lane,
 *     contiguous over the group) into a private LDS ring of two chunks, one
 *     chunk being prefetched in registers while the other is consumed.
 *   - The row-start chain (row r+1 begins where row r ends, and row r's length
 *     is known only from its own width field) is walked in LDS by all lanes of
 *     the group redundantly (broadcast reads).
 *   - The upper-row neighbours come from registers: in-lane for the inner pixels,
 *     DPP wave shifts for the two pixels at the lane's edges.
 *   - With all three channels in one lane, interleaved RGB leaves the lane as
 *     one contiguous store of 3*PPL bytes; a wave row is a contiguous run.
 */
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>
#include <new>

#include "l3_internal.h"

namespace {

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

struct __attribute__((packed, aligned(1))) U32x3u { uint32_t a, b, c; };
struct __attribute__((packed, aligned(1))) U32u { uint32_t v; };
struct __attribute__((packed, aligned(1))) U16u { uint16_t v; };
struct __attribute__((packed, aligned(1))) U64u { uint64_t v; };

constexpr int kWavesPerBlock = 4;

template <int N, int PPL>
struct Geom {
    static_assert(N == 32 || N == 64 || N == 128, "patch sizes of the GPU path");
    static_assert(PPL == 2 || PPL == 4, "pixels per lane");
    static constexpr int LPT = N / PPL;          /* lanes per patch */
    static constexpr int TPW = 64 / LPT;         /* patches per wave */
    static constexpr int NP = PPL / 2;           /* packed registers per channel row */
    static constexpr int CHUNK = LPT * 16;       /* bytes per refill of one stream */
    static constexpr int RING = 2 * CHUNK;       /* ring bytes per stream */
    static constexpr int RING_WORDS = RING / 4 + 4; /* + 16-byte mirror of the ring start */
    static_assert(LPT >= 1 && TPW >= 1 && CHUNK >= N + 16, "ring invariants");
};

/* ---- small device helpers ------------------------------------------------ */

__device__ __forceinline__ uint32_t dpp_from_lower_lane(uint32_t v) {   /* lane i <- lane i-1 */
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x138 /* wave_shr:1 */, 0xF, 0xF, false);
}
__device__ __forceinline__ uint32_t dpp_from_upper_lane(uint32_t v) {   /* lane i <- lane i+1 */
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x130 /* wave_shl:1 */, 0xF, 0xF, false);
}

__device__ __forceinline__ uint32_t pk_mad_i16(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t d;
    asm("v_pk_mad_i16 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

/* Section 4.2, custom Paeth filter, on two pixels at once (16-bit fields holding
 * 0..255).  Value-wise the nearest of TL, TR, T to TL + TR - T is: with
 * lo = min(TL,TR), hi = max(TL,TR), dl = T - lo, dh = hi - T (signed):
 * lo if dl >= 2*dh, else hi if dh >= 2*dl, else T.  The stated tie order
 * (TL, TR, T) only ever chooses between equal values, except T against a
 * neighbour, where the neighbour wins: that is the ">=" above.
 * `border` has all ones in the fields whose pixel sits in the first or last
 * column of its patch, where the prediction is T. */
__device__ __forceinline__ uint32_t predict2(uint32_t TL, uint32_t TR, uint32_t T, uint32_t border) {
    const u16x2 a = __builtin_bit_cast(u16x2, TL), b = __builtin_bit_cast(u16x2, TR),
                c = __builtin_bit_cast(u16x2, T);
    const u16x2 lo = __builtin_elementwise_min(a, b), hi = __builtin_elementwise_max(a, b);
    const uint32_t dl = __builtin_bit_cast(uint32_t, (u16x2)(c - lo));
    const uint32_t dh = __builtin_bit_cast(uint32_t, (u16x2)(hi - c));
    const uint32_t minus2 = 0xFFFEFFFEu;
    const s16x2 t_lo = __builtin_bit_cast(s16x2, pk_mad_i16(dh, minus2, dl));   /* dl - 2 dh */
    const s16x2 t_hi = __builtin_bit_cast(s16x2, pk_mad_i16(dl, minus2, dh));   /* dh - 2 dl */
    uint32_t not_lo = __builtin_bit_cast(uint32_t, (s16x2)(t_lo >> 15));
    uint32_t not_hi = __builtin_bit_cast(uint32_t, (s16x2)(t_hi >> 15));
    asm("" : "+v"(not_lo));   /* keep the masks packed: no per-half compare/select */
    asm("" : "+v"(not_hi));
    const uint32_t H = __builtin_bit_cast(uint32_t, hi), L = __builtin_bit_cast(uint32_t, lo);
    const uint32_t r = (not_hi & T) | (~not_hi & H);
    const uint32_t p = (not_lo & r) | (~not_lo & L);
    return (border & T) | (~border & p);
}

/* 32 stream bits starting at bit `bit` of a ring (bit counts from the ring's
 * aligned origin; the ring holds the stream modulo RING bytes). */
template <int RING>
__device__ __forceinline__ uint32_t ring_bits(const uint32_t* ring, uint32_t bit) {
    const uint32_t i = (bit >> 5) & (RING / 4 - 1);
    const uint32_t lo = ring[i], hi = ring[i + 1];   /* i + 1 may be the mirror word */
    return __builtin_amdgcn_alignbit(hi, lo, bit);   /* ({hi,lo} >> (bit & 31)) */
}

__device__ __forceinline__ uint4 load_chunk(const uint8_t* p, const uint8_t* file_end16) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (p < file_end16) v = *reinterpret_cast<const uint4*>(p);
    return v;
}

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ uint32_t byte_of(uint32_t packed, int k) {   /* pixel k of a packed pair */
    return (packed >> (16 * k)) & 0xFFu;
}

/* ---- the decode kernel ---------------------------------------------------- */

template <int N, int PPL, int MODE>
__global__ __launch_bounds__(64 * kWavesPerBlock) void l3_decode_kernel(
    const L3ImageDesc* __restrict__ descs, uint32_t* __restrict__ status, uint32_t crop_w,
    uint32_t crop_h, const uint16_t* __restrict__ lut) {
    using G = Geom<N, PPL>;
    constexpr int LPT = G::LPT, TPW = G::TPW, NP = G::NP, CHUNK = G::CHUNK, RING = G::RING;

    __shared__ __attribute__((aligned(16))) uint32_t rings[kWavesPerBlock][TPW * 3][G::RING_WORDS];
    __shared__ uint16_t s_lut[MODE == L3_MODE_TENSOR ? 768 : 2];

    if (MODE == L3_MODE_TENSOR) {
        for (uint32_t i = threadIdx.x; i < 768; i += 64 * kWavesPerBlock) s_lut[i] = lut[i];
        __syncthreads();
    }

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const L3ImageDesc& d = descs[blockIdx.y];
    const uint32_t unit = blockIdx.x * kWavesPerBlock + wave;
    if (unit >= d.units) return;

    const uint32_t g = lane / LPT, xl = lane % LPT;
    const uint32_t trow = unit / d.groups_x, gx = unit - trow * d.groups_x;
    const uint32_t ty = d.tile_y_first + trow;
    const uint32_t txr = gx * TPW + g;
    const bool active = txr < d.tile_x_count;
    const uint32_t tx = d.tile_x_first + (active ? txr : d.tile_x_count - 1);
    const uint32_t x0 = tx * N, y0 = ty * N;
    const uint32_t pw = min((uint32_t)N, d.width - x0);
    const uint32_t ph = min((uint32_t)N, d.height - y0);     /* same for the whole wave */
    const uint32_t patches = d.tiles_x * d.tiles_y;
    const uint32_t data_len = (uint32_t)(d.file_len - d.header_bytes);
    const uint8_t* file_end16 =
        reinterpret_cast<const uint8_t*>(((uintptr_t)d.file + d.file_len + 15) & ~(uintptr_t)15);

    uint32_t flags = 0;
    uint32_t bitpos[3], fill[3], endbit[3];
    const uint8_t* gaddr[3];
    uint4 pf[3];
    uint32_t* ring[3];

#pragma unroll
    for (int c = 0; c < 3; ++c) {
        const uint32_t flat = c * patches + ty * d.tiles_x + tx;
        const uint8_t* otab = d.file + 13 + 4 * (size_t)flat;
        uint32_t off = reinterpret_cast<const U32u*>(otab)->v;
        uint32_t end = flat + 1 < 3 * patches ? reinterpret_cast<const U32u*>(otab + 4)->v : data_len;
        if (off > data_len || end > data_len || end < off) {
            flags |= L3_STATUS_BAD_OFFSET;
            off = min(off, data_len);
            end = min(max(end, off), data_len);
        }
        const uintptr_t a = (uintptr_t)(d.file + d.header_bytes + off);
        const uintptr_t ab = a & ~(uintptr_t)15;
        bitpos[c] = (uint32_t)(a - ab) * 8;
        endbit[c] = bitpos[c] + (end - off) * 8;
        gaddr[c] = reinterpret_cast<const uint8_t*>(ab) + xl * 16;
        fill[c] = 0;
        pf[c] = load_chunk(gaddr[c], file_end16);
        ring[c] = rings[wave][g * 3 + c];
    }

    /* per-lane constants of the row loop */
    const uint32_t xpix = xl * PPL;                         /* first pixel column of this lane */
    uint32_t border[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        const uint32_t xa = xpix + 2 * j, xb = xa + 1;
        border[j] = ((xa == 0 || xa + 1 == pw) ? 0x0000FFFFu : 0u) |
                    ((xb == 0 || xb + 1 == pw) ? 0xFFFF0000u : 0u);
    }
    const uint32_t nvalid = !active ? 0u : (xpix >= pw ? 0u : min((uint32_t)PPL, pw - xpix));

    uint32_t prev[3][NP];
#pragma unroll
    for (int c = 0; c < 3; ++c)
#pragma unroll
        for (int j = 0; j < NP; ++j) prev[c][j] = 0;   /* an all-zero row above predicts 0: row 0 is raw */

    for (uint32_t r = 0; r < ph; ++r) {
        /* keep each ring ahead of the longest possible row (12 + 8N bits) */
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            const uint32_t need = (bitpos[c] >> 3) + N + 12;
            if (fill[c] < need) {
                const uint32_t idx = (fill[c] + xl * 16) & (RING - 1);
                *reinterpret_cast<uint4*>(reinterpret_cast<uint8_t*>(ring[c]) + idx) = pf[c];
                if (idx == 0)
                    *reinterpret_cast<uint4*>(reinterpret_cast<uint8_t*>(ring[c]) + RING) = pf[c];
                fill[c] += CHUNK;
                pf[c] = load_chunk(gaddr[c] + fill[c], file_end16);
            }
        }
        wave_lds_fence();

        uint32_t cur[3][NP];
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            /* base-delta record of this row: width (4 bits), base (8 bits) */
            const uint32_t hdr = ring_bits<RING>(ring[c], bitpos[c]);
            uint32_t w = hdr & 15u;
            const uint32_t base = (hdr >> 4) & 255u;
            if (w > 8) {
                flags |= L3_STATUS_BAD_WIDTH;
                w = 8;
            }
            const uint32_t dbit = bitpos[c] + 12;
            bitpos[c] = dbit + pw * w;
            const uint32_t base2 = base | (base << 16);
            const uint32_t mask = (1u << w) - 1u;
            /* this lane's PPL deltas: PPL*w <= 32 contiguous bits */
            uint32_t x = ring_bits<RING>(ring[c], dbit + xpix * w);
            uint32_t delta[NP];
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                const uint32_t d0 = x & mask;
                x >>= w;
                const uint32_t d1 = x & mask;
                x >>= w;
                delta[j] = d0 | (d1 << 16);
            }
            /* inverse filter from the row above (registers + lane neighbours) */
            const uint32_t from_left = dpp_from_lower_lane(prev[c][NP - 1]);
            const uint32_t from_right = dpp_from_upper_lane(prev[c][0]);
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                const uint32_t T = prev[c][j];
                const uint32_t TL = __builtin_amdgcn_alignbit(T, j > 0 ? prev[c][j - 1] : from_left, 16);
                const uint32_t TR =
                    __builtin_amdgcn_alignbit(j < NP - 1 ? prev[c][j + 1] : from_right, T, 16);
                const uint32_t pred = predict2(TL, TR, T, border[j]);
                cur[c][j] = (pred + delta[j] + base2) & 0x00FF00FFu;
            }
        }

        /* store the row */
        const uint32_t y = y0 + r;
        if (MODE == L3_MODE_HWC) {
            uint8_t* dst = d.out + (size_t)y * d.row_stride + (size_t)(x0 + xpix) * 3;
            if (nvalid == PPL) {
                if (PPL == 4) {
                    U32x3u v;
                    v.a = byte_of(cur[0][0], 0) | (byte_of(cur[1][0], 0) << 8) |
                          (byte_of(cur[2][0], 0) << 16) | (byte_of(cur[0][0], 1) << 24);
                    v.b = byte_of(cur[1][0], 1) | (byte_of(cur[2][0], 1) << 8) |
                          (byte_of(cur[0][NP - 1], 0) << 16) | (byte_of(cur[1][NP - 1], 0) << 24);
                    v.c = byte_of(cur[2][NP - 1], 0) | (byte_of(cur[0][NP - 1], 1) << 8) |
                          (byte_of(cur[1][NP - 1], 1) << 16) | (byte_of(cur[2][NP - 1], 1) << 24);
                    *reinterpret_cast<U32x3u*>(dst) = v;
                } else {
                    const uint32_t a = byte_of(cur[0][0], 0) | (byte_of(cur[1][0], 0) << 8) |
                                       (byte_of(cur[2][0], 0) << 16) | (byte_of(cur[0][0], 1) << 24);
                    const uint32_t b = byte_of(cur[1][0], 1) | (byte_of(cur[2][0], 1) << 8);
                    reinterpret_cast<U32u*>(dst)->v = a;
                    reinterpret_cast<U16u*>(dst + 4)->v = (uint16_t)b;
                }
            } else {
#pragma unroll
                for (int k = 0; k < PPL; ++k)
                    if ((uint32_t)k < nvalid) {
#pragma unroll
                        for (int c = 0; c < 3; ++c) dst[3 * k + c] = (uint8_t)byte_of(cur[c][k >> 1], k & 1);
                    }
            }
        } else if (MODE == L3_MODE_CHW) {
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                uint8_t* dst = d.out + (size_t)c * d.plane_stride + (size_t)y * d.row_stride + x0 + xpix;
                if (nvalid == PPL) {
                    if (PPL == 4) {
                        reinterpret_cast<U32u*>(dst)->v =
                            byte_of(cur[c][0], 0) | (byte_of(cur[c][0], 1) << 8) |
                            (byte_of(cur[c][NP - 1], 0) << 16) | (byte_of(cur[c][NP - 1], 1) << 24);
                    } else {
                        reinterpret_cast<U16u*>(dst)->v =
                            (uint16_t)(byte_of(cur[c][0], 0) | (byte_of(cur[c][0], 1) << 8));
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < PPL; ++k)
                        if ((uint32_t)k < nvalid) dst[k] = (uint8_t)byte_of(cur[c][k >> 1], k & 1);
                }
            }
        } else {
            /* tensor mode: window test, optional mirror, table of the 256 normalised values */
            const int32_t row = (int32_t)y - d.crop_y0;
            if (row >= 0 && row < (int32_t)crop_h) {
                uint16_t* out16 = reinterpret_cast<uint16_t*>(d.out);
#pragma unroll
                for (int k = 0; k < PPL; ++k) {
                    int32_t col = (int32_t)(x0 + xpix + k) - d.crop_x0;
                    if ((uint32_t)k < nvalid && col >= 0 && col < (int32_t)crop_w) {
                        if (d.flip) col = (int32_t)crop_w - 1 - col;
#pragma unroll
                        for (int c = 0; c < 3; ++c)
                            out16[((size_t)c * crop_h + row) * crop_w + col] =
                                s_lut[c * 256 + byte_of(cur[c][k >> 1], k & 1)];
                    }
                }
            }
        }

#pragma unroll
        for (int c = 0; c < 3; ++c)
#pragma unroll
            for (int j = 0; j < NP; ++j) prev[c][j] = cur[c][j];
    }

#pragma unroll
    for (int c = 0; c < 3; ++c)
        if (bitpos[c] > endbit[c]) flags |= L3_STATUS_OVERRUN;
    if (flags && active && status) atomicOr(&status[d.status_index], flags);
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

/* ---- host side: context, planning, launch ------------------------------- */

constexpr int kSlots = 4;   /* descriptor staging slots: calls in flight before the host waits */

int pixels_per_lane() {
    static int v = [] {
        const char* e = std::getenv("L3_PIXELS_PER_LANE");
        return (e && e[0] == '2' && e[1] == 0) ? 2 : 4;
    }();
    return v;
}

typedef void (*decode_kernel_t)(const L3ImageDesc*, uint32_t*, uint32_t, uint32_t, const uint16_t*);

template <int N, int PPL>
decode_kernel_t kernel_for_mode(int mode) {
    switch (mode) {
        case L3_MODE_HWC: return l3_decode_kernel<N, PPL, L3_MODE_HWC>;
        case L3_MODE_CHW: return l3_decode_kernel<N, PPL, L3_MODE_CHW>;
        default: return l3_decode_kernel<N, PPL, L3_MODE_TENSOR>;
    }
}

decode_kernel_t pick_kernel(int n, int ppl, int mode, int* tiles_per_wave) {
    if (ppl == 2) {
        if (n == 32) { *tiles_per_wave = Geom<32, 2>::TPW; return kernel_for_mode<32, 2>(mode); }
        if (n == 64) { *tiles_per_wave = Geom<64, 2>::TPW; return kernel_for_mode<64, 2>(mode); }
        *tiles_per_wave = Geom<128, 2>::TPW; return kernel_for_mode<128, 2>(mode);
    }
    if (n == 32) { *tiles_per_wave = Geom<32, 4>::TPW; return kernel_for_mode<32, 4>(mode); }
    if (n == 64) { *tiles_per_wave = Geom<64, 4>::TPW; return kernel_for_mode<64, 4>(mode); }
    *tiles_per_wave = Geom<128, 4>::TPW; return kernel_for_mode<128, 4>(mode);
}

}  // namespace

struct l3_ctx {
    int device = 0;
    size_t cap = 0;                       /* descriptors per slot */
    L3ImageDesc* h_stage[kSlots] = {};    /* pinned host */
    L3ImageDesc* d_descs[kSlots] = {};    /* device */
    uint16_t* d_table[kSlots] = {};       /* device: 768-entry normalisation table */
    hipEvent_t done[kSlots] = {};
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
    l3_status st = ensure_capacity(ctx, (size_t)n);
    if (st != L3_OK) return st;

    const int slot = ctx->next;
    if (ctx->pending[slot]) {
        if (hipEventSynchronize(ctx->done[slot]) != hipSuccess) return L3_ERR_DEVICE;
        ctx->pending[slot] = false;
    }
    L3ImageDesc* stage = ctx->h_stage[slot];

    /* descriptors grouped by patch size: classes 32, 64, 128 in this order */
    static const int kClasses[3] = {32, 64, 128};
    int class_begin[4] = {0, 0, 0, 0};
    const int ppl = pixels_per_lane();
    int filled = 0;
    uint32_t max_units[3] = {0, 0, 0};
    for (int k = 0; k < 3; ++k) {
        class_begin[k] = filled;
        int tpw = 1;
        (void)pick_kernel(kClasses[k], ppl, mode, &tpw);
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

    L3ImageDesc* d_descs = ctx->d_descs[slot];
    if (hipMemcpyAsync(d_descs, stage, (size_t)n * sizeof(L3ImageDesc), hipMemcpyHostToDevice,
                       stream) != hipSuccess)
        return L3_ERR_DEVICE;
    if (d_status)
        hipLaunchKernelGGL(l3_fill_u32_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, d_status,
                           (uint32_t)n, 0u);
    const uint16_t* table = nullptr;
    if (mode == L3_MODE_TENSOR) {
        hipLaunchKernelGGL(l3_build_table_kernel, dim3(3), dim3(256), 0, stream, mean[0], mean[1],
                           mean[2], stdv[0], stdv[1], stdv[2], dtype, ctx->d_table[slot]);
        table = ctx->d_table[slot];
    }
    for (int k = 0; k < 3; ++k) {
        const int count = class_begin[k + 1] - class_begin[k];
        if (count == 0 || max_units[k] == 0) continue;
        int tpw = 1;
        decode_kernel_t kern = pick_kernel(kClasses[k], ppl, mode, &tpw);
        const uint32_t gx = (max_units[k] + kWavesPerBlock - 1) / kWavesPerBlock;
        for (int first = 0; first < count; first += 65535) {
            const int m = count - first < 65535 ? count - first : 65535;
            hipLaunchKernelGGL(kern, dim3(gx, (uint32_t)m), dim3(64 * kWavesPerBlock), 0, stream,
                               d_descs + class_begin[k] + first, d_status, crop_w, crop_h, table);
        }
    }
    if (hipGetLastError() != hipSuccess) return L3_ERR_DEVICE;
    if (hipEventRecord(ctx->done[slot], stream) != hipSuccess) return L3_ERR_DEVICE;
    ctx->pending[slot] = true;
    ctx->next = (slot + 1) % kSlots;
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
