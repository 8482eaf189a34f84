/*
 * Decoder variants for the ablation of arxiv 2208.08711 Section 5.5 (see
 * include/l3_ablation.h).  Deliberately plain: one wave per patch of one channel,
 * the patch stream copied to local memory, then the two stages of Section 4.2 in
 * decoding order, each either by all lanes or by lane 0 alone, then the write-out.
 * The variants share everything except who does the work of a stage, so that the
 * differences measured between them are the differences Section 5.5 is about.
 * The tuned decoder is in l3_device.hip and shares no kernel code with this file.
 */
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <vector>

#include "l3_ablation.h"
#include "l3_ctx.h"

namespace {

constexpr int kMaxN = 128;
constexpr int kLanes = 64;
/* longest canonical stream of a patch: N rows of 12 + 8N bits, rounded up */
constexpr uint32_t kMaxStream = kMaxN * kMaxN + (12 * kMaxN + 7) / 8;
constexpr uint32_t kStreamWords = (kMaxStream + 3) / 4 + 2;   /* zero-filled slack for 32-bit peeks */

struct AblationDesc {
    const uint8_t* file;
    uint8_t* out;
    uint64_t file_len;
    uint64_t row_stride;
    uint32_t width, height;
    uint32_t n;                 /* patch size */
    uint32_t tiles_x, tiles_y;
    uint32_t header_bytes;
};

__device__ __forceinline__ uint32_t read_u32_bytes(const uint8_t* p) {
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24);
}

/* The 32 stream bits from bit `pos` on (at least 25 of them valid).  Past the end of a
 * patch's copy the buffer holds zeros, then whatever an earlier patch left: only a
 * damaged stream looks there. */
__device__ __forceinline__ uint32_t peek_bits(const uint32_t* words, uint32_t pos) {
    const uint32_t wi = pos >> 5, sh = pos & 31u;
    if (wi + 1 >= kStreamWords) return 0;
    const uint64_t two = (uint64_t)words[wi] | ((uint64_t)words[wi + 1] << 32);
    return (uint32_t)(two >> sh);
}

/* Section 4.2, custom filter: nearest of top-left, top-right, top to TL + TR - T. */
__device__ __forceinline__ int select_custom(int tl, int t, int tr) {
    const int d_tl = abs(tr - t), d_tr = abs(tl - t), d_t = abs(tl + tr - 2 * t);
    if (d_tl <= d_tr && d_tl <= d_t) return tl;
    return d_tr <= d_t ? tr : t;
}

/* The original filter: nearest of left, top, top-left to L + T - C. */
__device__ __forceinline__ int select_original(int left, int top, int corner) {
    const int d_l = abs(top - corner), d_t = abs(left - corner), d_c = abs(left + top - 2 * corner);
    if (d_l <= d_t && d_l <= d_c) return left;
    return d_t <= d_c ? top : corner;
}

template <bool PIXEL_BD, bool CUSTOM>
__global__ __launch_bounds__(kLanes) void l3_ablation_kernel(const AblationDesc* __restrict__ descs,
                                                             int serial_patches, int diagonal) {
    __shared__ uint32_t s_stream[kStreamWords];
    __shared__ uint8_t s_pix[kMaxN * kMaxN];

    const AblationDesc d = descs[blockIdx.y];
    const uint32_t lane = threadIdx.x;
    const uint32_t n = d.n;
    const uint32_t patches = d.tiles_x * d.tiles_y;
    const uint32_t per_image = 3 * patches;
    const uint32_t data_len = (uint32_t)(d.file_len - d.header_bytes);
    const uint32_t first = serial_patches ? 0u : blockIdx.x;
    const uint32_t last = serial_patches ? per_image : min(blockIdx.x + 1u, per_image);

    for (uint32_t unit = first; unit < last; ++unit) {
        const uint32_t c = unit / patches, i = unit - c * patches;
        const uint32_t ty = i / d.tiles_x, tx = i - ty * d.tiles_x;
        const uint32_t x0 = tx * n, y0 = ty * n;
        const uint32_t pw = min(n, d.width - x0), ph = min(n, d.height - y0);

        /* Section 4.3: the patch's byte range from the offset array */
        uint32_t off = read_u32_bytes(d.file + 13 + 4 * (size_t)unit);
        uint32_t end = unit + 1 < per_image ? read_u32_bytes(d.file + 13 + 4 * (size_t)(unit + 1))
                                            : data_len;
        off = min(off, data_len);
        end = min(max(end, off), data_len);
        const uint32_t len = min(end - off, kMaxStream);
        const uint8_t* src = d.file + d.header_bytes + off;

        /* the stream into local memory (all lanes, whatever the variant) */
        const uint32_t copy_words = min(kStreamWords, len / 4 + 3);   /* zero-filled past the end */
        for (uint32_t w = lane; w < copy_words; w += kLanes) {
            uint32_t v = 0;
            for (uint32_t b = 0; b < 4; ++b) {
                const uint32_t k = 4 * w + b;
                if (k < len) v |= (uint32_t)src[k] << (8 * b);
            }
            s_stream[w] = v;
        }
        __syncthreads();

        /* stage 1 of decoding: base-delta, residuals into s_pix */
        if (PIXEL_BD) {
            uint32_t bitpos = 0;
            for (uint32_t r = 0; r < ph; ++r) {
                const uint32_t hdr = peek_bits(s_stream, bitpos);
                const uint32_t w = hdr & 15u, base = (hdr >> 4) & 255u;
                const uint32_t mask = (1u << w) - 1u;
                for (uint32_t x = lane; x < pw; x += kLanes)
                    s_pix[r * n + x] = (uint8_t)(base + (peek_bits(s_stream, bitpos + 12 + x * w) & mask));
                bitpos += 12 + pw * w;
            }
        } else if (lane == 0) {
            uint32_t bitpos = 0;
            for (uint32_t r = 0; r < ph; ++r) {
                const uint32_t hdr = peek_bits(s_stream, bitpos);
                const uint32_t w = hdr & 15u, base = (hdr >> 4) & 255u;
                const uint32_t mask = (1u << w) - 1u;
                bitpos += 12;
                for (uint32_t x = 0; x < pw; ++x) {
                    s_pix[r * n + x] = (uint8_t)(base + (peek_bits(s_stream, bitpos) & mask));
                    bitpos += w;
                }
            }
        }
        __syncthreads();

        /* stage 2 of decoding: the inverse filter, in place (row 0 is raw) */
        if (CUSTOM) {
            for (uint32_t r = 1; r < ph; ++r) {
                const uint8_t* up = &s_pix[(r - 1) * n];
                for (uint32_t x = lane; x < pw; x += kLanes) {
                    const int pred = (x == 0 || x + 1 == pw) ? up[x]
                                                             : select_custom(up[x - 1], up[x], up[x + 1]);
                    s_pix[r * n + x] = (uint8_t)(s_pix[r * n + x] + pred);
                }
                __syncthreads();
            }
        } else if (diagonal) {
            /* the original filter's dependencies (left, top, top-left) all point to the two
             * previous anti-diagonals x + y = d - 1, d - 2: one diagonal per step, its pixels
             * in parallel */
            for (uint32_t d = 1; d + 1 < pw + ph; ++d) {
                for (uint32_t x = lane; x < pw; x += kLanes) {
                    const uint32_t y = d - x;              /* wraps to a huge value when x > d */
                    if (y >= 1 && y < ph) {
                        uint8_t* cur = &s_pix[y * n];
                        const uint8_t* up = cur - n;
                        const int pred = x == 0 ? up[0] : select_original(cur[x - 1], up[x], up[x - 1]);
                        cur[x] = (uint8_t)(cur[x] + pred);
                    }
                }
                __syncthreads();
            }
        } else if (lane == 0) {
            for (uint32_t r = 1; r < ph; ++r) {
                const uint8_t* up = &s_pix[(r - 1) * n];
                uint8_t* cur = &s_pix[r * n];
                cur[0] = (uint8_t)(cur[0] + up[0]);
                for (uint32_t x = 1; x < pw; ++x)
                    cur[x] = (uint8_t)(cur[x] + select_original(cur[x - 1], up[x], up[x - 1]));
            }
        }
        __syncthreads();

        /* write-out: interleaved RGB, channel c */
        for (uint32_t r = 0; r < ph; ++r) {
            uint8_t* dst = d.out + (size_t)(y0 + r) * d.row_stride + (size_t)x0 * 3 + c;
            for (uint32_t x = lane; x < pw; x += kLanes) dst[3 * (size_t)x] = s_pix[r * n + x];
        }
        __syncthreads();   /* local memory is reused by the next patch */
    }
}

}  // namespace

struct L3AblationState {
    AblationDesc* d_descs = nullptr;
    size_t cap = 0;
    std::vector<AblationDesc> uploaded;   /* what d_descs holds */
};

void l3_ablation_state_free(L3AblationState* s) {
    if (!s) return;
    if (s->d_descs) (void)hipFree(s->d_descs);
    delete s;
}

extern "C" l3_status l3_ablation_decode_batch(l3_ctx* ctx, const l3_item* items, int n, int variant,
                                              void* stream_v) {
    if (!ctx || n < 0 || (n > 0 && !items) || (variant & ~15)) return L3_ERR_INVALID_ARG;
    if ((variant & L3_ABLATION_DIAGONAL) && (variant & L3_ABLATION_CUSTOM_FILTER))
        return L3_ERR_INVALID_ARG;
    if (n == 0) return L3_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return L3_ERR_DEVICE;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);

    std::vector<AblationDesc> descs((size_t)n);
    uint32_t max_units = 0;
    for (int i = 0; i < n; ++i) {
        const l3_item& it = items[i];
        const uint32_t w = it.info.width, h = it.info.height, pn = it.info.patch;
        if (!it.d_file || !it.d_out || w == 0 || h == 0 || pn == 0) return L3_ERR_INVALID_ARG;
        if (pn > kMaxN) return L3_ERR_UNSUPPORTED;
        const uint64_t tx = (w + pn - 1) / pn, ty = (h + pn - 1) / pn, p = tx * ty;
        if (p > 0x7FFFFFFFull / 3 || it.info.patches_per_channel != p ||
            it.info.header_bytes != 13 + 12 * p || it.file_len <= it.info.header_bytes ||
            it.file_len - it.info.header_bytes > 0xFFFFFFFFull ||
            it.out_row_stride < (size_t)w * 3)
            return L3_ERR_INVALID_ARG;
        AblationDesc& d = descs[(size_t)i];
        std::memset(&d, 0, sizeof d);   /* padding too: the table is compared bytewise */
        d.file = it.d_file;
        d.out = it.d_out;
        d.file_len = it.file_len;
        d.row_stride = it.out_row_stride;
        d.width = w;
        d.height = h;
        d.n = pn;
        d.tiles_x = (uint32_t)tx;
        d.tiles_y = (uint32_t)ty;
        d.header_bytes = (uint32_t)it.info.header_bytes;
        if (3 * (uint32_t)p > max_units) max_units = 3 * (uint32_t)p;
    }

    if (!ctx->abl) {
        ctx->abl = new (std::nothrow) L3AblationState;
        if (!ctx->abl) return L3_ERR_DEVICE;
    }
    L3AblationState* st = ctx->abl;
    if (st->cap < (size_t)n) {
        /* earlier launches may still read the old table */
        if (hipDeviceSynchronize() != hipSuccess) return L3_ERR_DEVICE;
        if (st->d_descs) (void)hipFree(st->d_descs);
        st->d_descs = nullptr;
        st->cap = 0;
        st->uploaded.clear();
        if (hipMalloc(reinterpret_cast<void**>(&st->d_descs), (size_t)n * sizeof(AblationDesc)) !=
            hipSuccess)
            return L3_ERR_DEVICE;
        st->cap = (size_t)n;
    }
    /* The table is uploaded only when it differs from the one already there (a timing
     * loop repeats one batch).  Blocking, after everything enqueued on the device: an
     * earlier launch may still read the old table. */
    if (st->uploaded.size() != descs.size() ||
        std::memcmp(st->uploaded.data(), descs.data(), descs.size() * sizeof(AblationDesc)) != 0) {
        st->uploaded.clear();
        if (hipDeviceSynchronize() != hipSuccess ||
            hipMemcpy(st->d_descs, descs.data(), (size_t)n * sizeof(AblationDesc),
                      hipMemcpyHostToDevice) != hipSuccess)
            return L3_ERR_DEVICE;
        st->uploaded = descs;
    }

    const int serial = (variant & L3_ABLATION_SERIAL_PATCHES) ? 1 : 0;
    const int diagonal = (variant & L3_ABLATION_DIAGONAL) ? 1 : 0;
    const dim3 grid(serial ? 1u : max_units, (uint32_t)n), block(kLanes);
    const bool pixel_bd = variant & L3_ABLATION_PIXEL_BD, custom = variant & L3_ABLATION_CUSTOM_FILTER;
    if (pixel_bd && custom)
        hipLaunchKernelGGL((l3_ablation_kernel<true, true>), grid, block, 0, stream, st->d_descs, serial, diagonal);
    else if (pixel_bd)
        hipLaunchKernelGGL((l3_ablation_kernel<true, false>), grid, block, 0, stream, st->d_descs, serial, diagonal);
    else if (custom)
        hipLaunchKernelGGL((l3_ablation_kernel<false, true>), grid, block, 0, stream, st->d_descs, serial, diagonal);
    else
        hipLaunchKernelGGL((l3_ablation_kernel<false, false>), grid, block, 0, stream, st->d_descs, serial, diagonal);
    return hipGetLastError() == hipSuccess ? L3_OK : L3_ERR_DEVICE;
}
