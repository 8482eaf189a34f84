/*
 * Host-only part of the L3 library: status strings, the patch-size rule, the
 * CPU encoder and the header parser/validator.  No GPU call in this file.
 * Format: arxiv 2208.08711 Section 4.2 (two-stage patch coding) and Section 4.3
 * (file layout); conventions fixed by this library are listed in include/l3.h.
 */
#include <cstring>
#include <vector>

#include "l3_internal.h"
#include "l3_ablation.h"

namespace {

constexpr uint8_t kSignature[4] = {0x4C, 0x33, 0x00, 0x01};
constexpr size_t kFixedHeader = 13;

inline uint32_t rd32(const uint8_t* p) {
    uint32_t v;
    std::memcpy(&v, p, 4);   /* little-endian host */
    return v;
}
inline void wr32(uint8_t* p, uint32_t v) { std::memcpy(p, &v, 4); }

inline uint32_t tiles(uint32_t extent, uint32_t n) { return extent / n + (extent % n != 0); }

/* Appends bit fields, least significant bit first, to a byte buffer. */
class BitSink {
public:
    explicit BitSink(std::vector<uint8_t>& dst) : dst_(dst) {}
    void put(uint32_t value, unsigned nbits) {
        acc_ |= (uint64_t)value << fill_;
        fill_ += nbits;
        while (fill_ >= 8) {
            dst_.push_back((uint8_t)acc_);
            acc_ >>= 8;
            fill_ -= 8;
        }
    }
    void flush_to_byte() {
        if (fill_) dst_.push_back((uint8_t)acc_);
        acc_ = 0;
        fill_ = 0;
    }
private:
    std::vector<uint8_t>& dst_;
    uint64_t acc_ = 0;
    unsigned fill_ = 0;
};

/* Section 4.2 stage 1: which of the three upper neighbours is nearest to
 * TL + TR - T.  Distances are |TR-T| (for TL), |TL-T| (for TR), |TL+TR-2T| (for T). */
inline int nearest_upper(int tl, int t, int tr) {
    int d_tl = tr > t ? tr - t : t - tr;
    int d_tr = tl > t ? tl - t : t - tl;
    int s = tl + tr - 2 * t;
    int d_t = s < 0 ? -s : s;
    if (d_tl <= d_tr && d_tl <= d_t) return tl;
    return d_tr <= d_t ? tr : t;
}

inline unsigned bits_for(unsigned range) {
    unsigned n = 0;
    while (range >> n) ++n;
    return n;
}

/* Section 4.2, the filter the custom one replaces: nearest of left, top, top-left to
 * left + top - top_left, ties in that order.  Distances are |T-C| (for L), |L-C| (for T)
 * and |L+T-2C| (for C = top-left). */
inline int nearest_original(int left, int top, int corner) {
    int d_l = top > corner ? top - corner : corner - top;
    int d_t = left > corner ? left - corner : corner - left;
    int s = left + top - 2 * corner;
    int d_c = s < 0 ? -s : s;
    if (d_l <= d_t && d_l <= d_c) return left;
    return d_t <= d_c ? top : corner;
}

/* Encodes one pw x ph patch held as a dense plane.  original_filter selects the
 * left/top/top-left predictor (ablation baseline of Section 5.5) for rows >= 1. */
void encode_plane_patch(const uint8_t* plane, uint32_t pw, uint32_t ph, bool original_filter,
                        std::vector<uint8_t>& dst, std::vector<int>& row) {
    BitSink sink(dst);
    row.resize(pw);
    for (uint32_t y = 0; y < ph; ++y) {
        const uint8_t* cur = plane + (size_t)y * pw;
        const uint8_t* up = cur - pw;
        int vmin, vmax;
        if (y == 0) {
            for (uint32_t x = 0; x < pw; ++x) row[x] = cur[x];
        } else if (original_filter) {
            row[0] = (int8_t)(uint8_t)(cur[0] - up[0]);
            for (uint32_t x = 1; x < pw; ++x)
                row[x] = (int8_t)(uint8_t)(cur[x] - nearest_original(cur[x - 1], up[x], up[x - 1]));
        } else {
            row[0] = (int8_t)(uint8_t)(cur[0] - up[0]);
            for (uint32_t x = 1; x + 1 < pw; ++x)
                row[x] = (int8_t)(uint8_t)(cur[x] - nearest_upper(up[x - 1], up[x], up[x + 1]));
            if (pw > 1) row[pw - 1] = (int8_t)(uint8_t)(cur[pw - 1] - up[pw - 1]);
        }
        vmin = vmax = row[0];
        for (uint32_t x = 1; x < pw; ++x) {
            if (row[x] < vmin) vmin = row[x];
            if (row[x] > vmax) vmax = row[x];
        }
        unsigned width = bits_for((unsigned)(vmax - vmin));
        sink.put(width | (((uint32_t)vmin & 0xFFu) << 4), 12);
        if (width)
            for (uint32_t x = 0; x < pw; ++x) sink.put((uint32_t)(row[x] - vmin), width);
    }
    sink.flush_to_byte();
}

/* binary32 -> binary16 bits, round to nearest, ties to even (subnormals, overflow to
 * infinity; a NaN stays a quiet NaN with the top of its payload) */
uint16_t f32_to_f16_bits(float f) {
    uint32_t x;
    std::memcpy(&x, &f, 4);
    const uint32_t sign = (x >> 16) & 0x8000u;
    x &= 0x7FFFFFFFu;
    if (x > 0x7F800000u) return (uint16_t)(sign | 0x7E00u | ((x >> 13) & 0x01FFu));
    if (x >= 0x47800000u) return (uint16_t)(sign | 0x7C00u);   /* 65536 and beyond, infinity */
    if (x >= 0x38800000u) {                                    /* a normal binary16: 2^-14 and beyond */
        uint32_t h = (((x >> 23) - 112u) << 10) | ((x & 0x007FFFFFu) >> 13);
        const uint32_t rest = x & 0x1FFFu;
        if (rest > 0x1000u || (rest == 0x1000u && (h & 1u))) ++h;   /* may carry up to infinity: correct */
        return (uint16_t)(sign | h);
    }
    if (x < 0x33000000u) return (uint16_t)sign;                /* below 2^-25: zero (2^-25 itself ties to zero) */
    const uint32_t mant = (x & 0x007FFFFFu) | 0x00800000u;     /* a subnormal binary16: units of 2^-24 */
    const uint32_t shift = 126u - (x >> 23);                   /* 14 .. 24 */
    uint32_t h = mant >> shift;
    const uint32_t rest = mant & ((1u << shift) - 1u), half = 1u << (shift - 1u);
    if (rest > half || (rest == half && (h & 1u))) ++h;
    return (uint16_t)(sign | h);
}

uint16_t f32_to_bf16_bits(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

}  // namespace

extern "C" {

l3_status l3_normalized_values(const float mean[3], const float stdv[3], l3_dtype dtype,
                               uint16_t out[768]) {
    if (!mean || !stdv || !out || (dtype != L3_BF16 && dtype != L3_FP16)) return L3_ERR_INVALID_ARG;
    for (int c = 0; c < 3; ++c)
        for (int v = 0; v < 256; ++v) {
            /* three roundings, none fused: the build switches contraction off */
            const float scaled = (float)v / 255.0f;
            const float centred = scaled - mean[c];
            const float y = centred / stdv[c];
            out[c * 256 + v] = dtype == L3_BF16 ? f32_to_bf16_bits(y) : f32_to_f16_bits(y);
        }
    return L3_OK;
}

const char* l3_status_string(l3_status s) {
    switch (s) {
        case L3_OK: return "ok";
        case L3_ERR_INVALID_ARG: return "invalid argument";
        case L3_ERR_BAD_MAGIC: return "not an L3 file (bad signature)";
        case L3_ERR_TRUNCATED: return "buffer shorter than the L3 header";
        case L3_ERR_CORRUPT: return "inconsistent L3 header or patch offsets";
        case L3_ERR_BUFFER_TOO_SMALL: return "output buffer too small";
        case L3_ERR_UNSUPPORTED: return "not supported by this build";
        case L3_ERR_DEVICE: return "HIP runtime error or no usable GPU";
        case L3_ERR_LIMIT: return "request exceeds a fixed limit of the entry point";
    }
    return "unknown status";
}

uint8_t l3_default_patch(uint32_t width, uint32_t height) {
    const uint64_t px = (uint64_t)width * height;
    if (px < 1080ull * 720ull) return 32;
    if (px <= 1920ull * 1080ull) return 64;
    return 128;
}

size_t l3_encode_bound(uint32_t width, uint32_t height, uint8_t patch) {
    if (width == 0 || height == 0) return 0;
    const uint32_t n = patch ? patch : l3_default_patch(width, height);
    const uint64_t tx = tiles(width, n), ty = tiles(height, n);
    /* a patch row costs at most 12 + 8*pw bits; one byte of padding per patch */
    const uint64_t per_channel = (uint64_t)width * height + 2ull * height * tx + tx * ty;
    return (size_t)(kFixedHeader + 12ull * tx * ty + 3ull * per_channel);
}

}  // extern "C"

namespace {
l3_status encode_file(const uint8_t* rgb, uint32_t width, uint32_t height, size_t row_stride,
                      uint8_t patch, bool original_filter, uint8_t* out, size_t out_cap,
                      size_t* out_len) {
    if (!rgb || !out || !out_len || width == 0 || height == 0 ||
        row_stride < (size_t)width * 3)
        return L3_ERR_INVALID_ARG;
    const uint32_t n = patch ? patch : l3_default_patch(width, height);
    const uint32_t tx = tiles(width, n), ty = tiles(height, n);
    const uint64_t p = (uint64_t)tx * ty;
    const uint64_t header = kFixedHeader + 12 * p;
    if (out_cap < header) return L3_ERR_BUFFER_TOO_SMALL;

    std::memcpy(out, kSignature, 4);
    wr32(out + 4, width);
    wr32(out + 8, height);
    out[12] = (uint8_t)n;

    std::vector<uint8_t> plane((size_t)n * n), coded;
    std::vector<int> row;
    uint64_t pos = 0;   /* bytes of the data section written so far */
    for (uint32_t c = 0; c < 3; ++c)
        for (uint32_t j = 0; j < ty; ++j)
            for (uint32_t i = 0; i < tx; ++i) {
                const uint32_t x0 = i * n, y0 = j * n;
                const uint32_t pw = width - x0 < n ? width - x0 : n;
                const uint32_t ph = height - y0 < n ? height - y0 : n;
                for (uint32_t y = 0; y < ph; ++y) {
                    const uint8_t* src = rgb + (size_t)(y0 + y) * row_stride + (size_t)x0 * 3 + c;
                    for (uint32_t x = 0; x < pw; ++x) plane[(size_t)y * pw + x] = src[3 * (size_t)x];
                }
                coded.clear();
                encode_plane_patch(plane.data(), pw, ph, original_filter, coded, row);
                if (pos > 0xFFFFFFFFull) return L3_ERR_UNSUPPORTED;
                if (header + pos + coded.size() > out_cap) return L3_ERR_BUFFER_TOO_SMALL;
                wr32(out + kFixedHeader + 4 * ((uint64_t)c * p + (uint64_t)j * tx + i), (uint32_t)pos);
                std::memcpy(out + header + pos, coded.data(), coded.size());
                pos += coded.size();
            }
    *out_len = (size_t)(header + pos);
    return L3_OK;
}
}  // namespace

extern "C" {

l3_status l3_encode_cpu(const uint8_t* rgb, uint32_t width, uint32_t height, size_t row_stride,
                        uint8_t patch, uint8_t* out, size_t out_cap, size_t* out_len) {
    return encode_file(rgb, width, height, row_stride, patch, false, out, out_cap, out_len);
}

l3_status l3_ablation_encode_cpu(const uint8_t* rgb, uint32_t width, uint32_t height,
                                 size_t row_stride, uint8_t patch, int original_filter,
                                 uint8_t* out, size_t out_cap, size_t* out_len) {
    return encode_file(rgb, width, height, row_stride, patch, original_filter != 0, out, out_cap,
                       out_len);
}

l3_status l3_peek_header(const uint8_t* file, size_t len, l3_info* info) {
    if (!file || !info) return L3_ERR_INVALID_ARG;
    if (len < kFixedHeader) return L3_ERR_TRUNCATED;
    if (std::memcmp(file, kSignature, 4) != 0) return L3_ERR_BAD_MAGIC;
    const uint32_t w = rd32(file + 4), h = rd32(file + 8), n = file[12];
    if (w == 0 || h == 0 || n == 0) return L3_ERR_CORRUPT;
    const uint64_t tx = tiles(w, n), ty = tiles(h, n), p = tx * ty;
    if (p > 0x7FFFFFFFull / 3) return L3_ERR_CORRUPT;
    const uint64_t header = kFixedHeader + 12 * p;
    if (len < header) return L3_ERR_TRUNCATED;
    const uint64_t data_len = len - header;
    if (data_len > 0xFFFFFFFFull) return L3_ERR_CORRUPT;

    /* offsets: start at 0, strictly increasing, each patch long enough for the
     * 12-bit records of its rows, the last one ending at the end of the file */
    uint64_t prev = 0;
    for (uint64_t k = 0; k < 3 * p; ++k) {
        const uint64_t off = rd32(file + kFixedHeader + 4 * k);
        if (k == 0 ? off != 0 : off <= prev) return L3_ERR_CORRUPT;
        if (off >= data_len) return L3_ERR_CORRUPT;
        const uint64_t next = k + 1 < 3 * p ? rd32(file + kFixedHeader + 4 * (k + 1)) : data_len;
        const uint64_t j = (k % p) / tx;
        const uint64_t ph = (j + 1) * n <= h ? n : h - j * n;
        if (next < off || next - off < (12 * ph + 7) / 8) return L3_ERR_CORRUPT;
        prev = off;
    }
    info->width = w;
    info->height = h;
    info->patch = (uint8_t)n;
    info->patches_per_channel = (uint32_t)p;
    info->header_bytes = (size_t)header;
    return L3_OK;
}

}  // extern "C"

void l3_plan_units(L3ImageDesc* d, uint32_t patch, uint32_t tpw, bool flat_ok) {
    d->tile_x_first = d->tile_y_first = 0;
    d->tile_x_count = d->tiles_x;
    d->groups_x = (d->tiles_x + tpw - 1) / tpw;
    d->units = d->groups_x * d->tiles_y;
    d->flat_upper_rows = d->flat_upper_units = 0;
    /* Flat order where it saves units: patches taken in row-major order across the ends
     * of patch rows.  The lanes' 32-bit byte offsets must reach tpw patch rows down. */
    const uint64_t reach = (uint64_t)(tpw + 1) * patch * d->row_stride + 3ull * d->width;
    const uint64_t all = (uint64_t)d->tiles_x * d->tiles_y;
    if (!flat_ok || reach >= 0xFFFFFFFFull || all >= 0x7FFFFFFFull) return;
    const uint32_t upper_rows = (d->height % patch != 0 && d->tiles_y > 1) ? d->tiles_y - 1 : d->tiles_y;
    const uint32_t upper_units = (uint32_t)(((uint64_t)d->tiles_x * upper_rows + tpw - 1) / tpw);
    const uint32_t units = upper_units + (upper_rows < d->tiles_y ? (d->tiles_x + tpw - 1) / tpw : 0u);
    if (units < d->units) {
        d->groups_x = 0;
        d->units = units;
        d->flat_upper_rows = upper_rows;
        d->flat_upper_units = upper_units;
    }
}
