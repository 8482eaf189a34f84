/*
 * L3 oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT (see l3_oracle.h).
 *
 * Plain scalar C++; one pixel, one bit field at a time, in the order the
 * paper states the steps (Section 4.2 for the two stages, Section 4.3 for the
 * file).  No blocking, no tables, no intrinsics.
 */
#include "l3_oracle.h"

#include <cstdlib>
#include <cstring>
#include <vector>

namespace {

const uint8_t kMagic[4] = {0x4C, 0x33, 0x00, 0x01};

uint32_t ceil_div(uint32_t a, uint32_t b) { return (a + b - 1) / b; }

uint32_t load_u32le(const uint8_t* p) {
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) |
           ((uint32_t)p[3] << 24);
}

void store_u32le(uint8_t* p, uint32_t v) {
    p[0] = (uint8_t)v;
    p[1] = (uint8_t)(v >> 8);
    p[2] = (uint8_t)(v >> 16);
    p[3] = (uint8_t)(v >> 24);
}

/* Section 4.2, base-delta: per row a 4-bit width, an 8-bit base, then the deltas
 * at that width -- a stream of bit fields.  Bit k lives in byte k/8 at
 * bit position k%8; a field's least significant bit is written first. */
struct BitWriter {
    std::vector<uint8_t> bytes;
    uint64_t nbits = 0;
    void put(uint32_t value, unsigned width) {
        for (unsigned i = 0; i < width; ++i) {
            if ((nbits & 7) == 0) bytes.push_back(0);
            if ((value >> i) & 1u) bytes[nbits >> 3] |= (uint8_t)(1u << (nbits & 7));
            ++nbits;
        }
    }
};

struct BitReader {
    const uint8_t* bytes;
    uint64_t total_bits;
    uint64_t pos = 0;
    bool overrun = false;
    BitReader(const uint8_t* b, size_t len) : bytes(b), total_bits((uint64_t)len * 8) {}
    uint32_t get(unsigned width) {
        uint32_t v = 0;
        for (unsigned i = 0; i < width; ++i) {
            if (pos >= total_bits) { overrun = true; return 0; }
            uint32_t bit = (bytes[pos >> 3] >> (pos & 7)) & 1u;
            v |= bit << i;
            ++pos;
        }
        return v;
    }
};

/* Section 4.2, custom Paeth filter, steps 1 and 2: reference value
 * TL + TR - T, then the neighbour nearest to it. */
int predict_int(int tl, int t, int tr) {
    int ref = tl + tr - t;
    int d_tl = std::abs(ref - tl);
    int d_tr = std::abs(ref - tr);
    int d_t = std::abs(ref - t);
    if (d_tl <= d_tr && d_tl <= d_t) return tl;
    if (d_tr <= d_t) return tr;
    return t;
}

/* The predictor at column x of a patch row, from the row above it. */
int predict_at(const uint8_t* above, uint32_t x, uint32_t pw) {
    if (x == 0 || x + 1 >= pw) return above[x];
    return predict_int(above[x - 1], above[x], above[x + 1]);
}

/* Section 4.2, first paragraph of "Custom Paeth Filter": the original Paeth
 * filter, which looks at left, top and top-left.  Reference value
 * left + top - top_left, nearest of the three wins, ties in the order left,
 * top, top-left (the order PNG's filter type 4 uses). */
int predict_original_int(int left, int top, int top_left) {
    int ref = left + top - top_left;
    int d_left = std::abs(ref - left);
    int d_top = std::abs(ref - top);
    int d_tl = std::abs(ref - top_left);
    if (d_left <= d_top && d_left <= d_tl) return left;
    if (d_top <= d_tl) return top;
    return top_left;
}

/* The original predictor at column x of a row (rows >= 1), from the row above
 * and the pixels of the current row to the left.  In the first column there is
 * no left and no top-left pixel: the prediction is "top" (which is also what
 * the rule above gives when the two missing pixels count as 0). */
int predict_original_at(const uint8_t* above, const uint8_t* cur, uint32_t x) {
    if (x == 0) return above[0];
    return predict_original_int(cur[x - 1], above[x], above[x - 1]);
}

unsigned bit_length(unsigned v) {
    unsigned n = 0;
    while (v) { ++n; v >>= 1; }
    return n;
}

/* Encode one pw x ph patch of one channel (pixels at src, rows src_stride
 * apart, pixel_step bytes between pixels of a row) onto the bit writer. */
void encode_patch(const uint8_t* src, size_t src_stride, size_t pixel_step,
                  uint32_t pw, uint32_t ph, int width_mode, int predictor, BitWriter& bw) {
    std::vector<uint8_t> above(pw), cur(pw), resid(pw);
    for (uint32_t r = 0; r < ph; ++r) {
        for (uint32_t x = 0; x < pw; ++x) cur[x] = src[r * src_stride + x * pixel_step];
        /* stage 1: filter (first row skipped: kept raw) */
        for (uint32_t x = 0; x < pw; ++x) {
            if (r == 0) resid[x] = cur[x];
            else if (predictor == L3O_PREDICTOR_ORIGINAL)
                resid[x] = (uint8_t)(cur[x] - predict_original_at(above.data(), cur.data(), x));
            else resid[x] = (uint8_t)(cur[x] - predict_at(above.data(), x, pw));
        }
        /* stage 2: base-delta, steps 1-4 */
        int lo = 1 << 30, hi = -(1 << 30);
        for (uint32_t x = 0; x < pw; ++x) {
            int v = (r == 0) ? (int)resid[x] : (int)(int8_t)resid[x];
            if (v < lo) lo = v;
            if (v > hi) hi = v;
        }
        unsigned width = bit_length((unsigned)(hi - lo));
        if (width_mode == 1) width = 8;
        else if (width_mode == 2) width = width < 8 ? width + 1 : 8;
        bw.put(width, 4);
        bw.put((uint32_t)lo & 0xFFu, 8);
        for (uint32_t x = 0; x < pw; ++x) {
            int v = (r == 0) ? (int)resid[x] : (int)(int8_t)resid[x];
            bw.put((uint32_t)(v - lo), width);
        }
        above = cur;
    }
    /* every patch ends on a byte boundary: BitWriter's last byte is already
     * zero-filled above the last bit written */
    bw.nbits = (uint64_t)bw.bytes.size() * 8;
}

/* Base-delta decode of one patch stream into its residual plane. */
int unpack_patch(const uint8_t* stream, size_t len, uint32_t pw, uint32_t ph,
                 uint8_t* resid, size_t stride) {
    BitReader br(stream, len);
    for (uint32_t r = 0; r < ph; ++r) {
        uint32_t width = br.get(4);
        uint32_t base = br.get(8);
        if (br.overrun) return L3O_ERR_CORRUPT;
        if (width > 8) return L3O_ERR_CORRUPT;
        for (uint32_t x = 0; x < pw; ++x) {
            uint32_t delta = br.get(width);
            resid[r * stride + x] = (uint8_t)(base + delta);
        }
        if (br.overrun) return L3O_ERR_CORRUPT;
    }
    return L3O_OK;
}

/* Inverse filter over a residual plane, in place row by row into out. */
void unfilter_patch(const uint8_t* resid, size_t rstride, uint32_t pw, uint32_t ph,
                    int predictor, uint8_t* out, size_t ostride) {
    for (uint32_t x = 0; x < pw; ++x) out[x] = resid[x];
    for (uint32_t r = 1; r < ph; ++r) {
        const uint8_t* above = out + (size_t)(r - 1) * ostride;
        for (uint32_t x = 0; x < pw; ++x) {
            int pred = predictor == L3O_PREDICTOR_ORIGINAL
                           ? predict_original_at(above, out + (size_t)r * ostride, x)
                           : predict_at(above, x, pw);
            out[r * ostride + x] = (uint8_t)(pred + resid[r * rstride + x]);
        }
    }
}

/* Walks all patches of a parsed file; for each hands (channel, x0, y0, pw, ph,
 * stream, len) to fn.  Returns the first error. */
template <class Fn>
int for_each_patch(const uint8_t* file, size_t len, const l3o_info& info, Fn fn) {
    const uint32_t n = info.patch;
    const uint64_t patches = (uint64_t)info.px * info.py;
    const uint8_t* offsets = file + 13;
    const uint8_t* data = file + info.header_bytes;
    (void)len;
    for (uint32_t c = 0; c < 3; ++c) {
        for (uint32_t py = 0; py < info.py; ++py) {
            for (uint32_t px = 0; px < info.px; ++px) {
                uint64_t flat = (uint64_t)c * patches + (uint64_t)py * info.px + px;
                uint64_t begin = load_u32le(offsets + 4 * flat);
                uint64_t end = (flat + 1 < 3 * patches) ? load_u32le(offsets + 4 * (flat + 1))
                                                         : info.data_bytes;
                if (begin > end || end > info.data_bytes) return L3O_ERR_CORRUPT;
                uint32_t x0 = px * n, y0 = py * n;
                uint32_t pw = (info.width - x0 < n) ? info.width - x0 : n;
                uint32_t ph = (info.height - y0 < n) ? info.height - y0 : n;
                int rc = fn(c, x0, y0, pw, ph, data + begin, (size_t)(end - begin));
                if (rc != L3O_OK) return rc;
            }
        }
    }
    return L3O_OK;
}

uint32_t f32_bits(float x) {
    uint32_t u;
    std::memcpy(&u, &x, 4);
    return u;
}

}  // namespace

extern "C" {

uint32_t l3o_patch_rule(uint32_t width, uint32_t height) {
    uint64_t pixels = (uint64_t)width * height;
    if (pixels < (uint64_t)1080 * 720) return 32;
    if (pixels <= (uint64_t)1920 * 1080) return 64;
    return 128;
}

uint8_t l3o_predict(uint8_t tl, uint8_t t, uint8_t tr) {
    return (uint8_t)predict_int(tl, t, tr);
}

void l3o_predict_batch(const uint8_t* tl, const uint8_t* t, const uint8_t* tr,
                       uint8_t* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = l3o_predict(tl[i], t[i], tr[i]);
}

uint8_t l3o_predict_original(uint8_t left, uint8_t top, uint8_t top_left) {
    return (uint8_t)predict_original_int(left, top, top_left);
}

void l3o_predict_original_batch(const uint8_t* left, const uint8_t* top, const uint8_t* top_left,
                                uint8_t* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = l3o_predict_original(left[i], top[i], top_left[i]);
}

size_t l3o_encode_bound(uint32_t width, uint32_t height, uint32_t patch) {
    if (patch == 0) patch = l3o_patch_rule(width, height);
    uint64_t px = ceil_div(width, patch), py = ceil_div(height, patch);
    /* per patch: every row at most 12 + 8*pw bits, plus one padding byte */
    uint64_t per_channel = (uint64_t)height * px * 2 + (uint64_t)width * height + px * py;
    return (size_t)(13 + 12 * px * py + 3 * per_channel);
}

int l3o_encode(const uint8_t* rgb, uint32_t width, uint32_t height, size_t row_stride,
               uint32_t patch, int width_mode, uint8_t* out, size_t out_cap,
               size_t* out_len) {
    return l3o_encode_with(rgb, width, height, row_stride, patch, width_mode,
                           L3O_PREDICTOR_CUSTOM, out, out_cap, out_len);
}

int l3o_encode_with(const uint8_t* rgb, uint32_t width, uint32_t height, size_t row_stride,
                    uint32_t patch, int width_mode, int predictor, uint8_t* out, size_t out_cap,
                    size_t* out_len) {
    if (!rgb || !out || !out_len || width == 0 || height == 0 || patch > 255 ||
        row_stride < (size_t)width * 3 || width_mode < 0 || width_mode > 2 ||
        (predictor != L3O_PREDICTOR_CUSTOM && predictor != L3O_PREDICTOR_ORIGINAL))
        return L3O_ERR_ARG;
    if (patch == 0) patch = l3o_patch_rule(width, height);
    const uint32_t px = ceil_div(width, patch), py = ceil_div(height, patch);
    const uint64_t patches = (uint64_t)px * py;
    const uint64_t header = 13 + 12 * patches;
    if (out_cap < header) return L3O_ERR_SPACE;
    std::memcpy(out, kMagic, 4);
    store_u32le(out + 4, width);
    store_u32le(out + 8, height);
    out[12] = (uint8_t)patch;

    uint64_t data_pos = 0;
    for (uint32_t c = 0; c < 3; ++c) {
        for (uint32_t ty = 0; ty < py; ++ty) {
            for (uint32_t tx = 0; tx < px; ++tx) {
                uint32_t x0 = tx * patch, y0 = ty * patch;
                uint32_t pw = (width - x0 < patch) ? width - x0 : patch;
                uint32_t ph = (height - y0 < patch) ? height - y0 : patch;
                BitWriter bw;
                encode_patch(rgb + (size_t)y0 * row_stride + (size_t)x0 * 3 + c, row_stride, 3,
                             pw, ph, width_mode, predictor, bw);
                uint64_t flat = (uint64_t)c * patches + (uint64_t)ty * px + tx;
                if (data_pos > 0xFFFFFFFFull) return L3O_ERR_ARG;
                store_u32le(out + 13 + 4 * flat, (uint32_t)data_pos);
                if (header + data_pos + bw.bytes.size() > out_cap) return L3O_ERR_SPACE;
                std::memcpy(out + header + data_pos, bw.bytes.data(), bw.bytes.size());
                data_pos += bw.bytes.size();
            }
        }
    }
    *out_len = (size_t)(header + data_pos);
    return L3O_OK;
}

int l3o_parse_header(const uint8_t* file, size_t len, l3o_info* info) {
    if (!file || !info) return L3O_ERR_ARG;
    if (len < 13) return L3O_ERR_TRUNCATED;
    if (std::memcmp(file, kMagic, 4) != 0) return L3O_ERR_MAGIC;
    info->width = load_u32le(file + 4);
    info->height = load_u32le(file + 8);
    info->patch = file[12];
    if (info->width == 0 || info->height == 0 || info->patch == 0) return L3O_ERR_CORRUPT;
    info->px = ceil_div(info->width, info->patch);
    info->py = ceil_div(info->height, info->patch);
    info->header_bytes = 13 + 12 * (uint64_t)info->px * info->py;
    if (len < info->header_bytes) return L3O_ERR_TRUNCATED;
    info->data_bytes = len - info->header_bytes;
    return L3O_OK;
}

int l3o_decode_patch(const uint8_t* stream, size_t len, uint32_t pw, uint32_t ph,
                     uint8_t* out, size_t out_stride) {
    return l3o_decode_patch_with(stream, len, pw, ph, L3O_PREDICTOR_CUSTOM, out, out_stride);
}

int l3o_decode_patch_with(const uint8_t* stream, size_t len, uint32_t pw, uint32_t ph,
                          int predictor, uint8_t* out, size_t out_stride) {
    if (!stream || !out || pw == 0 || ph == 0 || out_stride < pw ||
        (predictor != L3O_PREDICTOR_CUSTOM && predictor != L3O_PREDICTOR_ORIGINAL))
        return L3O_ERR_ARG;
    std::vector<uint8_t> resid((size_t)pw * ph);
    int rc = unpack_patch(stream, len, pw, ph, resid.data(), pw);
    if (rc != L3O_OK) return rc;
    unfilter_patch(resid.data(), pw, pw, ph, predictor, out, out_stride);
    return L3O_OK;
}

int l3o_decode(const uint8_t* file, size_t len, uint8_t* rgb, size_t row_stride) {
    return l3o_decode_with(file, len, L3O_PREDICTOR_CUSTOM, rgb, row_stride);
}

int l3o_decode_with(const uint8_t* file, size_t len, int predictor, uint8_t* rgb,
                    size_t row_stride) {
    l3o_info info;
    int rc = l3o_parse_header(file, len, &info);
    if (rc != L3O_OK) return rc;
    if (!rgb || row_stride < (size_t)info.width * 3) return L3O_ERR_ARG;
    std::vector<uint8_t> pixels;
    return for_each_patch(file, len, info,
        [&](uint32_t c, uint32_t x0, uint32_t y0, uint32_t pw, uint32_t ph,
            const uint8_t* stream, size_t slen) -> int {
            pixels.assign((size_t)pw * ph, 0);
            int r = l3o_decode_patch_with(stream, slen, pw, ph, predictor, pixels.data(), pw);
            if (r != L3O_OK) return r;
            for (uint32_t y = 0; y < ph; ++y)
                for (uint32_t x = 0; x < pw; ++x)
                    rgb[(size_t)(y0 + y) * row_stride + (size_t)(x0 + x) * 3 + c] =
                        pixels[(size_t)y * pw + x];
            return L3O_OK;
        });
}

int l3o_decode_residuals(const uint8_t* file, size_t len, uint8_t* planes) {
    l3o_info info;
    int rc = l3o_parse_header(file, len, &info);
    if (rc != L3O_OK) return rc;
    if (!planes) return L3O_ERR_ARG;
    const size_t w = info.width, h = info.height;
    return for_each_patch(file, len, info,
        [&](uint32_t c, uint32_t x0, uint32_t y0, uint32_t pw, uint32_t ph,
            const uint8_t* stream, size_t slen) -> int {
            return unpack_patch(stream, slen, pw, ph,
                                planes + (size_t)c * w * h + (size_t)y0 * w + x0, w);
        });
}

uint16_t l3o_f32_to_bf16(float x) {
    uint32_t u = f32_bits(x);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) /* NaN: keep quiet */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lower = u & 0xFFFFu;
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) ++upper;
    return (uint16_t)upper;
}

uint16_t l3o_f32_to_f16(float x) {
    uint32_t u = f32_bits(x);
    uint32_t sign = (u >> 16) & 0x8000u;
    int32_t exp = (int32_t)((u >> 23) & 0xFF);
    uint32_t man = u & 0x007FFFFFu;
    if (exp == 0xFF) return (uint16_t)(sign | 0x7C00u | (man ? 0x0200u : 0u));
    int32_t e = exp - 127 + 15;            /* binary16 biased exponent */
    if (e >= 31) return (uint16_t)(sign | 0x7C00u);   /* overflow -> inf */
    uint64_t sig;                          /* significand with the hidden bit */
    int shift;                             /* bits to drop from sig */
    if (e <= 0) {                          /* subnormal or zero in binary16 */
        if (e < -10) return (uint16_t)sign;
        sig = (uint64_t)(man | 0x00800000u);
        shift = 14 - e;                    /* 13 + (1 - e) */
        e = 0;
    } else {
        sig = man;
        shift = 13;
    }
    uint64_t kept = sig >> shift;
    uint64_t rest = sig & (((uint64_t)1 << shift) - 1);
    uint64_t half = (uint64_t)1 << (shift - 1);
    uint32_t h = (uint32_t)((uint32_t)e << 10) + (uint32_t)kept;
    if (rest > half || (rest == half && (kept & 1))) ++h;   /* carries into the exponent */
    return (uint16_t)(sign | h);
}

int l3o_crop_normalize(const uint8_t* rgb, uint32_t width, uint32_t height, size_t row_stride,
                       int32_t x0, int32_t y0, int flip, uint32_t crop_w, uint32_t crop_h,
                       const float mean[3], const float stdv[3], int dtype,
                       uint16_t* out) {
    if (!rgb || !out || !mean || !stdv || x0 < 0 || y0 < 0 || crop_w == 0 || crop_h == 0 ||
        (uint64_t)x0 + crop_w > width || (uint64_t)y0 + crop_h > height ||
        (dtype != 0 && dtype != 1))
        return L3O_ERR_ARG;
    for (uint32_t c = 0; c < 3; ++c)
        for (uint32_t i = 0; i < crop_h; ++i)
            for (uint32_t j = 0; j < crop_w; ++j) {
                uint32_t sx = flip ? (uint32_t)x0 + crop_w - 1 - j : (uint32_t)x0 + j;
                uint8_t v = rgb[(size_t)((uint32_t)y0 + i) * row_stride + (size_t)sx * 3 + c];
                volatile float scaled = (float)v / 255.0f;
                volatile float centred = scaled - mean[c];
                float y = centred / stdv[c];
                out[((size_t)c * crop_h + i) * crop_w + j] =
                    dtype == 0 ? l3o_f32_to_bf16(y) : l3o_f32_to_f16(y);
            }
    return L3O_OK;
}

}  // extern "C"
