/*
 * The oracle (oracle/l3_oracle.cpp) under AddressSanitizer and UBSan.  Built by
 * tests/test_oracle_sanitizers.py with the host compiler; CPU only.
 *
 * Every buffer is a heap block of exactly the size the call is told about:
 *   - round trips decode(encode(x)) == x on edge shapes (1-pixel images, widths and heights
 *     one off a multiple of the patch size), patch sizes 1..255, all three width modes and
 *     both predictors, with output rows ending exactly where the block ends;
 *   - encode into a buffer of exactly the file's length, and one byte short (must be refused);
 *   - every truncation of a file and single-byte damage at every header and offset byte and at
 *     sampled stream bytes: the decoder must return a status, never touch memory outside its
 *     blocks (arxiv 2208.08711 Section 4.3: signature, sizes, patch size, offset arrays;
 *     Section 4.2: 4-bit width, 8-bit base, deltas);
 *   - the crop / normalise epilogue on windows touching every border.
 * Prints "ok <cases>" and exits 0; any finding aborts.
 */
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "l3_oracle.h"

namespace {

uint64_t state = 0x9E3779B97F4A7C15ull;
uint32_t rnd() {   /* xorshift64*; only the harness's own choice of cases */
    state ^= state >> 12;
    state ^= state << 25;
    state ^= state >> 27;
    return (uint32_t)((state * 0x2545F4914F6CDD1Dull) >> 32);
}

struct Block {   /* exact-size heap block */
    uint8_t* p;
    size_t n;
    explicit Block(size_t n_) : p((uint8_t*)std::malloc(n_ ? n_ : 1)), n(n_) {
        if (!p) std::abort();
    }
    ~Block() { std::free(p); }
    Block(const Block&) = delete;
    Block& operator=(const Block&) = delete;
};

void require(bool ok, const char* what, uint32_t w, uint32_t h, unsigned patch) {
    if (!ok) {
        std::fprintf(stderr, "FAILED: %s (width %u height %u patch %u)\n", what, w, h, patch);
        std::exit(1);
    }
}

long cases = 0;

void fill(Block& img, uint32_t w, uint32_t h, size_t stride, int kind) {
    for (uint32_t y = 0; y < h; ++y)
        for (uint32_t x = 0; x < 3 * w; ++x) {
            uint8_t v;
            switch (kind) {
                case 0: v = (uint8_t)rnd(); break;                          /* noise: width 8 */
                case 1: v = (uint8_t)(40 + x / 3 + 2 * y + (rnd() & 3)); break; /* ramp + small noise */
                case 2: v = 200; break;                                     /* constant: width 0 */
                default: v = (uint8_t)(((x / 3 + y) & 1) * 255); break;     /* wrap around 256 */
            }
            img.p[y * stride + x] = v;
        }
}

void round_trip(uint32_t w, uint32_t h, uint32_t patch, int kind, int width_mode, int predictor) {
    const size_t stride = 3 * (size_t)w + (rnd() % 5);
    Block img(stride * (h - 1) + 3 * (size_t)w);          /* the last row ends with the block */
    fill(img, w, h, stride, kind);
    const uint32_t n = patch ? patch : l3o_patch_rule(w, h);
    const size_t bound = l3o_encode_bound(w, h, n);
    require(bound > 0, "encode bound", w, h, patch);
    Block file(bound);
    size_t len = 0;
    int st = l3o_encode_with(img.p, w, h, stride, patch, width_mode, predictor, file.p, file.n, &len);
    require(st == L3O_OK && len <= bound, "encode", w, h, patch);
    {   /* exactly the file's length is enough, one byte less is refused */
        Block exact(len), shorter(len - 1);
        size_t l2 = 0;
        require(l3o_encode_with(img.p, w, h, stride, patch, width_mode, predictor, exact.p, exact.n, &l2) == L3O_OK &&
                    l2 == len && std::memcmp(exact.p, file.p, len) == 0, "exact-size encode", w, h, patch);
        require(l3o_encode_with(img.p, w, h, stride, patch, width_mode, predictor, shorter.p, shorter.n, &l2) ==
                    L3O_ERR_SPACE, "short encode buffer", w, h, patch);
    }
    Block exact(len);
    std::memcpy(exact.p, file.p, len);
    l3o_info info;
    require(l3o_parse_header(exact.p, len, &info) == L3O_OK && info.width == w && info.height == h &&
                info.patch == n, "header", w, h, patch);
    const size_t ostride = 3 * (size_t)w + (rnd() % 3);
    Block out(ostride * (h - 1) + 3 * (size_t)w);
    require(l3o_decode_with(exact.p, len, predictor, out.p, ostride) == L3O_OK, "decode", w, h, patch);
    for (uint32_t y = 0; y < h; ++y)
        require(std::memcmp(out.p + y * ostride, img.p + y * stride, 3 * (size_t)w) == 0, "round trip", w, h, patch);
    Block planes(3 * (size_t)w * h);
    require(l3o_decode_residuals(exact.p, len, planes.p) == L3O_OK, "residual planes", w, h, patch);
    ++cases;
}

/* Damaged and truncated files: any status is fine, touching memory outside the blocks is not. */
void hostile(uint32_t w, uint32_t h, uint32_t patch) {
    Block img(3 * (size_t)w * h);
    fill(img, w, h, 3 * (size_t)w, 1);
    Block file(l3o_encode_bound(w, h, patch));
    size_t len = 0;
    require(l3o_encode(img.p, w, h, 3 * (size_t)w, patch, 0, file.p, file.n, &len) == L3O_OK, "encode", w, h, patch);
    l3o_info info;
    require(l3o_parse_header(file.p, len, &info) == L3O_OK, "header", w, h, patch);
    Block out(3 * (size_t)w * h);
    for (size_t cut = 0; cut < len; cut += (cut < 64 ? 1 : 1 + rnd() % 7)) {      /* truncations */
        Block part(cut);
        std::memcpy(part.p, file.p, cut);
        const int st = l3o_decode(part.p, cut, out.p, 3 * (size_t)w);
        require(st != L3O_OK, "truncated file accepted", w, h, patch);
        ++cases;
    }
    for (size_t at = 0; at < len; at += (at < info.header_bytes ? 1 : 1 + rnd() % 11)) {   /* one damaged byte */
        for (int rep = 0; rep < 2; ++rep) {
            Block bad(len);
            std::memcpy(bad.p, file.p, len);
            bad.p[at] = rep ? (uint8_t)(bad.p[at] ^ (1u << (rnd() % 8))) : (uint8_t)rnd();
            l3o_info i2;
            (void)l3o_parse_header(bad.p, len, &i2);
            /* a changed size field would ask for another output size: decode only what still
             * describes this image */
            if (l3o_parse_header(bad.p, len, &i2) == L3O_OK && i2.width == w && i2.height == h)
                (void)l3o_decode(bad.p, len, out.p, 3 * (size_t)w);
            ++cases;
        }
    }
}

void epilogue(uint32_t w, uint32_t h, uint32_t cw, uint32_t ch) {
    Block img(3 * (size_t)w * h);
    fill(img, w, h, 3 * (size_t)w, 0);
    const float mean[3] = {0.485f, 0.456f, 0.406f}, stdv[3] = {0.229f, 0.224f, 0.225f};
    const int32_t xs[3] = {0, (int32_t)(w - cw), (int32_t)((w - cw) / 2)};
    const int32_t ys[3] = {0, (int32_t)(h - ch), (int32_t)((h - ch) / 2)};
    for (int a = 0; a < 3; ++a)
        for (int b = 0; b < 3; ++b)
            for (int flip = 0; flip < 2; ++flip)
                for (int dtype = 0; dtype < 2; ++dtype) {
                    Block out(2 * 3 * (size_t)cw * ch);
                    require(l3o_crop_normalize(img.p, w, h, 3 * (size_t)w, xs[a], ys[b], flip, cw, ch, mean, stdv,
                                               dtype, (uint16_t*)out.p) == L3O_OK, "epilogue", w, h, 0);
                    ++cases;
                }
}

}  // namespace

int main() {
    static const uint32_t shapes[][2] = {{1, 1}, {2, 1}, {1, 2}, {3, 5}, {31, 33}, {33, 31}, {32, 32}, {63, 65},
                                         {65, 63}, {127, 3}, {129, 127}, {130, 129}, {257, 40}, {40, 257}};
    static const uint32_t patches[] = {0, 1, 2, 3, 32, 64, 128, 255};
    for (const auto& s : shapes)
        for (uint32_t patch : patches)
            for (int kind = 0; kind < 4; ++kind)
                round_trip(s[0], s[1], patch, kind, (int)(rnd() % 3), (int)(rnd() % 2));
    hostile(37, 29, 32);
    hostile(70, 5, 64);
    hostile(9, 40, 3);
    epilogue(50, 40, 50, 40);
    epilogue(61, 47, 24, 16);
    std::printf("ok %ld\n", cases);
    return 0;
}
