/*
 * Brute force over tiny images through the oracle's full encode -> decode path
 * (test driver; links the oracle library).  For every case it checks
 *   (1) decode(encode(x)) == x,
 *   (2) the residual plane the oracle reports against expectations computed
 *       here from the format statement: row 0 raw; first and last column of
 *       later rows = pixel - top (mod 256); for 3-wide images the centre
 *       residual r satisfies (selected + r) mod 256 == pixel with selected one
 *       of the three upper neighbours at minimal distance from TL + TR - T,
 *   (3) for 1-wide images the exact file bytes (closed form: two rows of width
 *       0, bases p0 and p1 - p0 mod 256, each a 12-bit record).
 * Prints "OK <cases> widths-seen-mask" or a line describing the first failure.
 */
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../oracle/l3_oracle.h"

static const int grid[8] = {0, 1, 127, 128, 129, 200, 254, 255};
static unsigned widths_seen = 0;

static int fail(const char* what, const uint8_t* img, int w, int h) {
    std::printf("FAIL %s: image", what);
    for (int i = 0; i < w * h; ++i) std::printf(" %d", img[i * 3]);
    std::printf("\n");
    return 1;
}

/* img: w*h*3 with all three channels equal to the grey value under test */
static int check(const uint8_t* img, int w, int h) {
    uint8_t file[256], back[64], resid[64];
    size_t len = 0;
    if (l3o_encode(img, w, h, (size_t)w * 3, (uint32_t)(w > h ? w : h), 0, file, sizeof file, &len))
        return fail("encode", img, w, h);
    if (l3o_decode(file, len, back, (size_t)w * 3)) return fail("decode", img, w, h);
    if (std::memcmp(back, img, (size_t)w * h * 3)) return fail("round trip", img, w, h);
    if (l3o_decode_residuals(file, len, resid)) return fail("residuals", img, w, h);
    /* stream of the first channel starts at 13 + 12; row r's width nibble */
    {
        const uint8_t* s = file + 25;
        unsigned w0 = s[0] & 15u;
        widths_seen |= 1u << w0;
        unsigned bit = 12 + (unsigned)w * w0;
        unsigned w1 = ((s[bit >> 3] | (s[(bit >> 3) + 1] << 8)) >> (bit & 7)) & 15u;
        widths_seen |= 1u << w1;
    }
    for (int x = 0; x < w; ++x)
        if (resid[x] != img[x * 3]) return fail("row 0 not raw", img, w, h);
    for (int x = 0; x < w; ++x) {
        int p = img[(w + x) * 3], r = resid[w + x];
        if (x == 0 || x == w - 1) {
            if (((img[x * 3] + r) & 255) != p) return fail("border residual", img, w, h);
        } else {
            int tl = img[(x - 1) * 3], t = img[x * 3], tr = img[(x + 1) * 3];
            int sel = (p - r) & 255, ref = tl + tr - t;
            int best = std::abs(ref - tl);
            if (std::abs(ref - tr) < best) best = std::abs(ref - tr);
            if (std::abs(ref - t) < best) best = std::abs(ref - t);
            bool ok = (sel == tl && std::abs(ref - tl) == best) ||
                      (sel == tr && std::abs(ref - tr) == best) ||
                      (sel == t && std::abs(ref - t) == best);
            if (!ok) return fail("centre residual", img, w, h);
        }
    }
    if (w == 1) {
        unsigned b0 = img[0], b1 = (unsigned)(img[3] - img[0]) & 255u;
        uint8_t expect[3] = {(uint8_t)((b0 & 15u) << 4), (uint8_t)(b0 >> 4), (uint8_t)b1};
        if (len != 13 + 12 + 9 || std::memcmp(file + 25, expect, 3) ||
            std::memcmp(file + 28, expect, 3) || std::memcmp(file + 31, expect, 3))
            return fail("1-wide file bytes", img, w, h);
    }
    return 0;
}

static void set(uint8_t* img, int i, int v) { img[i * 3] = img[i * 3 + 1] = img[i * 3 + 2] = (uint8_t)v; }

int main(int argc, char** argv) {
    const char* which = argc > 1 ? argv[1] : "all";
    unsigned long cases = 0;
    uint8_t img[64];
    if (!std::strcmp(which, "1x2") || !std::strcmp(which, "all")) {
        for (int a = 0; a < 256; ++a)
            for (int b = 0; b < 256; ++b) {
                set(img, 0, a); set(img, 1, b);
                if (check(img, 1, 2)) return 1;
                ++cases;
            }
    }
    if (!std::strcmp(which, "2x2") || !std::strcmp(which, "all")) {
        for (int sweep = 0; sweep < 4; ++sweep)
            for (int g = 0; g < 8 * 8 * 8; ++g)
                for (int v = 0; v < 256; ++v) {
                    int k = 0, gg = g;
                    for (int i = 0; i < 4; ++i) {
                        if (i == sweep) set(img, i, v);
                        else { set(img, i, grid[gg & 7]); gg >>= 3; ++k; }
                    }
                    if (check(img, 2, 2)) return 1;
                    ++cases;
                }
    }
    if (!std::strcmp(which, "3x2") || !std::strcmp(which, "all")) {
        for (int g = 0; g < 8 * 8 * 8 * 8 * 8; ++g)
            for (int v = 0; v < 256; ++v) {
                int gg = g;
                for (int i = 0; i < 6; ++i) {
                    if (i == 4) set(img, i, v);       /* bottom centre swept */
                    else { set(img, i, grid[gg & 7]); gg >>= 3; }
                }
                if (check(img, 3, 2)) return 1;
                ++cases;
            }
    }
    std::printf("OK %lu %u\n", cases, widths_seen);
    return 0;
}
