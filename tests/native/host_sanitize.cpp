/*
 * The library's host code (CPU encoder, encode bound, header validator) under
 * AddressSanitizer and UBSan.  Built by tests/test_host_sanitizers.py from
 * paper_2208_08711_amd/csrc/l3_host.cpp with the host compiler; no GPU, no HIP.
 *
 * Every buffer handed to the library is a heap block of exactly the size the
 * call is told about, so that one byte read or written past it stops the run:
 *   - images whose last row ends where the block ends (row stride > 3 * width),
 *   - output buffers of exactly l3_encode_bound() bytes, of exactly the file's
 *     length, and one byte short of it (must be refused, nothing written past),
 *   - files cut at every length, and files with damaged headers and offsets
 *     (Section 4.3 of arxiv 2208.08711: signature, width, height, patch size, the
 *     three offset arrays), for the validator,
 *   - and the host planner's dealing of patches to work units, against the mapping the
 *     decode kernel applies to it.
 * Prints "ok <cases>" and exits 0; any finding aborts.
 */
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "l3.h"
#include "l3_ablation.h"
#include "l3_internal.h"   /* the host planner's descriptor and l3_plan_units */

namespace {

uint64_t state = 0x243F6A8885A308D3ull;
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

/* what a caller may rely on after l3_peek_header said L3_OK */
void check_accepted(const uint8_t* f, size_t len, const l3_info& info) {
    const uint64_t tx = (info.width + info.patch - 1) / info.patch;
    const uint64_t ty = (info.height + info.patch - 1) / info.patch;
    require(info.patches_per_channel == tx * ty, "patch count", info.width, info.height, info.patch);
    require(info.header_bytes == 13 + 12 * tx * ty && info.header_bytes <= len, "header size",
            info.width, info.height, info.patch);
    const uint64_t data = len - info.header_bytes;
    uint64_t prev = 0;
    for (uint64_t k = 0; k < 3 * tx * ty; ++k) {
        uint32_t off;
        std::memcpy(&off, f + 13 + 4 * k, 4);
        require(k == 0 ? off == 0 : off > prev, "offsets increase", info.width, info.height, info.patch);
        require(off < data, "offset inside the data section", info.width, info.height, info.patch);
        prev = off;
    }
}

/* The host's dealing of patches to work units (per-row and flat order), checked against
 * what the decode kernel does with it, written out again here: unit u, lane group g of
 * tpw -> patch (tx, ty).  Every patch must be taken exactly once, all patches of a unit
 * must have the same number of rows, a unit's first group must be the topmost, and the
 * flat order must never need more units than the per-row order. */
unsigned long check_plans() {
    unsigned long cases = 0;
    const uint32_t sizes[] = {1, 2, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 200, 255, 256, 257, 450, 500, 1000, 1920, 2048};
    const uint32_t nsizes = sizeof sizes / sizeof *sizes;
    for (uint32_t np = 32; np <= 128; np *= 2)
        for (uint32_t tpw = 256 / np; tpw <= 512 / np; tpw *= 2)      /* 4 and 8 pixels per lane */
            for (uint32_t wi = 0; wi < nsizes; ++wi)
                for (uint32_t hi = 0; hi < nsizes; ++hi)
                    for (int flat_ok = 0; flat_ok < 2; ++flat_ok) {
                        L3ImageDesc d;
                        std::memset(&d, 0, sizeof d);
                        d.width = sizes[wi];
                        d.height = sizes[hi];
                        d.tiles_x = (d.width + np - 1) / np;
                        d.tiles_y = (d.height + np - 1) / np;
                        d.row_stride = 3ull * d.width + (wi % 3);
                        l3_plan_units(&d, np, tpw, flat_ok != 0);
                        const uint32_t per_row = ((d.tiles_x + tpw - 1) / tpw) * d.tiles_y;
                        require(d.units <= per_row && d.units >= 1, "unit count", d.width, d.height, np);
                        require(flat_ok || d.groups_x != 0, "flat order only when allowed", d.width, d.height, np);
                        std::vector<unsigned> taken((size_t)d.tiles_x * d.tiles_y, 0);
                        for (uint32_t u = 0; u < d.units; ++u) {
                            uint32_t base_ty = 0, rows = 0;
                            for (uint32_t g = 0; g < tpw; ++g) {
                                uint32_t tx, ty, ty_base;
                                bool active;
                                if (d.groups_x == 0) {
                                    const bool upper = u < d.flat_upper_units;
                                    const uint32_t first = (upper ? u : u - d.flat_upper_units) * tpw;
                                    const uint32_t count = upper ? d.tiles_x * d.flat_upper_rows : d.tiles_x;
                                    const uint32_t row_off = upper ? 0u : d.flat_upper_rows;
                                    require(first < count, "unit inside its block", d.width, d.height, np);
                                    const uint32_t fl = first + g;
                                    active = fl < count;
                                    const uint32_t flc = active ? fl : count - 1;
                                    ty = row_off + flc / d.tiles_x;
                                    tx = flc % d.tiles_x;
                                    ty_base = row_off + first / d.tiles_x;
                                } else {
                                    const uint32_t trow = u / d.groups_x, gx = u % d.groups_x;
                                    const uint32_t txr = gx * tpw + g;
                                    active = txr < d.tile_x_count;
                                    tx = d.tile_x_first + (active ? txr : d.tile_x_count - 1);
                                    ty = ty_base = d.tile_y_first + trow;
                                }
                                require(tx < d.tiles_x && ty < d.tiles_y && ty_base <= ty, "patch inside the image",
                                        d.width, d.height, np);
                                const uint32_t ph = d.height - ty * np < np ? d.height - ty * np : np;
                                if (g == 0) {
                                    base_ty = ty_base;
                                    rows = ph;
                                    require(ty == ty_base, "first group is the topmost", d.width, d.height, np);
                                }
                                require(ty_base == base_ty && ph == rows, "one height per unit", d.width, d.height, np);
                                /* the lane's 32-bit output offset reaches its patch row */
                                require((uint64_t)(ty - ty_base) * np * d.row_stride + 3ull * d.width < 0xFFFFFFFFull,
                                        "offset fits 32 bits", d.width, d.height, np);
                                if (active) ++taken[(size_t)ty * d.tiles_x + tx];
                            }
                        }
                        for (size_t k = 0; k < taken.size(); ++k)
                            require(taken[k] == 1, "every patch exactly once", d.width, d.height, np);
                        ++cases;
                    }
    /* where the offsets would not fit, the per-row order stays */
    {
        L3ImageDesc d;
        std::memset(&d, 0, sizeof d);
        d.width = 450;
        d.height = 337;
        d.tiles_x = 15;
        d.tiles_y = 11;
        d.row_stride = 1ull << 28;
        l3_plan_units(&d, 32, 8, true);
        require(d.groups_x == 2 && d.units == 22, "per-row order for huge strides", d.width, d.height, 32);
    }
    return cases;
}

}  // namespace

int main() {
    const unsigned patches[] = {0, 1, 2, 3, 5, 7, 16, 32, 64, 128, 255};
    unsigned long cases = 0;
    for (int round = 0; round < 160; ++round) {
        const uint32_t w = 1 + rnd() % (round % 8 == 0 ? 300 : 70);
        const uint32_t h = 1 + rnd() % (round % 8 == 1 ? 300 : 70);
        const unsigned patch = patches[rnd() % (sizeof patches / sizeof *patches)];
        const size_t stride = 3 * (size_t)w + rnd() % 9;
        Block img((size_t)(h - 1) * stride + 3 * (size_t)w);
        const unsigned kind = rnd() % 4;
        for (uint32_t y = 0; y < h; ++y)
            for (uint32_t x = 0; x < 3 * w; ++x) {
                uint8_t v;
                if (kind == 0) v = (uint8_t)rnd();
                else if (kind == 1) v = (uint8_t)(x / 3 + 2 * y + (rnd() & 3));
                else if (kind == 2) v = (uint8_t)(((x / 3) ^ y) & 1 ? 255 : 0);
                else v = 7;
                img.p[y * stride + x] = v;
            }
        for (int original = 0; original < 2; ++original) {
            const size_t bound = l3_encode_bound(w, h, (uint8_t)patch);
            require(bound >= 13, "encode bound", w, h, patch);
            Block out(bound);
            size_t len = 0;
            l3_status s = l3_ablation_encode_cpu(img.p, w, h, stride, (uint8_t)patch, original, out.p,
                                                 out.n, &len);
            require(s == L3_OK && len <= bound, "encode into a buffer of the bound's size", w, h, patch);
            {
                Block exact(len);
                size_t len2 = 0;
                s = original ? l3_ablation_encode_cpu(img.p, w, h, stride, (uint8_t)patch, 1, exact.p, exact.n, &len2)
                             : l3_encode_cpu(img.p, w, h, stride, (uint8_t)patch, exact.p, exact.n, &len2);
                require(s == L3_OK && len2 == len && std::memcmp(exact.p, out.p, len) == 0,
                        "encode into a buffer of the file's size", w, h, patch);
                Block tight(len - 1);
                s = l3_ablation_encode_cpu(img.p, w, h, stride, (uint8_t)patch, original, tight.p, tight.n, &len2);
                require(s == L3_ERR_BUFFER_TOO_SMALL, "one byte short is refused", w, h, patch);
                const size_t some = rnd() % len;
                Block small(some);
                s = l3_ablation_encode_cpu(img.p, w, h, stride, (uint8_t)patch, original, small.p, small.n, &len2);
                require(s == L3_ERR_BUFFER_TOO_SMALL, "a short buffer is refused", w, h, patch);
                cases += 4;
            }
            /* the validator: the file as it is, every shorter length (sampled when long),
             * and damaged headers */
            l3_info info;
            {
                Block f(len);
                std::memcpy(f.p, out.p, len);
                require(l3_peek_header(f.p, f.n, &info) == L3_OK, "own file accepted", w, h, patch);
                check_accepted(f.p, f.n, info);
            }
            const size_t step = len > 4000 ? 1 + len / 997 : 1;
            for (size_t cut = 0; cut < len; cut += (cut < 64 ? 1 : step)) {
                Block f(cut);
                std::memcpy(f.p, out.p, cut);
                l3_info got;
                if (l3_peek_header(f.p, f.n, &got) == L3_OK) check_accepted(f.p, f.n, got);
                ++cases;
            }
            const size_t header = info.header_bytes;
            for (int k = 0; k < 200; ++k) {
                Block f(len);
                std::memcpy(f.p, out.p, len);
                const int hits = 1 + rnd() % 3;
                for (int t = 0; t < hits; ++t) {
                    const size_t at = rnd() % header;
                    const unsigned how = rnd() % 3;
                    f.p[at] = how == 0 ? (uint8_t)rnd() : how == 1 ? (uint8_t)(f.p[at] ^ (1u << (rnd() & 7))) : 0xFF;
                }
                l3_info got;
                if (l3_peek_header(f.p, f.n, &got) == L3_OK) check_accepted(f.p, f.n, got);
                ++cases;
            }
        }
    }
    /* argument errors */
    {
        uint8_t px[3] = {1, 2, 3}, o[64];
        size_t n = 0;
        l3_info info;
        if (l3_encode_cpu(nullptr, 1, 1, 3, 0, o, sizeof o, &n) != L3_ERR_INVALID_ARG ||
            l3_encode_cpu(px, 0, 1, 3, 0, o, sizeof o, &n) != L3_ERR_INVALID_ARG ||
            l3_encode_cpu(px, 1, 1, 2, 0, o, sizeof o, &n) != L3_ERR_INVALID_ARG ||
            l3_encode_cpu(px, 1, 1, 3, 0, o, sizeof o, nullptr) != L3_ERR_INVALID_ARG ||
            l3_peek_header(nullptr, 20, &info) != L3_ERR_INVALID_ARG ||
            l3_peek_header(o, 20, nullptr) != L3_ERR_INVALID_ARG || l3_encode_bound(0, 5, 0) != 0) {
            std::fprintf(stderr, "FAILED: argument errors\n");
            return 1;
        }
    }
    cases += check_plans();
    std::printf("ok %lu\n", cases);
    return 0;
}
