/*
 * L3 oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, single-threaded CPU encoder and decoder for the L3 lossless
 * image format (arxiv 2208.08711, Section 4.2 "Algorithm" and Section 4.3
 * "L3 File Format").  It exists so that the GPU decoder can be checked byte
 * for byte against something a reader can verify against the paper by eye.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may load
 * it.  It shares no code, header, table or helper with the GPU path.
 *
 * Where the paper is silent, these readings are frozen (all of them are
 * listed with their reasons in the design notes of this repository):
 *   - predictor ties: top-left wins, then top-right, then top;
 *   - at the first and last column of a patch the predictor is "top";
 *   - all value arithmetic is modulo 256; the encoder looks at the residuals
 *     of rows >= 1 as signed bytes and at row 0 as unsigned bytes when it
 *     takes min and max;
 *   - a constant row has width 0 and carries no payload bits;
 *   - bit k of a patch stream is bit (k mod 8) of byte k/8, a field's least
 *     significant bit comes first; rows follow each other with no padding,
 *     every patch is padded with zero bits to a whole byte;
 *   - header: bytes 4C 33 00 01, then width, height as little-endian u32,
 *     then one byte N; then three arrays (R, G, B) of ceil(W/N)*ceil(H/N)
 *     little-endian u32 byte offsets relative to the data section;
 *   - edge patches are clipped to the image;
 *   - default N by pixel count: < 1080*720 -> 32, <= 1920*1080 -> 64, else 128.
 *
 * Pins (tests/test_oracle_*.py): the 74/65/9 worked example of Section 4.2,
 * the closed-form size of a uniform-random FHD image (Table "compratio",
 * 1.02x), exhaustive predictor properties, brute force over tiny images,
 * hand-assembled streams, ramps and constant images, segment independence;
 * the original Paeth predictor against an independent PNG decoder (its filter
 * type 4 is that predictor).
 * Unpinned against the authors' own files (not available): tie order, border
 * rule and the byte-level conventions above -- "parity unpinned" for
 * interoperability; the build is self-consistent only.
 */
#ifndef L3_ORACLE_H
#define L3_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    L3O_OK = 0,
    L3O_ERR_ARG = 1,
    L3O_ERR_MAGIC = 2,
    L3O_ERR_TRUNCATED = 3,
    L3O_ERR_CORRUPT = 4,
    L3O_ERR_SPACE = 5
};

typedef struct {
    uint32_t width, height;
    uint32_t patch;            /* N */
    uint32_t px, py;           /* patches per row / per column */
    uint64_t header_bytes;     /* 13 + 12 * px * py */
    uint64_t data_bytes;       /* file length - header_bytes */
} l3o_info;

/* Section 4.3: the empirical patch-size rule, by pixel count. */
uint32_t l3o_patch_rule(uint32_t width, uint32_t height);

/* Section 4.2 "Custom Paeth Filter": the selected neighbour for one pixel. */
uint8_t l3o_predict(uint8_t top_left, uint8_t top, uint8_t top_right);
void l3o_predict_batch(const uint8_t* tl, const uint8_t* t, const uint8_t* tr,
                       uint8_t* out, size_t n);

/* Section 4.2, what the custom filter replaces: the original Paeth filter on
 * left, top and top-left (reference value left + top - top_left, nearest wins,
 * ties left, top, top-left).  Only the ablation of Section 5.5 uses it: the
 * same container and base-delta stage, with this predictor in rows >= 1 (the
 * first row stays raw; in the first column the prediction is "top"). */
enum { L3O_PREDICTOR_CUSTOM = 0, L3O_PREDICTOR_ORIGINAL = 1 };
uint8_t l3o_predict_original(uint8_t left, uint8_t top, uint8_t top_left);
void l3o_predict_original_batch(const uint8_t* left, const uint8_t* top,
                                const uint8_t* top_left, uint8_t* out, size_t n);

/* Upper bound of the file size for any content. */
size_t l3o_encode_bound(uint32_t width, uint32_t height, uint32_t patch);

/* width_mode: 0 = minimal width (canonical), 1 = always 8 bits,
 * 2 = minimal + 1 (capped at 8).  Modes 1 and 2 produce valid, non-canonical
 * streams that must decode to the same image. */
int l3o_encode(const uint8_t* rgb_hwc, uint32_t width, uint32_t height,
               size_t row_stride, uint32_t patch, int width_mode,
               uint8_t* out, size_t out_cap, size_t* out_len);

/* As l3o_encode, with the filter of stage 1 chosen by `predictor`. */
int l3o_encode_with(const uint8_t* rgb_hwc, uint32_t width, uint32_t height,
                    size_t row_stride, uint32_t patch, int width_mode, int predictor,
                    uint8_t* out, size_t out_cap, size_t* out_len);

int l3o_parse_header(const uint8_t* file, size_t len, l3o_info* info);

/* Whole file -> interleaved RGB (HWC), rows row_stride bytes apart. */
int l3o_decode(const uint8_t* file, size_t len, uint8_t* rgb_hwc, size_t row_stride);

/* As l3o_decode, for a file whose stage 1 used `predictor`. */
int l3o_decode_with(const uint8_t* file, size_t len, int predictor, uint8_t* rgb_hwc,
                    size_t row_stride);

/* Whole file -> the residual planes (after base-delta decoding, before the
 * inverse filter), planar: plane c at out + c*width*height, rows width apart. */
int l3o_decode_residuals(const uint8_t* file, size_t len, uint8_t* planes);

/* One patch stream of pw x ph pixels -> pixels, rows out_stride apart. */
int l3o_decode_patch(const uint8_t* stream, size_t len, uint32_t pw, uint32_t ph,
                     uint8_t* out, size_t out_stride);

int l3o_decode_patch_with(const uint8_t* stream, size_t len, uint32_t pw, uint32_t ph,
                          int predictor, uint8_t* out, size_t out_stride);

/* Training-input epilogue (not in the paper; defined by the benchmark
 * configuration): crop window at (x0,y0) of crop_w x crop_h, optional
 * horizontal mirror inside the window, y = (x/255 - mean[c]) / stdv[c] in
 * IEEE binary32 with no contraction, rounded to nearest-even to bfloat16
 * (dtype 0) or binary16 (dtype 1); out is [3][crop_h][crop_w] of 16-bit words. */
int l3o_crop_normalize(const uint8_t* rgb_hwc, uint32_t width, uint32_t height,
                       size_t row_stride, int32_t x0, int32_t y0, int flip,
                       uint32_t crop_w, uint32_t crop_h,
                       const float mean[3], const float stdv[3], int dtype,
                       uint16_t* out_chw);

/* binary32 -> bfloat16 / binary16 bit patterns, round to nearest even. */
uint16_t l3o_f32_to_bf16(float x);
uint16_t l3o_f32_to_f16(float x);

#ifdef __cplusplus
}
#endif
#endif
