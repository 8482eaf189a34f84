/*
 * l3_ablation.h -- C ABI of the decoder variants that the ablation study of the L3
 * paper (arxiv 2208.08711, Section 5.5, the figure on normalised decoder execution
 * time) compares.  Measurement aids, not the product path: l3_decode_batch of l3.h is
 * the decoder to use.
 *
 * Section 5.5 switches three things on and off:
 *   - the filter: the original Paeth filter on left, top and top-left, which can only
 *     be undone pixel after pixel, against the custom filter on top-left, top and
 *     top-right of Section 4.2, which is undone a row at a time;
 *   - base-delta decoding: one thread walking the patch from its first pixel to its
 *     last, against one thread per pixel of a row (Section 4.4);
 *   - patch-level parallelism (Section 4.4): all patches at once, against the patches
 *     of an image one after another.
 * A file for the original filter has the same container and base-delta stage as an
 * L3 file; only the predictor of rows >= 1 differs (first row raw, first column
 * predicted by the pixel above).  Nothing in the file says which filter wrote it: the
 * caller passes the matching flag.
 */
#ifndef L3_ABLATION_H
#define L3_ABLATION_H

#include "l3.h"

#ifdef __cplusplus
extern "C" {
#endif

/* As l3_encode_cpu; original_filter != 0 selects the original Paeth filter (nearest of
 * left, top, top-left to left + top - top_left, ties in that order). */
l3_status l3_ablation_encode_cpu(const uint8_t* rgb_hwc, uint32_t width, uint32_t height,
                                 size_t row_stride, uint8_t patch, int original_filter,
                                 uint8_t* out, size_t out_cap, size_t* out_len);

enum {
    L3_ABLATION_PIXEL_BD = 1,        /* one lane per pixel of a row extracts its delta */
    L3_ABLATION_CUSTOM_FILTER = 2,   /* files use the custom filter; undone row-parallel */
    L3_ABLATION_SERIAL_PATCHES = 4,  /* one workgroup per image takes its patches in turn */
    L3_ABLATION_DIAGONAL = 8         /* original filter undone one anti-diagonal per step (not in
                                        the paper: the best schedule its dependencies allow);
                                        not together with L3_ABLATION_CUSTOM_FILTER */
};

/* Decodes n files (l3_item as for l3_decode_batch; interleaved RGB output) with the
 * variant that `variant` (a combination of the flags above) selects.  Without
 * L3_ABLATION_PIXEL_BD a single lane decodes the base-delta stream of a patch;
 * without L3_ABLATION_CUSTOM_FILTER the files must have been written with the
 * original filter and a single lane undoes it in raster order (or, with
 * L3_ABLATION_DIAGONAL, all lanes undo it along anti-diagonals).  One wave works on one
 * patch of one channel, from a copy of the patch stream in local memory.
 * Any patch size 1..128.  A damaged stream yields unspecified pixels inside the
 * image's own output rectangle; nothing is read outside the file or written outside
 * the rectangle.  The call returns after the kernel is enqueued on `stream`; when the
 * batch differs from the previous call's it first waits for the device to go idle
 * and uploads its descriptors with a blocking copy (not meant for overlap).
 * Errors: INVALID_ARG, UNSUPPORTED (N > 128), DEVICE. */
l3_status l3_ablation_decode_batch(l3_ctx* ctx, const l3_item* items, int n, int variant,
                                   void* stream);

#ifdef __cplusplus
}
#endif
#endif /* L3_ABLATION_H */
