/*
 * l3.h -- C ABI of the MI355X batched decoder for the L3 lossless image format
 * (arxiv 2208.08711).
 *
 * The format, as the paper states it:
 *   - Section 4.3 "L3 File Format": a file is a header (4-byte signature, 4-byte
 *     width, 4-byte height, 1-byte patch size N, three arrays of patch offsets,
 *     one array per colour channel) followed by a data section of encoded
 *     patches.  The image is split per channel (R, G, B) into N x N patches,
 *     each encoded on its own.
 *   - Section 4.2: a patch is encoded in two stages.  Stage 1, the custom Paeth
 *     filter: for rows after the first, each pixel is replaced by its difference
 *     from whichever of the three pixels above it (top-left, top, top-right) is
 *     nearest to top_left + top_right - top; the first row stays raw.  Stage 2,
 *     row-wise base-delta: per row, 4 bits = bits per delta, 8 bits = base (the
 *     row minimum), then one delta per pixel at that width; rows concatenated.
 *   - Section 4.4: the decoder reads each image's header on the host, splits the
 *     image into patches and decodes all patches in parallel on the GPU.
 *
 * Conventions the paper leaves open and this library fixes: signature bytes
 * 4C 33 00 01; width/height/offsets little-endian u32; offsets are byte offsets
 * from the start of the data section, in the order all-R, all-G, all-B patches,
 * each row-major, strictly increasing; a patch ends where the next one starts
 * (the last at the end of the file); stream bit k is bit (k mod 8) of byte k/8
 * and a field's least significant bit comes first; each patch is padded with
 * zero bits to a whole byte; edge patches are clipped to the image; all value
 * arithmetic is modulo 256; at the first and last column of a patch the
 * predictor is the pixel above; predictor ties resolve top-left, top-right, top;
 * a constant row has width 0.
 *
 * General rules of this ABI: plain C, no exceptions cross it, every call
 * returns an l3_status.  The caller owns every buffer it passes; the library
 * owns only l3_ctx.  "host" pointers are ordinary CPU memory, "device"
 * pointers are HIP device memory of the context's GPU.
 */
#ifndef L3_H
#define L3_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    L3_OK = 0,
    L3_ERR_INVALID_ARG = 1,      /* NULL pointer, negative count, zero size, bad enum */
    L3_ERR_BAD_MAGIC = 2,        /* file does not start with the L3 signature */
    L3_ERR_TRUNCATED = 3,        /* buffer shorter than the header it announces */
    L3_ERR_CORRUPT = 4,          /* header fields or offsets inconsistent */
    L3_ERR_BUFFER_TOO_SMALL = 5, /* output capacity insufficient */
    L3_ERR_UNSUPPORTED = 6,      /* valid file, but not handled by the GPU path */
    L3_ERR_DEVICE = 7,           /* a HIP runtime call failed / no usable GPU */
    L3_ERR_LIMIT = 8             /* the request exceeds a fixed limit of the entry point */
} l3_status;

/* Static, NUL-terminated description of a status value.  Never NULL. */
const char* l3_status_string(l3_status s);

/* ------------------------------------------------------------------------
 * Host side (CPU only, no GPU needed)
 * ------------------------------------------------------------------------ */

/* Section 4.3: the patch size the paper's empirical rule picks for an image
 * (32 below 1080x720 pixels, 64 up to 1920x1080, 128 above). */
uint8_t l3_default_patch(uint32_t width, uint32_t height);

/* Upper bound, in bytes, of the encoded size of any width x height image with
 * patch size `patch` (0 = l3_default_patch).  0 if an argument is invalid. */
size_t l3_encode_bound(uint32_t width, uint32_t height, uint8_t patch);

/* Section 4.2 + 4.3, encoder: interleaved 8-bit RGB (host, rows `row_stride`
 * bytes apart, row_stride >= 3*width) -> one L3 file written to `out` (host,
 * capacity out_cap); *out_len receives its length.  patch = 0 selects
 * l3_default_patch.  Deterministic: minimal width per row, base = row minimum
 * (rows after the first taken as signed bytes).
 * Errors: INVALID_ARG (NULL, zero size, stride too small), BUFFER_TOO_SMALL
 * (nothing useful is left in out), UNSUPPORTED (encoded data beyond 4 GiB). */
l3_status l3_encode_cpu(const uint8_t* rgb_hwc, uint32_t width, uint32_t height,
                        size_t row_stride, uint8_t patch,
                        uint8_t* out, size_t out_cap, size_t* out_len);

typedef struct {
    uint32_t width, height;          /* pixels */
    uint8_t  patch;                  /* N */
    uint32_t patches_per_channel;    /* ceil(width/N) * ceil(height/N) */
    size_t   header_bytes;           /* 13 + 12 * patches_per_channel */
} l3_info;

/* Section 4.4, header parse on the host ahead of the GPU work: parse and
 * validate the header of a file held in HOST memory (`file`, `len` bytes) and
 * fill *info.  Checks the signature, non-zero sizes, that the header fits in
 * len, that the 3*P offsets start at 0, increase strictly and stay inside the
 * data section, and that every patch is at least as long as its rows' 12-bit
 * records.  Reads nothing outside [file, file+len).
 * Errors: INVALID_ARG, BAD_MAGIC, TRUNCATED, CORRUPT. */
l3_status l3_peek_header(const uint8_t* file, size_t len, l3_info* info);

/* ------------------------------------------------------------------------
 * Device side (one GPU per context)
 * ------------------------------------------------------------------------ */

/* A context holds a small descriptor workspace on one GPU (grown on demand,
 * reused between calls).  Not thread-safe: one thread per context at a time.
 * Calls that share a context must be enqueued on the same stream, or the
 * caller must order them (the workspace is reused). */
typedef struct l3_ctx l3_ctx;

/* Creates a context on HIP device `device`.  Errors: INVALID_ARG, DEVICE. */
l3_status l3_ctx_create(l3_ctx** out, int device);
/* Waits for the context's outstanding work and frees it.  NULL is allowed. */
void l3_ctx_destroy(l3_ctx* ctx);

typedef struct {
    const uint8_t* d_file;     /* DEVICE: the whole L3 file, any alignment */
    size_t         file_len;   /* its length in bytes */
    l3_info        info;       /* HOST copy of what l3_peek_header returned for it */
    uint8_t*       d_out;      /* DEVICE: decoded pixels (unused by the fused call) */
    size_t         out_row_stride; /* bytes between output rows */
} l3_item;

typedef enum {
    L3_LAYOUT_HWC = 0,  /* out[y*stride + 3*x + c]; stride >= 3*width */
    L3_LAYOUT_CHW = 1   /* out[(c*height + y)*stride + x]; stride >= width */
} l3_layout;

/* Section 4.2 (decoding direction) + Section 4.4: decode n files to 8-bit RGB.
 *   items     HOST array of n entries (copied before return); images may differ
 *             in size and patch size.  Each d_file must stay valid and unchanged
 *             until the stream has run the work.  The decoder may read up to 15
 *             bytes past d_file + file_len, never beyond the 16-byte-aligned
 *             block that holds the file's last byte.
 *   d_status  DEVICE array of n u32, or NULL.  Entry i is set to 0 when image i
 *             decoded cleanly and to a non-zero bit mask when its stream is
 *             damaged (bit 0: a row width above 8, bit 1: a patch's rows run past
 *             the patch's end, bit 2: a patch offset outside the data section);
 *             such an image's output is unspecified, nothing is written outside
 *             the image's own output rectangle and nothing is read outside the
 *             file (beyond the 15 bytes above).
 *   stream    a hipStream_t (NULL = the default stream).  The call returns after
 *             enqueueing; completion is observed on the stream.
 * A batch with at most 256 images of each patch size carries its descriptors in the
 * kernel arguments: such a call makes no copy, waits for nothing and (once the context
 * has served a batch of that size) allocates nothing, so it can be captured into a HIP
 * graph; the captured launches keep the pointers and sizes of the capture.  Larger
 * batches go through a pinned descriptor table that a small kernel pulls at run time:
 * not meant for capture.
 * GPU path supports N in {32, 64, 128}; any other N gives UNSUPPORTED.
 * Errors (all synchronous, nothing is enqueued): INVALID_ARG (NULL pointers,
 * n < 0, stride too small, info inconsistent with file_len), UNSUPPORTED,
 * DEVICE.  n == 0 is L3_OK and does nothing. */
l3_status l3_decode_batch(l3_ctx* ctx, const l3_item* items, int n, l3_layout layout,
                          uint32_t* d_status, void* stream);

typedef struct {
    int32_t x0, y0;   /* top-left corner of the crop window inside the image */
    uint8_t flip;     /* non-zero: mirror horizontally inside the window */
} l3_crop;

typedef enum { L3_BF16 = 0, L3_FP16 = 1 } l3_dtype;

/* Training-input path (defined by the benchmark configuration, not by the
 * paper): decode only the patches that intersect each image's crop window and
 * write y = (x/255 - mean[c]) / stdv[c] (IEEE binary32, no contraction, rounded
 * to nearest-even to the 16-bit type) as a dense tensor
 *   d_out_nchw[((i*3 + c)*crop_h + row)*crop_w + col]   (16-bit elements),
 * where col counts from the right edge of the window when crops[i].flip is set.
 * items[i].d_out / out_row_stride are ignored.  crops is a HOST array of n
 * entries; every window must lie inside its image.  mean and stdv are HOST
 * arrays of 3 floats (stdv non-zero).  Other arguments as l3_decode_batch.
 * The 768 possible values of y (l3_normalized_values) travel inside the arguments of the
 * call's kernels: no table in device memory, nothing built ahead of the decode kernel, the
 * same work recorded under stream capture as outside it, and calls with different constants
 * may run at the same time on different streams.  (The context remembers the values of the
 * last call's constants in host memory.)
 * Errors: as l3_decode_batch, plus INVALID_ARG for a window outside its image. */
l3_status l3_decode_crop_normalize_batch(l3_ctx* ctx, const l3_item* items,
                                         const l3_crop* crops, int n,
                                         uint32_t crop_w, uint32_t crop_h,
                                         const float mean[3], const float stdv[3],
                                         l3_dtype dtype, void* d_out_nchw,
                                         uint32_t* d_status, void* stream);

/* The values the fused call can write, as 16-bit patterns: out[c*256 + v] holds
 * y = (v/255 - mean[c]) / stdv[c] for byte value v of channel c, worked out as stated above
 * (IEEE binary32: divide, subtract, divide, each rounded, nothing fused; then rounded to
 * nearest-even to dtype).  Host only; all pointers HOST.  Errors: INVALID_ARG (NULL pointer,
 * unknown dtype). */
l3_status l3_normalized_values(const float mean[3], const float stdv[3], l3_dtype dtype,
                               uint16_t out[768]);

/* For callers that cannot allocate device memory while they run (work recorded under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same call as
 * l3_decode_crop_normalize_batch, with the same arguments, results and errors, that
 * allocates nothing, on the host or on the device.  Its table of normalised values lives in
 * a static device array of the library (1536 bytes per GPU, held until the process ends),
 * which is rebuilt on `stream` by every call; descriptors travel in the kernel arguments.
 * At most L3_NOALLOC_MAX_IMAGES images per call: more give L3_ERR_LIMIT and enqueue
 * nothing (so does an image with more work units than one launch holds).
 * All calls on one GPU, from any context, share that one table: calls that may overlap on
 * the device (different streams) race on it unless they use the same constants. */
#define L3_NOALLOC_MAX_IMAGES 256
l3_status l3_decode_crop_normalize_batch_noalloc(l3_ctx* ctx, const l3_item* items,
                                                 const l3_crop* crops, int n,
                                                 uint32_t crop_w, uint32_t crop_h,
                                                 const float mean[3], const float stdv[3],
                                                 l3_dtype dtype, void* d_out_nchw,
                                                 uint32_t* d_status, void* stream);

typedef struct {
    const uint8_t* d_rgb;      /* DEVICE: interleaved 8-bit RGB, rows row_stride bytes apart */
    size_t         row_stride; /* >= 3 * width */
    uint32_t       width, height;
    uint8_t        patch;      /* N, 1..128; 0 = l3_default_patch */
    uint8_t*       d_file;     /* DEVICE: receives the L3 file */
    size_t         file_cap;   /* its capacity in bytes (l3_encode_bound is always enough) */
} l3_encode_item;

/* Section 4.2 (encoding direction) + Section 4.3 on the GPU: encode n images held
 * in device memory into n L3 files in device memory.  The files are byte for byte
 * the ones l3_encode_cpu writes for the same pixels and patch size.
 *   items       HOST array of n entries (copied before return).
 *   d_file_len  DEVICE array of n u64: entry i receives the length of file i (the
 *               length it needs, if the capacity was too small).
 *   d_status    DEVICE array of n u32, or NULL: 0 = file written; bit 0 = file_cap
 *               too small (header and offsets are written if they fit, no patch
 *               data; nothing is written beyond file_cap); bit 1 = encoded data
 *               beyond 4 GiB (not representable in the format's 32-bit offsets).
 *   stream      a hipStream_t; the call returns after enqueueing.  Calls on one
 *               context share one workspace: on the device a call runs after the
 *               kernels of the previous one, whatever their streams; the host
 *               waits for them only when the workspace has to grow (batches of
 *               more than 32 images, or with a patch size other than 32, 64, 128,
 *               go through a ring of four pinned descriptor tables, so the host
 *               can run at most four such calls ahead of the device).
 * Patch sizes above 128 give UNSUPPORTED.  Errors are synchronous: INVALID_ARG,
 * UNSUPPORTED, DEVICE (a HIP call failed; some kernels may have been enqueued). */
l3_status l3_encode_batch(l3_ctx* ctx, const l3_encode_item* items, int n,
                          uint64_t* d_file_len, uint32_t* d_status, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* L3_H */
