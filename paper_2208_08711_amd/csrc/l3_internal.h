/*
 * Internal declarations shared by the host planner and the gfx950 kernels of
 * the L3 decoder.  Not part of the public ABI (see include/l3.h).
 */
#ifndef L3_INTERNAL_H
#define L3_INTERNAL_H

#include <stdint.h>

#include "l3.h"

/* One entry per image of a launch, read by every wave that works on the image
 * (Section 4.4: the host reads the header and hands the GPU what it needs to
 * enumerate the patches). */
struct L3ImageDesc {
    const uint8_t* file;      /* device: start of the L3 file */
    uint8_t* out;             /* device: output of this image */
    uint64_t file_len;
    uint64_t row_stride;      /* bytes between output rows (pixel modes) */
    uint64_t plane_stride;    /* bytes between channel planes (CHW and tensor modes) */
    uint32_t width, height;
    uint32_t tiles_x, tiles_y;      /* patches per row / column */
    uint32_t header_bytes;          /* 13 + 12 * tiles_x * tiles_y */
    uint32_t status_index;          /* which d_status word belongs to this image */
    uint32_t tile_x_first, tile_y_first; /* first patch column / row to decode */
    uint32_t tile_x_count;               /* patch columns to decode */
    uint32_t groups_x;                   /* wave work units per patch row; 0: flat order (below) */
    uint32_t units;                      /* work units of this image */
    int32_t crop_x0, crop_y0;            /* tensor mode: window origin */
    uint32_t flip;                       /* tensor mode: mirror inside the window */
    /* Flat order (pixel modes): a unit takes consecutive patches in row-major order, also
     * across the end of a patch row, so that only the last unit of a block has idle lane
     * groups.  The patch rows of full height form the upper block; a shorter last row is
     * a block of its own, so that all patches of a unit have the same number of rows. */
    uint32_t flat_upper_rows;            /* patch rows in the upper block */
    uint32_t flat_upper_units;           /* units of the upper block */
    uint32_t pad_;
};

/* bits of a d_status word */
enum {
    L3_STATUS_BAD_WIDTH = 1u,
    L3_STATUS_OVERRUN = 2u,
    L3_STATUS_BAD_OFFSET = 4u
};

enum { L3_MODE_HWC = 0, L3_MODE_CHW = 1, L3_MODE_TENSOR = 2 };

/* Host planning for the pixel modes (whole image): deals the image's patches to work units
 * of tpw patches.  Needs width, height, tiles_x, tiles_y and row_stride of *d; sets the
 * tile window, groups_x, units and the flat_ fields.  Per-row order: groups_x units per
 * patch row.  Flat order (only if flat_ok, where it saves units and the lanes' 32-bit
 * offsets reach far enough): see the flat_ fields of L3ImageDesc.  (l3_host.cpp) */
void l3_plan_units(L3ImageDesc* d, uint32_t patch, uint32_t tpw, bool flat_ok);

#endif
