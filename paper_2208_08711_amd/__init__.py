"""MI355X-native batched decoder for the L3 lossless image format (arxiv 2208.08711).

The work is done by hand-written gfx950 kernels behind a C ABI (include/l3.h,
built into libl3.so next to this file).  This package only marshals arguments.
"""
from .binding import (  # noqa: F401
    L3Error, Context, Info, default_patch, encode_bound, encode_cpu, peek_header, normalized_values,
    decode_batch, decode_crop_normalize_batch, PreparedBatch, decode_batch_prepared,
    PreparedCropBatch, decode_crop_normalize_batch_prepared, encode_batch, library_path, status_string,
    LAYOUT_HWC, LAYOUT_CHW, BF16, FP16, EXPORTED_SYMBOLS, NOALLOC_MAX_IMAGES,
    ablation_decode_batch, ABLATION_PIXEL_BD, ABLATION_CUSTOM_FILTER, ABLATION_SERIAL_PATCHES, ABLATION_DIAGONAL,
)
