"""Thin ctypes binding of the C ABI declared in include/l3.h.

Same names as the C entry points (without the l3_ prefix); argument marshalling
only.  torch is used for device memory and streams, nothing else.  There is no
CPU fallback: if libl3.so is missing, every call raises.
"""
import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
# L3_LIBRARY selects another build of the same library (for experiments)
_LIB_PATH = os.environ.get("L3_LIBRARY") or os.path.join(HERE, "libl3.so")

LAYOUT_HWC, LAYOUT_CHW = 0, 1
BF16, FP16 = 0, 1

EXPORTED_SYMBOLS = (
    "l3_status_string", "l3_default_patch", "l3_encode_bound", "l3_encode_cpu", "l3_peek_header",
    "l3_normalized_values",
    "l3_ctx_create", "l3_ctx_destroy", "l3_decode_batch", "l3_decode_crop_normalize_batch",
    "l3_decode_crop_normalize_batch_noalloc", "l3_encode_batch", "l3_ablation_encode_cpu", "l3_ablation_decode_batch",
)


class L3Error(RuntimeError):
    def __init__(self, code, what):
        self.code = int(code)
        super().__init__(f"{what}: {status_string(code)} (l3_status {int(code)})")


class Info(ctypes.Structure):
    _fields_ = [("width", ctypes.c_uint32), ("height", ctypes.c_uint32),
                ("patch", ctypes.c_uint8), ("patches_per_channel", ctypes.c_uint32),
                ("header_bytes", ctypes.c_size_t)]


class _Item(ctypes.Structure):
    _fields_ = [("d_file", ctypes.c_void_p), ("file_len", ctypes.c_size_t), ("info", Info),
                ("d_out", ctypes.c_void_p), ("out_row_stride", ctypes.c_size_t)]


class _EncodeItem(ctypes.Structure):
    _fields_ = [("d_rgb", ctypes.c_void_p), ("row_stride", ctypes.c_size_t),
                ("width", ctypes.c_uint32), ("height", ctypes.c_uint32), ("patch", ctypes.c_uint8),
                ("d_file", ctypes.c_void_p), ("file_cap", ctypes.c_size_t)]


class _Crop(ctypes.Structure):
    _fields_ = [("x0", ctypes.c_int32), ("y0", ctypes.c_int32), ("flip", ctypes.c_uint8)]


_lib = None


def library_path():
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2208_08711_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    lib.l3_status_string.restype = ctypes.c_char_p
    lib.l3_status_string.argtypes = [ctypes.c_int]
    lib.l3_default_patch.restype = ctypes.c_uint8
    lib.l3_default_patch.argtypes = [ctypes.c_uint32, ctypes.c_uint32]
    lib.l3_encode_bound.restype = ctypes.c_size_t
    lib.l3_encode_bound.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint8]
    lib.l3_encode_cpu.restype = ctypes.c_int
    lib.l3_encode_cpu.argtypes = [u8p, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_size_t,
                                  ctypes.c_uint8, u8p, ctypes.c_size_t,
                                  ctypes.POINTER(ctypes.c_size_t)]
    lib.l3_ablation_encode_cpu.restype = ctypes.c_int
    lib.l3_ablation_encode_cpu.argtypes = [u8p, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_size_t,
                                           ctypes.c_uint8, ctypes.c_int, u8p, ctypes.c_size_t,
                                           ctypes.POINTER(ctypes.c_size_t)]
    lib.l3_ablation_decode_batch.restype = ctypes.c_int
    lib.l3_ablation_decode_batch.argtypes = [ctypes.c_void_p, ctypes.POINTER(_Item), ctypes.c_int,
                                             ctypes.c_int, ctypes.c_void_p]
    lib.l3_peek_header.restype = ctypes.c_int
    lib.l3_peek_header.argtypes = [u8p, ctypes.c_size_t, ctypes.POINTER(Info)]
    lib.l3_normalized_values.restype = ctypes.c_int
    lib.l3_normalized_values.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float),
                                         ctypes.c_int, ctypes.POINTER(ctypes.c_uint16)]
    lib.l3_ctx_create.restype = ctypes.c_int
    lib.l3_ctx_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int]
    lib.l3_ctx_destroy.restype = None
    lib.l3_ctx_destroy.argtypes = [ctypes.c_void_p]
    lib.l3_decode_batch.restype = ctypes.c_int
    lib.l3_decode_batch.argtypes = [ctypes.c_void_p, ctypes.POINTER(_Item), ctypes.c_int,
                                    ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    lib.l3_decode_crop_normalize_batch.restype = ctypes.c_int
    lib.l3_decode_crop_normalize_batch.argtypes = [
        ctypes.c_void_p, ctypes.POINTER(_Item), ctypes.POINTER(_Crop), ctypes.c_int,
        ctypes.c_uint32, ctypes.c_uint32, ctypes.POINTER(ctypes.c_float),
        ctypes.POINTER(ctypes.c_float), ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_void_p]
    lib.l3_decode_crop_normalize_batch_noalloc.restype = ctypes.c_int
    lib.l3_decode_crop_normalize_batch_noalloc.argtypes = lib.l3_decode_crop_normalize_batch.argtypes
    lib.l3_encode_batch.restype = ctypes.c_int
    lib.l3_encode_batch.argtypes = [ctypes.c_void_p, ctypes.POINTER(_EncodeItem), ctypes.c_int,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    _lib = lib
    return lib


def status_string(code):
    return _load().l3_status_string(int(code)).decode()


def _check(code, what):
    if code != 0:
        raise L3Error(code, what)


def _u8(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def default_patch(width, height):
    return int(_load().l3_default_patch(width, height))


def encode_bound(width, height, patch=0):
    return int(_load().l3_encode_bound(width, height, patch))


def encode_cpu(rgb, patch=0, original_filter=False):
    """rgb: uint8 numpy array [H, W, 3] (host).  Returns the L3 file as bytes.
    original_filter=True writes the ablation baseline's files (l3_ablation_encode_cpu)."""
    rgb = np.asarray(rgb)
    if rgb.dtype != np.uint8 or rgb.ndim != 3 or rgb.shape[2] != 3:
        raise ValueError("expected uint8 [H, W, 3]")
    if rgb.strides[2] != 1 or rgb.strides[1] != 3:
        rgb = np.ascontiguousarray(rgb)
    h, w = rgb.shape[:2]
    lib = _load()
    cap = lib.l3_encode_bound(w, h, patch)
    out = np.empty(max(cap, 1), dtype=np.uint8)
    n = ctypes.c_size_t(0)
    if original_filter:
        _check(lib.l3_ablation_encode_cpu(_u8(rgb), w, h, rgb.strides[0], patch, 1, _u8(out), cap,
                                          ctypes.byref(n)), "l3_ablation_encode_cpu")
    else:
        _check(lib.l3_encode_cpu(_u8(rgb), w, h, rgb.strides[0], patch, _u8(out), cap,
                                 ctypes.byref(n)), "l3_encode_cpu")
    return out[:n.value].tobytes()


def peek_header(file):
    """file: bytes-like or uint8 numpy array in host memory.  Returns an Info."""
    a = np.frombuffer(file, dtype=np.uint8) if not isinstance(file, np.ndarray) else file
    a = np.ascontiguousarray(a, dtype=np.uint8)
    info = Info()
    _check(_load().l3_peek_header(_u8(a), a.size, ctypes.byref(info)), "l3_peek_header")
    return info


def normalized_values(mean, stdv, dtype=0):
    """l3_normalized_values: uint16 numpy array [3, 256] of the bit patterns the fused call
    writes for every byte value of every channel (dtype: BF16 = 0 or FP16 = 1)."""
    m = (ctypes.c_float * 3)(*mean)
    s = (ctypes.c_float * 3)(*stdv)
    out = np.empty((3, 256), dtype=np.uint16)
    _check(_load().l3_normalized_values(m, s, int(dtype), out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))),
           "l3_normalized_values")
    return out


class Context:
    """Owns one l3_ctx (a small descriptor workspace on one GPU)."""

    def __init__(self, device=0):
        self._h = ctypes.c_void_p()
        _check(_load().l3_ctx_create(ctypes.byref(self._h), int(device)), "l3_ctx_create")

    def close(self):
        if self._h:
            _load().l3_ctx_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h


def _items(files, infos, outs, strides):
    n = len(files)
    arr = (_Item * max(n, 1))()
    for i in range(n):
        f = files[i]
        arr[i].d_file = f.data_ptr()
        arr[i].file_len = f.numel()
        arr[i].info = infos[i]
        if outs is not None:
            arr[i].d_out = outs[i].data_ptr()
            arr[i].out_row_stride = strides[i]
    return arr


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def decode_batch(ctx, files, infos, outs, layout=LAYOUT_HWC, status=None, stream=None,
                 row_strides=None):
    """files: list of uint8 device tensors (whole L3 files); infos: list of Info;
    outs: list of uint8 device tensors to decode into ([H, W, 3] for HWC, [3, H, W] for
    CHW, contiguous unless row_strides is given); status: optional int32/uint32 device
    tensor of len(files) words.  Enqueues on `stream` (default: torch's current)."""
    n = len(files)
    if row_strides is None:
        row_strides = [int(infos[i].width) * (3 if layout == LAYOUT_HWC else 1) for i in range(n)]
    arr = _items(files, infos, outs, row_strides)
    _check(_load().l3_decode_batch(ctx.handle, arr, n, layout,
                                   ctypes.c_void_p(status.data_ptr() if status is not None else None),
                                   _stream_ptr(stream)), "l3_decode_batch")


ABLATION_PIXEL_BD, ABLATION_CUSTOM_FILTER, ABLATION_SERIAL_PATCHES, ABLATION_DIAGONAL = 1, 2, 4, 8


def ablation_decode_batch(ctx, batch, variant, stream=None):
    """l3_ablation_decode_batch on a PreparedBatch (interleaved RGB outputs)."""
    _check(_load().l3_ablation_decode_batch(ctx.handle, batch.items, batch.n, int(variant),
                                            _stream_ptr(stream)), "l3_ablation_decode_batch")


class PreparedBatch:
    """Marshalled l3_item array, reusable across calls (keeps the tensors alive)."""

    def __init__(self, files, infos, outs, layout=LAYOUT_HWC, row_strides=None):
        n = len(files)
        if row_strides is None:
            row_strides = [int(infos[i].width) * (3 if layout == LAYOUT_HWC else 1)
                           for i in range(n)]
        self.n, self.layout = n, layout
        self.items = _items(files, infos, outs, row_strides)
        self._keep = (files, outs)


def decode_batch_prepared(ctx, batch, status=None, stream=None):
    """l3_decode_batch on a PreparedBatch: no per-call marshalling."""
    _check(_load().l3_decode_batch(ctx.handle, batch.items, batch.n, batch.layout,
                                   ctypes.c_void_p(status.data_ptr() if status is not None else None),
                                   _stream_ptr(stream)), "l3_decode_batch")


NOALLOC_MAX_IMAGES = 256


def decode_crop_normalize_batch(ctx, files, infos, crops, crop_w, crop_h, mean, stdv, out,
                                dtype=BF16, status=None, stream=None, noalloc=False):
    """crops: list of (x0, y0, flip); out: 16-bit device tensor [n, 3, crop_h, crop_w].
    noalloc=True calls l3_decode_crop_normalize_batch_noalloc with the same arguments."""
    n = len(files)
    arr = _items(files, infos, None, None)
    cr = (_Crop * max(n, 1))()
    for i, (x0, y0, flip) in enumerate(crops):
        cr[i].x0, cr[i].y0, cr[i].flip = int(x0), int(y0), int(bool(flip))
    m = (ctypes.c_float * 3)(*mean)
    s = (ctypes.c_float * 3)(*stdv)
    lib = _load()
    call = lib.l3_decode_crop_normalize_batch_noalloc if noalloc else lib.l3_decode_crop_normalize_batch
    _check(call(
        ctx.handle, arr, cr, n, crop_w, crop_h, m, s, dtype, ctypes.c_void_p(out.data_ptr()),
        ctypes.c_void_p(status.data_ptr() if status is not None else None), _stream_ptr(stream)),
        "l3_decode_crop_normalize_batch_noalloc" if noalloc else "l3_decode_crop_normalize_batch")


class PreparedCropBatch:
    """Marshalled l3_item and l3_crop arrays for the fused call, reusable across calls."""

    def __init__(self, files, infos, crops, mean, stdv):
        self.n = len(files)
        self.items = _items(files, infos, None, None)
        self.crops = (_Crop * max(self.n, 1))()
        for i, (x0, y0, flip) in enumerate(crops):
            self.crops[i].x0, self.crops[i].y0, self.crops[i].flip = int(x0), int(y0), int(bool(flip))
        self.mean = (ctypes.c_float * 3)(*mean)
        self.stdv = (ctypes.c_float * 3)(*stdv)
        self._keep = files


def decode_crop_normalize_batch_prepared(ctx, batch, crop_w, crop_h, out, dtype=BF16, status=None,
                                         stream=None):
    """l3_decode_crop_normalize_batch on a PreparedCropBatch: no per-call marshalling."""
    _check(_load().l3_decode_crop_normalize_batch(
        ctx.handle, batch.items, batch.crops, batch.n, crop_w, crop_h, batch.mean, batch.stdv, dtype,
        ctypes.c_void_p(out.data_ptr()),
        ctypes.c_void_p(status.data_ptr() if status is not None else None), _stream_ptr(stream)),
        "l3_decode_crop_normalize_batch")


def encode_batch(ctx, images, files, file_len, patch=0, status=None, stream=None, row_strides=None):
    """images: list of uint8 device tensors [H, W, 3] (rows contiguous unless row_strides is
    given); files: list of uint8 device tensors that receive the L3 files; file_len: int64 (or
    uint64) device tensor of len(images) words; patch: one N for all or a list."""
    n = len(images)
    arr = (_EncodeItem * max(n, 1))()
    for i in range(n):
        h, w = int(images[i].shape[0]), int(images[i].shape[1])
        arr[i].d_rgb = images[i].data_ptr()
        arr[i].row_stride = row_strides[i] if row_strides is not None else 3 * w
        arr[i].width, arr[i].height = w, h
        arr[i].patch = patch[i] if isinstance(patch, (list, tuple)) else patch
        arr[i].d_file = files[i].data_ptr()
        arr[i].file_cap = files[i].numel()
    _check(_load().l3_encode_batch(ctx.handle, arr, n, ctypes.c_void_p(file_len.data_ptr()),
                                   ctypes.c_void_p(status.data_ptr() if status is not None else None),
                                   _stream_ptr(stream)), "l3_encode_batch")
