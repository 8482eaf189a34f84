"""ctypes binding of the oracle library (test infrastructure, not the product).

Argument marshalling only; all arithmetic is in l3_oracle.cpp.
"""
import ctypes
import os

import numpy as np

from . import build as _build

__all__ = [
    "OracleError", "patch_rule", "predict", "predict_batch", "encode", "parse_header",
    "decode", "decode_residuals", "decode_patch", "crop_normalize", "f32_to_bf16",
    "f32_to_f16", "predict_original_batch", "PREDICTOR_CUSTOM", "PREDICTOR_ORIGINAL", "ERR_ARG", "ERR_MAGIC", "ERR_TRUNCATED", "ERR_CORRUPT", "ERR_SPACE",
]

OK, ERR_ARG, ERR_MAGIC, ERR_TRUNCATED, ERR_CORRUPT, ERR_SPACE = range(6)


class OracleError(Exception):
    def __init__(self, code, what):
        super().__init__(f"{what}: oracle error {code}")
        self.code = code


class _Info(ctypes.Structure):
    _fields_ = [("width", ctypes.c_uint32), ("height", ctypes.c_uint32),
                ("patch", ctypes.c_uint32), ("px", ctypes.c_uint32), ("py", ctypes.c_uint32),
                ("header_bytes", ctypes.c_uint64), ("data_bytes", ctypes.c_uint64)]


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    path = _build.OUT
    if not os.path.exists(path):
        _build.build(force=True)
    lib = ctypes.CDLL(path)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    lib.l3o_patch_rule.restype = ctypes.c_uint32
    lib.l3o_patch_rule.argtypes = [ctypes.c_uint32, ctypes.c_uint32]
    lib.l3o_predict.restype = ctypes.c_uint8
    lib.l3o_predict.argtypes = [ctypes.c_uint8] * 3
    lib.l3o_predict_batch.restype = None
    lib.l3o_predict_batch.argtypes = [u8p, u8p, u8p, u8p, ctypes.c_size_t]
    lib.l3o_encode_bound.restype = ctypes.c_size_t
    lib.l3o_encode_bound.argtypes = [ctypes.c_uint32] * 3
    lib.l3o_encode.restype = ctypes.c_int
    lib.l3o_encode.argtypes = [u8p, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_size_t,
                               ctypes.c_uint32, ctypes.c_int, u8p, ctypes.c_size_t,
                               ctypes.POINTER(ctypes.c_size_t)]
    lib.l3o_encode_with.restype = ctypes.c_int
    lib.l3o_encode_with.argtypes = [u8p, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_size_t,
                                    ctypes.c_uint32, ctypes.c_int, ctypes.c_int, u8p,
                                    ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
    lib.l3o_decode_with.restype = ctypes.c_int
    lib.l3o_decode_with.argtypes = [u8p, ctypes.c_size_t, ctypes.c_int, u8p, ctypes.c_size_t]
    lib.l3o_decode_patch_with.restype = ctypes.c_int
    lib.l3o_decode_patch_with.argtypes = [u8p, ctypes.c_size_t, ctypes.c_uint32, ctypes.c_uint32,
                                          ctypes.c_int, u8p, ctypes.c_size_t]
    lib.l3o_predict_original.restype = ctypes.c_uint8
    lib.l3o_predict_original.argtypes = [ctypes.c_uint8] * 3
    lib.l3o_predict_original_batch.restype = None
    lib.l3o_predict_original_batch.argtypes = [u8p, u8p, u8p, u8p, ctypes.c_size_t]
    lib.l3o_parse_header.restype = ctypes.c_int
    lib.l3o_parse_header.argtypes = [u8p, ctypes.c_size_t, ctypes.POINTER(_Info)]
    lib.l3o_decode.restype = ctypes.c_int
    lib.l3o_decode.argtypes = [u8p, ctypes.c_size_t, u8p, ctypes.c_size_t]
    lib.l3o_decode_residuals.restype = ctypes.c_int
    lib.l3o_decode_residuals.argtypes = [u8p, ctypes.c_size_t, u8p]
    lib.l3o_decode_patch.restype = ctypes.c_int
    lib.l3o_decode_patch.argtypes = [u8p, ctypes.c_size_t, ctypes.c_uint32, ctypes.c_uint32,
                                     u8p, ctypes.c_size_t]
    f3 = ctypes.POINTER(ctypes.c_float)
    lib.l3o_crop_normalize.restype = ctypes.c_int
    lib.l3o_crop_normalize.argtypes = [u8p, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_size_t,
                                       ctypes.c_int32, ctypes.c_int32, ctypes.c_int,
                                       ctypes.c_uint32, ctypes.c_uint32, f3, f3, ctypes.c_int,
                                       ctypes.POINTER(ctypes.c_uint16)]
    lib.l3o_f32_to_bf16.restype = ctypes.c_uint16
    lib.l3o_f32_to_bf16.argtypes = [ctypes.c_float]
    lib.l3o_f32_to_f16.restype = ctypes.c_uint16
    lib.l3o_f32_to_f16.argtypes = [ctypes.c_float]
    _lib = lib
    return lib


def _u8(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def _bytes_arr(b):
    a = np.frombuffer(b, dtype=np.uint8) if not isinstance(b, np.ndarray) else b
    return np.ascontiguousarray(a, dtype=np.uint8)


def patch_rule(width, height):
    return int(_load().l3o_patch_rule(width, height))


def predict(tl, t, tr):
    return int(_load().l3o_predict(tl, t, tr))


def predict_batch(tl, t, tr):
    tl, t, tr = (np.ascontiguousarray(v, dtype=np.uint8).ravel() for v in (tl, t, tr))
    out = np.empty_like(t)
    _load().l3o_predict_batch(_u8(tl), _u8(t), _u8(tr), _u8(out), t.size)
    return out


PREDICTOR_CUSTOM, PREDICTOR_ORIGINAL = 0, 1


def predict_original_batch(left, top, top_left):
    left, top, top_left = (np.ascontiguousarray(v, dtype=np.uint8).ravel()
                           for v in (left, top, top_left))
    out = np.empty_like(top)
    _load().l3o_predict_original_batch(_u8(left), _u8(top), _u8(top_left), _u8(out), top.size)
    return out


def encode(rgb, patch=0, width_mode=0, predictor=PREDICTOR_CUSTOM):
    """rgb: uint8 array [H, W, 3] (rows may be strided).  Returns bytes."""
    rgb = np.asarray(rgb)
    assert rgb.dtype == np.uint8 and rgb.ndim == 3 and rgb.shape[2] == 3
    if rgb.strides[2] != 1 or rgb.strides[1] != 3:
        rgb = np.ascontiguousarray(rgb)
    h, w = rgb.shape[:2]
    lib = _load()
    cap = lib.l3o_encode_bound(w, h, patch)
    out = np.empty(cap, dtype=np.uint8)
    n = ctypes.c_size_t(0)
    rc = lib.l3o_encode_with(_u8(rgb), w, h, rgb.strides[0], patch, width_mode, predictor,
                             _u8(out), cap, ctypes.byref(n))
    if rc != OK:
        raise OracleError(rc, "encode")
    return out[:n.value].tobytes()


def parse_header(file):
    a = _bytes_arr(file)
    info = _Info()
    rc = _load().l3o_parse_header(_u8(a), a.size, ctypes.byref(info))
    if rc != OK:
        raise OracleError(rc, "parse_header")
    return {k: int(getattr(info, k)) for k, _ in _Info._fields_}


def decode(file, row_stride=None, predictor=PREDICTOR_CUSTOM):
    a = _bytes_arr(file)
    info = parse_header(a)
    w, h = info["width"], info["height"]
    stride = row_stride or 3 * w
    out = np.zeros((h, stride), dtype=np.uint8)
    rc = _load().l3o_decode_with(_u8(a), a.size, predictor, _u8(out), stride)
    if rc != OK:
        raise OracleError(rc, "decode")
    return out[:, :3 * w].reshape(h, w, 3)


def decode_residuals(file):
    a = _bytes_arr(file)
    info = parse_header(a)
    out = np.zeros((3, info["height"], info["width"]), dtype=np.uint8)
    rc = _load().l3o_decode_residuals(_u8(a), a.size, _u8(out))
    if rc != OK:
        raise OracleError(rc, "decode_residuals")
    return out


def decode_patch(stream, pw, ph, predictor=PREDICTOR_CUSTOM):
    a = _bytes_arr(stream)
    out = np.zeros((ph, pw), dtype=np.uint8)
    rc = _load().l3o_decode_patch_with(_u8(a), a.size, pw, ph, predictor, _u8(out), pw)
    if rc != OK:
        raise OracleError(rc, "decode_patch")
    return out


def crop_normalize(rgb, x0, y0, flip, crop_w, crop_h, mean, stdv, dtype=0):
    rgb = np.ascontiguousarray(rgb, dtype=np.uint8)
    h, w = rgb.shape[:2]
    m = (ctypes.c_float * 3)(*mean)
    s = (ctypes.c_float * 3)(*stdv)
    out = np.zeros((3, crop_h, crop_w), dtype=np.uint16)
    rc = _load().l3o_crop_normalize(_u8(rgb), w, h, rgb.strides[0], x0, y0, int(flip), crop_w,
                                    crop_h, m, s, dtype,
                                    out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)))
    if rc != OK:
        raise OracleError(rc, "crop_normalize")
    return out


def f32_to_bf16(x):
    return int(_load().l3o_f32_to_bf16(x))


def f32_to_f16(x):
    return int(_load().l3o_f32_to_f16(x))
