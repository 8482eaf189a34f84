"""Test-side helpers written independently of the oracle and of the GPU path.

A tiny pure-Python reading of the L3 container (Section 4.3) and of the patch
stream (Section 4.2), used to take files apart, to assemble streams by hand and
to cross-check both implementations on small inputs.  Slow on purpose.
"""
import struct

import numpy as np

MAGIC = bytes([0x4C, 0x33, 0x00, 0x01])


def read_golden(path):
    """key value... lines, '#' comments -> dict of key -> list of tokens."""
    out = {}
    with open(path) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if line:
                key, *vals = line.split()
                out[key] = vals
    return out


def split_file(file):
    """-> dict(width, height, patch, px, py, offsets[3][P], data(bytes), streams[c][i])."""
    file = bytes(file)
    assert file[:4] == MAGIC
    w, h = struct.unpack_from("<II", file, 4)
    n = file[12]
    px, py = -(-w // n), -(-h // n)
    p = px * py
    flat = list(struct.unpack_from("<%dI" % (3 * p), file, 13))
    data = file[13 + 12 * p:]
    ends = flat[1:] + [len(data)]
    streams = [[data[flat[c * p + i]:ends[c * p + i]] for i in range(p)] for c in range(3)]
    return dict(width=w, height=h, patch=n, px=px, py=py, offsets=[flat[c * p:(c + 1) * p]
                for c in range(3)], data=data, streams=streams, header_bytes=13 + 12 * p)


def patch_rect(info, i):
    n = info["patch"]
    tx, ty = i % info["px"], i // info["px"]
    x0, y0 = tx * n, ty * n
    return x0, y0, min(n, info["width"] - x0), min(n, info["height"] - y0)


def join_file(width, height, patch, streams):
    """Inverse of split_file: streams[c][i] bytes -> file bytes."""
    p = len(streams[0])
    offs, pos, data = [], 0, b""
    for c in range(3):
        for i in range(p):
            offs.append(pos)
            data += streams[c][i]
            pos += len(streams[c][i])
    return MAGIC + struct.pack("<II", width, height) + bytes([patch]) + \
        struct.pack("<%dI" % (3 * p), *offs) + data


class Bits:
    """LSB-first bit string builder / reader over Python ints."""

    def __init__(self, data=b""):
        self.value = int.from_bytes(data, "little")
        self.nbits = 8 * len(data)
        self.pos = 0

    def put(self, v, width):
        assert 0 <= v < (1 << width) or width == 0 and v == 0
        self.value |= v << self.nbits
        self.nbits += width

    def get(self, width):
        if self.pos + width > self.nbits:
            raise EOFError
        v = (self.value >> self.pos) & ((1 << width) - 1)
        self.pos += width
        return v

    def tobytes(self):
        return self.value.to_bytes((self.nbits + 7) // 8, "little")


def pack_rows(rows):
    """rows: list of (width, base, [deltas]) -> patch stream bytes."""
    b = Bits()
    for width, base, deltas in rows:
        b.put(width, 4)
        b.put(base & 0xFF, 8)
        for d in deltas:
            b.put(d, width)
    return b.tobytes()


def py_predict(tl, t, tr):
    ref = tl + tr - t
    cands = [(abs(ref - tl), 0, tl), (abs(ref - tr), 1, tr), (abs(ref - t), 2, t)]
    return min(cands)[2]          # nearest; ties by order TL, TR, T


def py_decode_patch(stream, pw, ph):
    b = Bits(stream)
    out = np.zeros((ph, pw), dtype=np.int64)
    for r in range(ph):
        width, base = b.get(4), b.get(8)
        assert width <= 8
        v = [(base + b.get(width)) & 255 for _ in range(pw)]
        for x in range(pw):
            if r == 0:
                pred = 0
            elif x == 0 or x == pw - 1:
                pred = out[r - 1, x]
            else:
                pred = py_predict(int(out[r - 1, x - 1]), int(out[r - 1, x]), int(out[r - 1, x + 1]))
            out[r, x] = (pred + v[x]) & 255
    return out.astype(np.uint8)


def py_decode(file):
    info = split_file(file)
    img = np.zeros((info["height"], info["width"], 3), dtype=np.uint8)
    for c in range(3):
        for i, s in enumerate(info["streams"][c]):
            x0, y0, pw, ph = patch_rect(info, i)
            img[y0:y0 + ph, x0:x0 + pw, c] = py_decode_patch(s, pw, ph)
    return img


def row_widths_from_residuals(resid_patch):
    """Independent recomputation of each row's minimal width from a residual patch."""
    widths = []
    for r, row in enumerate(resid_patch):
        v = row.astype(np.int64)
        if r > 0:
            v = np.where(v >= 128, v - 256, v)
        widths.append(int(int(v.max() - v.min())).bit_length())
    return widths
