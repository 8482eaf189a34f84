"""Pins of the oracle's *original* Paeth filter (left, top, top-left), which only the
decoder ablation of arxiv 2208.08711 Section 5.5 uses as its baseline.

Section 4.2 points to PNG as the best-known user of that filter: PNG's scanline
filter type 4 is that predictor, with pixels outside the image counting as 0.  So a patch's residual plane, written out as PNG scanlines (row 0 with filter
type 0 = raw, every later row with type 4), must be decoded by an independent PNG
reader to the original pixels.  No GPU needed.
"""
import io
import struct
import zlib

import numpy as np
import pytest

import oracle
from oracle import binding as ob
from paper_2208_08711_amd import synth

PIL_Image = pytest.importorskip("PIL.Image")


def _png_from_scanlines(width, height, filter_types, rows):
    """8-bit greyscale PNG whose IDAT holds exactly these filter bytes and row bytes."""
    def chunk(kind, body):
        return (struct.pack(">I", len(body)) + kind + body +
                struct.pack(">I", zlib.crc32(kind + body) & 0xFFFFFFFF))
    raw = b"".join(bytes([ft]) + bytes(r) for ft, r in zip(filter_types, rows))
    return (b"\x89PNG\r\n\x1a\n" +
            chunk(b"IHDR", struct.pack(">IIBBBBB", width, height, 8, 0, 0, 0, 0)) +
            chunk(b"IDAT", zlib.compress(raw)) + chunk(b"IEND", b""))


def _images():
    yield synth.gradient_noise(5, 40, 23, sigma=2.0)
    yield synth.voronoi_scene(6, 61, 37, sites=7)
    yield synth.uniform_bytes(7, 19, 31)
    yield synth.cosine_field(8, 33, 9)


@pytest.mark.parametrize("patch", [16, 64])
def test_residuals_are_png_filter_4_scanlines(patch):
    """Every patch of every channel: residual rows fed to a PNG decoder as filter-4
    scanlines give back the patch.  Catches a wrong neighbour (top-right for left), a
    wrong tie order (PNG: left, top, top-left), a flipped residual sign, a filtered
    first row and a wrong first column."""
    for img in _images():
        h, w = img.shape[:2]
        f = oracle.encode(img, patch=patch, predictor=ob.PREDICTOR_ORIGINAL)
        res = oracle.decode_residuals(f)
        for c in range(3):
            for y0 in range(0, h, patch):
                for x0 in range(0, w, patch):
                    ph, pw = min(patch, h - y0), min(patch, w - x0)
                    rows = [res[c, y0 + r, x0:x0 + pw] for r in range(ph)]
                    png = _png_from_scanlines(pw, ph, [0] + [4] * (ph - 1), rows)
                    got = np.array(PIL_Image.open(io.BytesIO(png)).convert("L"))
                    assert np.array_equal(got, img[y0:y0 + ph, x0:x0 + pw, c])


def test_original_predictor_exhaustive():
    """All 256^3 triples: one of the inputs, at minimal distance from
    left + top - top_left, ties left, top, top-left; distances equal |top - tl|,
    |left - tl| and |left + top - 2 tl|."""
    top, tl_ = np.meshgrid(np.arange(256, dtype=np.int32), np.arange(256, dtype=np.int32),
                           indexing="ij")
    top, tl_ = top.ravel(), tl_.ravel()
    for a in range(256):
        left = np.full_like(top, a)
        got = ob.predict_original_batch(left, top, tl_).astype(np.int32)
        d_left, d_top = np.abs(top - tl_), np.abs(left - tl_)
        d_tl = np.abs(left + top - 2 * tl_)
        best = np.minimum(np.minimum(d_left, d_top), d_tl)
        want = np.where(d_left == best, left, np.where(d_top == best, top, tl_))
        assert np.array_equal(got, want)


def test_original_round_trip_and_difference_from_custom():
    """decode(encode(x)) == x with the original filter on ragged, multi-patch images;
    the same file read with the custom filter is a different image (the choice is
    really threaded through), while row 0 and every patch's first row agree (raw)."""
    for img in _images():
        for patch in (7, 32):
            f = oracle.encode(img, patch=patch, predictor=ob.PREDICTOR_ORIGINAL)
            assert np.array_equal(oracle.decode(f, predictor=ob.PREDICTOR_ORIGINAL), img)
            other = oracle.decode(f)
            assert np.array_equal(other[::patch], img[::patch])
    img = synth.voronoi_scene(6, 61, 37, sites=7)
    f = oracle.encode(img, patch=32, predictor=ob.PREDICTOR_ORIGINAL)
    assert not np.array_equal(oracle.decode(f), img)


def test_original_hand_worked_patch():
    """2 x 3 patch worked by hand.  Row 0 raw: 10 20 30.  Row 1 pixels 12 25 29:
    x=0: predict top 10 -> 2;  x=1: left 12, top 20, tl 10: ref 22, distances 10, 2, 12
    -> top 20 -> 5;  x=2: left 25, top 30, tl 20: ref 35, distances 10, 5, 15 -> top 30
    -> -1 = 255."""
    img = np.zeros((2, 3, 3), dtype=np.uint8)
    img[0, :, :] = np.array([10, 20, 30])[:, None]
    img[1, :, :] = np.array([12, 25, 29])[:, None]
    f = oracle.encode(img, patch=3, predictor=ob.PREDICTOR_ORIGINAL)
    res = oracle.decode_residuals(f)
    assert res[0, 0].tolist() == [10, 20, 30]
    assert res[0, 1].tolist() == [2, 5, 255]
