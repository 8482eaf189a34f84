"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these needs a GPU.  Each test names the passage of arxiv 2208.08711 it
pins and the mistake it would catch.
"""
import os
import struct
import subprocess

import numpy as np
import pytest

import oracle
import oracle.build as oracle_build
from paper_2208_08711_amd import synth

import l3_testlib as tl

HERE = os.path.dirname(os.path.abspath(__file__))
GOLD = os.path.join(HERE, "golden")
ROOT = os.path.dirname(HERE)


# ---------------------------------------------------------------------------
# Section 4.2, custom Paeth filter

def test_worked_example_74_65_9():
    """The paper's example: pixel 74, selected neighbour 65, stored 9, decoded 65+9=74.
    Catches a flipped residual sign (neighbour - pixel) and a wrong selection."""
    g = tl.read_golden(os.path.join(GOLD, "paeth_worked_example.txt"))
    a, b, c = int(g["top_left"][0]), int(g["top"][0]), int(g["top_right"][0])
    pixel, sel, res = int(g["pixel"][0]), int(g["selected"][0]), int(g["residual"][0])
    assert oracle.predict(a, b, c) == sel
    img = np.zeros((2, 3, 3), dtype=np.uint8)
    img[0, :, :] = np.array([a, b, c])[:, None]
    img[1, 1, :] = pixel
    img[1, 0, :] = a
    img[1, 2, :] = c
    f = oracle.encode(img, patch=3)
    assert oracle.decode_residuals(f)[0, 1, 1] == res
    assert oracle.decode(f)[1, 1, 0] == sel + res == pixel


def test_predictor_exhaustive_properties():
    """All 256^3 neighbour triples: result is one of the neighbours, at minimal distance
    from TL + TR - T, ties TL then TR then T; closed-form identities; and an
    independently derived form (thirds rule on min/max) gives the same value."""
    t, tr = np.meshgrid(np.arange(256, dtype=np.int32), np.arange(256, dtype=np.int32),
                        indexing="ij")
    t, tr = t.ravel(), tr.ravel()
    for a in range(256):
        tlv = np.full_like(t, a)
        got = oracle.predict_batch(tlv, t, tr).astype(np.int32)
        ref = tlv + tr - t
        da, db, dc = np.abs(ref - tlv), np.abs(ref - tr), np.abs(ref - t)
        best = np.minimum(np.minimum(da, db), dc)
        assert np.all((got == tlv) | (got == t) | (got == tr))
        assert np.all(np.abs(ref - got) == best)
        # tie order: TL whenever it is (one of) the nearest; else TR if nearest; else T
        want = np.where(da == best, tlv, np.where(db == best, tr, t))
        assert np.array_equal(got, want)
        # identities: distances are |TR-T|, |TL-T|, |TL+TR-2T|
        assert np.array_equal(da, np.abs(tr - t)) and np.array_equal(db, np.abs(tlv - t))
        # TL == T -> value TR; TR == T -> value TL
        m = tlv == t
        assert np.array_equal(got[m], tr[m])
        m = tr == t
        assert np.array_equal(got[m], tlv[m])
        # thirds rule: with lo=min(TL,TR), hi=max, S=hi-lo, d=T-lo:
        # 3d <= S -> hi; 3d >= 2S -> lo; else T (value-wise)
        lo, hi = np.minimum(tlv, tr), np.maximum(tlv, tr)
        s, d = hi - lo, t - lo
        alt = np.where(3 * d >= 2 * s, lo, np.where(3 * d <= s, hi, t))
        assert np.array_equal(got, alt)
    # symmetric spread around T selects T
    for d in (1, 2, 50):
        assert oracle.predict(100 - d, 100, 100 + d) == 100


def test_brute_force_tiny_images(tmp_path):
    """Every 1x2 image (exact file bytes in closed form), 2x2 and 3x2 images over a
    grid with one pixel swept 0..255: round trip, raw first row, border rule,
    centre residual nearest-neighbour; all widths 0..8 reached.  Catches wrap
    mistakes, border mistakes and bit-order mistakes."""
    exe = str(tmp_path / "brute")
    libdir = os.path.dirname(oracle_build.OUT)       # where the library under test lies
    subprocess.run(["g++", "-O2", "-std=c++17", "-o", exe,
                    os.path.join(HERE, "native", "brute_force.cpp"),
                    "-I" + os.path.join(ROOT, "oracle"), "-L" + libdir, "-ll3_oracle",
                    "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([exe, "all"], capture_output=True, text=True, timeout=600)
    assert out.returncode == 0, out.stdout
    status, cases, widths = out.stdout.split()
    assert status == "OK" and int(cases) == 65536 + 4 * 512 * 256 + 8 ** 5 * 256
    assert int(widths) == 0x1FF


# ---------------------------------------------------------------------------
# Section 4.2 base-delta record and Section 4.3 file layout

def test_handmade_file_decodes_and_encoder_reproduces_it():
    """A file assembled by hand from the format statement: the decoder must read it,
    the canonical encoder must produce exactly these bytes."""
    g = tl.read_golden(os.path.join(GOLD, "handmade_3x2.txt"))
    w, h, n = int(g["width"][0]), int(g["height"][0]), int(g["patch"][0])
    file = bytes(int(x, 16) for x in g["file"])
    pixels = np.array([int(x) for x in g["pixels"]], dtype=np.uint8).reshape(h, w, 3)
    resid = np.array([int(x) for x in g["residuals"]], dtype=np.uint8).reshape(3, h, w)
    assert np.array_equal(oracle.decode(file), pixels)
    assert np.array_equal(oracle.decode_residuals(file), resid)
    assert oracle.encode(pixels, patch=n) == file
    info = oracle.parse_header(file)
    assert (info["width"], info["height"], info["patch"], info["header_bytes"]) == (w, h, n, 25)


def test_header_layout():
    """4-byte signature, 4-byte width, 4-byte height, 1-byte patch size, three offset
    arrays (Section 4.3)."""
    img = synth.cosine_field(11, 70, 45)
    f = oracle.encode(img, patch=32)
    assert f[:4] == tl.MAGIC
    assert struct.unpack_from("<II", f, 4) == (70, 45)
    assert f[12] == 32
    info = tl.split_file(f)
    assert info["px"] == 3 and info["py"] == 2
    flat = sum(info["offsets"], [])
    assert flat[0] == 0 and all(b > a for a, b in zip(flat, flat[1:]))
    assert flat[-1] < len(info["data"])


def test_patch_rule_thresholds():
    """N = 32 below HD, 64 from HD to FHD, 128 above (Section 4.3)."""
    assert oracle.patch_rule(1079, 720) == 32
    assert oracle.patch_rule(1080, 720) == 64
    assert oracle.patch_rule(1920, 1080) == 64
    assert oracle.patch_rule(1921, 1080) == 128
    assert oracle.patch_rule(2048, 1024) == 128
    assert oracle.patch_rule(3840, 2160) == 128
    assert oracle.patch_rule(5760, 3840) == 128
    assert oracle.patch_rule(500, 375) == 32
    assert oracle.patch_rule(64, 64) == 32


def test_random_image_size_closed_form():
    """Table "compratio", Random column: a uniform-random FHD image compresses to
    1.02x; closed form 6,372,733 bytes.  Catches a wrong record size (not 12 bits),
    per-row byte padding (1.03x), a wrong default N (1.05x / 1.01x)."""
    g = tl.read_golden(os.path.join(GOLD, "compratio_synthetic.txt"))
    img = synth.uniform_bytes(77, 1920, 1080)
    f = oracle.encode(img)
    assert f[12] == 64
    assert len(f) == int(g["random_bytes"][0])
    assert "%.2f" % (len(f) / img.size) == g["paper_random_ratio"][0]
    assert np.array_equal(oracle.decode(f), img)


def test_black_image_size_closed_form():
    """Constant rows carry no payload: every row is one 12-bit record."""
    g = tl.read_golden(os.path.join(GOLD, "compratio_synthetic.txt"))
    img = np.zeros((1080, 1920, 3), dtype=np.uint8)
    f = oracle.encode(img)
    assert len(f) == int(g["black_bytes"][0])
    assert np.array_equal(oracle.decode(f), img)


def test_length_invariant():
    """Patch bytes = ceil(sum_r (12 + pw * w_r) / 8) with w_r recomputed here from the
    residual planes; file = 13 + 12 P + sum of patches."""
    for img, n in ((synth.cosine_field(5, 150, 101), 32), (synth.voronoi_scene(6, 200, 130), 64),
                   (synth.gradient_noise(7, 90, 140, 4.0), 128)):
        f = oracle.encode(img, patch=n)
        info = tl.split_file(f)
        resid = oracle.decode_residuals(f)
        total = info["header_bytes"]
        for c in range(3):
            for i, s in enumerate(info["streams"][c]):
                x0, y0, pw, ph = tl.patch_rect(info, i)
                ws = tl.row_widths_from_residuals(resid[c, y0:y0 + ph, x0:x0 + pw])
                bits = sum(12 + pw * w for w in ws)
                assert len(s) == (bits + 7) // 8
                total += len(s)
        assert total == len(f)


# ---------------------------------------------------------------------------
# losslessness, edges

EDGE_SHAPES = [(1, 1), (1, 7), (7, 1), (2, 2), (31, 33), (33, 31), (65, 63), (129, 127),
               (200, 3), (3, 200)]


@pytest.mark.parametrize("patch", [1, 2, 3, 32, 64, 128, 255])
def test_round_trip_edge_shapes(patch):
    for k, (w, h) in enumerate(EDGE_SHAPES):
        if patch <= 3 and w * h > 2500:
            continue
        for img in (synth.uniform_bytes(100 + k, w, h), synth.cosine_field(200 + k, w, h),
                    np.zeros((h, w, 3), np.uint8), np.full((h, w, 3), 255, np.uint8),
                    (((np.add.outer(np.arange(h), np.arange(w)) & 1) * 255).astype(np.uint8)
                     [:, :, None].repeat(3, axis=2))):
            f = oracle.encode(img, patch=patch)
            assert np.array_equal(oracle.decode(f), img), (w, h, patch)


def test_round_trip_configs_small():
    """The benchmark configurations at reduced batch size (full shapes)."""
    imgs = synth.config1() + synth.config2(3) + synth.config3(1) + \
        [synth.gradient_noise(4000, 640, 360, 2.0, span=255.0), synth.uniform_bytes(4004, 640, 360)]
    for img in imgs:
        f = oracle.encode(img)
        assert np.array_equal(oracle.decode(f), img)
        assert f[12] == oracle.patch_rule(img.shape[1], img.shape[0])


def test_strided_rows():
    img = synth.cosine_field(9, 50, 40)
    padded = np.zeros((40, 200), dtype=np.uint8)
    padded[:, :150] = img.reshape(40, 150)
    view = padded[:, :150].reshape(40, 50, 3)
    f1 = oracle.encode(img, patch=32)
    assert oracle.encode(np.ascontiguousarray(view), patch=32) == f1
    out = oracle.decode(f1, row_stride=256)
    assert np.array_equal(out, img)


def test_small_random_images_against_python_reading():
    """A second, independent reading of the decoder (pure Python, in the tests)."""
    for k in range(12):
        s = synth.Stream(900 + k)
        w, h = int(s.integers(1, 40)[0]), int(s.integers(1, 40)[0])
        n = int(s.integers(1, 48)[0])
        img = synth.cosine_field(300 + k, w, h) if k % 2 else synth.uniform_bytes(300 + k, w, h)
        f = oracle.encode(img, patch=n)
        assert np.array_equal(tl.py_decode(f), img)
        assert np.array_equal(oracle.decode(f), img)


# ---------------------------------------------------------------------------
# special cases with closed-form residuals

def test_constant_and_ramps():
    """Constant -> all widths 0; vertical ramp p = g*y -> residual g, width 0; horizontal
    ramp p = g*x -> interior residual 0 (TL + TR - T = T) and border residual 0."""
    h, w, n = 40, 48, 32
    const = np.full((h, w, 3), 93, dtype=np.uint8)
    f = oracle.encode(const, patch=n)
    info = tl.split_file(f)
    for c in range(3):
        for i, s in enumerate(info["streams"][c]):
            _, _, pw, ph = tl.patch_rect(info, i)
            assert len(s) == (12 * ph + 7) // 8
    r = oracle.decode_residuals(f)
    assert np.all(r[:, 0::n, :][:, 0, :] == 93)

    g = 5
    vr = (g * np.arange(h))[:, None, None].repeat(w, 1).repeat(3, 2).astype(np.uint8)
    r = oracle.decode_residuals(oracle.encode(vr, patch=n))
    for y in range(h):
        assert np.all(r[:, y, :] == (vr[y, 0, 0] if y % n == 0 else g))

    hr = (g * np.arange(w))[None, :, None].repeat(h, 0).repeat(3, 2).astype(np.uint8)
    f = oracle.encode(hr, patch=n)
    r = oracle.decode_residuals(f)
    for y in range(h):
        if y % n:
            assert np.all(r[:, y, :] == 0)
    assert np.array_equal(oracle.decode(f), hr)


def test_wraparound_checkerboard_width():
    """0/255 alternation by row: residuals are +255 / -255 = -1 / +1 mod 256; the signed
    view keeps such rows narrow.  Pins the modulo-256 reading."""
    h, w = 16, 16
    img = np.zeros((h, w, 3), dtype=np.uint8)
    img[1::2] = 255
    f = oracle.encode(img, patch=16)
    r = oracle.decode_residuals(f)
    assert np.all(r[:, 1::2, :] == 255) and np.all(r[:, 2::2, :] == 1)
    info = tl.split_file(f)
    assert len(info["streams"][0][0]) == (12 * h + 7) // 8
    assert np.array_equal(oracle.decode(f), img)


# ---------------------------------------------------------------------------
# segment independence (Section 4.3 / 4.4: patches are decoded independently)

def test_segment_independence():
    img = synth.cosine_field(21, 100, 70)
    f = oracle.encode(img, patch=32)
    info = tl.split_file(f)
    # (a) each patch alone from (offset, length)
    for c in range(3):
        for i, s in enumerate(info["streams"][c]):
            x0, y0, pw, ph = tl.patch_rect(info, i)
            assert np.array_equal(oracle.decode_patch(s, pw, ph), img[y0:y0 + ph, x0:x0 + pw, c])
    # (b) damage inside one patch's payload changes only that patch (or is flagged)
    c, i = 1, 5
    streams = [list(ch) for ch in info["streams"]]
    s = bytearray(streams[c][i])
    s[len(s) // 2] ^= 0x10
    streams[c][i] = bytes(s)
    g = tl.join_file(100, 70, 32, streams)
    try:
        out = oracle.decode(g)
    except oracle.OracleError as e:
        assert e.code == oracle.ERR_CORRUPT
    else:
        x0, y0, pw, ph = tl.patch_rect(info, i)
        diff = out != img
        assert diff.any()
        diff[y0:y0 + ph, x0:x0 + pw, c] = False
        assert not diff.any()
    # (c) changing one patch's pixels leaves every other patch's bytes identical
    img2 = img.copy()
    x0, y0, pw, ph = tl.patch_rect(info, 6)
    img2[y0:y0 + ph, x0:x0 + pw, 2] ^= 0x5A
    info2 = tl.split_file(oracle.encode(img2, patch=32))
    for c in range(3):
        for i in range(len(info["streams"][c])):
            same = info["streams"][c][i] == info2["streams"][c][i]
            assert same == (not (c == 2 and i == 6))


def test_non_canonical_streams_decode_identically():
    """Any width >= minimal is a valid stream (the decoder's output is unique, the
    encoder's is not)."""
    for img in (synth.cosine_field(31, 77, 50), synth.voronoi_scene(32, 130, 70)):
        f0 = oracle.encode(img, patch=32, width_mode=0)
        f8 = oracle.encode(img, patch=32, width_mode=1)
        f1 = oracle.encode(img, patch=32, width_mode=2)
        assert len(f8) > len(f1) > len(f0)
        for f in (f0, f8, f1):
            assert np.array_equal(oracle.decode(f), img)
    # a hand-packed stream with a non-minimal base window
    rows = [(8, 0, [10, 20, 30, 40]), (3, 0xFE, [2, 3, 4, 2])]   # residuals 0, +1, +2, 0
    s = tl.pack_rows(rows)
    out = oracle.decode_patch(s, 4, 2)
    # row 1: borders add to the pixel above; interior triples (10,20,30), (20,30,40) are
    # symmetric around the top pixel, which is therefore selected
    assert out.tolist() == [[10, 20, 30, 40], [10, 21, 32, 40]]
    assert np.array_equal(out, tl.py_decode_patch(s, 4, 2))


# ---------------------------------------------------------------------------
# error paths

def test_corrupt_inputs_are_rejected():
    img = synth.cosine_field(41, 40, 40)
    f = bytearray(oracle.encode(img, patch=32))
    with pytest.raises(oracle.OracleError) as e:
        oracle.decode(bytes(f[:12]))
    assert e.value.code == oracle.ERR_TRUNCATED
    with pytest.raises(oracle.OracleError) as e:
        oracle.decode(bytes(f[:40]))
    assert e.value.code == oracle.ERR_TRUNCATED
    bad = bytearray(f)
    bad[0] = 0x4D
    with pytest.raises(oracle.OracleError) as e:
        oracle.decode(bytes(bad))
    assert e.value.code == oracle.ERR_MAGIC
    bad = bytearray(f)
    bad[12] = 0
    with pytest.raises(oracle.OracleError) as e:
        oracle.decode(bytes(bad))
    assert e.value.code == oracle.ERR_CORRUPT
    # a width field of 9..15
    info = tl.split_file(bytes(f))
    bad = bytearray(f)
    pos = info["header_bytes"]
    bad[pos] = (bad[pos] & 0xF0) | 0x0B
    with pytest.raises(oracle.OracleError) as e:
        oracle.decode(bytes(bad))
    assert e.value.code == oracle.ERR_CORRUPT
    # data cut short: the last patch overruns
    with pytest.raises(oracle.OracleError) as e:
        oracle.decode(bytes(f[:-3]))
    assert e.value.code == oracle.ERR_CORRUPT
    # an offset beyond the data section
    bad = bytearray(f)
    struct.pack_into("<I", bad, 13 + 4, 0x7FFFFFFF)
    with pytest.raises(oracle.OracleError) as e:
        oracle.decode(bytes(bad))
    assert e.value.code == oracle.ERR_CORRUPT


# ---------------------------------------------------------------------------
# the 16-bit float epilogue (defined by the benchmark configuration, not the paper)

def test_float_rounding_against_library():
    torch = pytest.importorskip("torch")
    s = synth.Stream(55)
    vals = np.concatenate([s.normal(20000) * 3.0, s.normal(2000) * 1e-6, s.normal(2000) * 7e4,
                           np.array([0.0, -0.0, 1.0, 65504.0, 65520.0, 1e-8, 6e-8, 6.1e-5,
                                     2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25, np.inf, -np.inf])])
    vals = vals.astype(np.float32)
    # ties: values exactly halfway between two bfloat16 / binary16 neighbours
    ties = (np.arange(0x3F800000, 0x3F800000 + 64 * 0x8000, 0x8000, dtype=np.uint32)
            .view(np.float32))
    ties16 = (np.arange(0x3F800000, 0x3F800000 + 64 * 0x1000, 0x1000, dtype=np.uint32)
              .view(np.float32))
    vals = np.concatenate([vals, ties, ties16])
    t = torch.from_numpy(vals)
    bf = t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    hf = t.to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    for v, b, h in zip(vals.tolist(), bf.tolist(), hf.tolist()):
        assert oracle.f32_to_bf16(v) == b, v
        assert oracle.f32_to_f16(v) == h, v


def test_crop_normalize_against_library():
    torch = pytest.importorskip("torch")
    img = synth.cosine_field(61, 300, 260)
    mean, std = synth.IMAGENET_MEAN, synth.IMAGENET_STD
    for x0, y0, flip, dtype in ((0, 0, 0, 0), (76, 36, 1, 0), (13, 5, 1, 1), (76, 36, 0, 1)):
        got = oracle.crop_normalize(img, x0, y0, flip, 224, 224, mean, std, dtype)
        win = torch.from_numpy(img[y0:y0 + 224, x0:x0 + 224].copy())
        if flip:
            win = win.flip(1)
        x = win.permute(2, 0, 1).to(torch.float32) / 255.0
        m = torch.tensor(mean, dtype=torch.float32)[:, None, None]
        s = torch.tensor(std, dtype=torch.float32)[:, None, None]
        y = ((x - m) / s).to(torch.bfloat16 if dtype == 0 else torch.float16)
        want = y.view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(got, want)
