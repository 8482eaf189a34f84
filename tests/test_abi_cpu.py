"""CPU-side checks of the C ABI: the library loads, exports every symbol that
include/l3.h declares, and its host-only entry points (encoder, header parser)
agree with the oracle.  No GPU compute call is made here."""
import ctypes
import os
import re
import struct

import numpy as np
import pytest

import oracle
import paper_2208_08711_amd as l3
from paper_2208_08711_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = "".join(open(os.path.join(ROOT, "include", name)).read()
                   for name in sorted(os.listdir(os.path.join(ROOT, "include"))) if name.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(l3_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    assert os.path.exists(l3.library_path()), "build the library first"
    lib = ctypes.CDLL(l3.library_path())
    names = declared_symbols()
    assert set(names) == set(l3.EXPORTED_SYMBOLS)
    for name in names:
        assert hasattr(lib, name), name


def test_status_strings():
    seen = {l3.status_string(k) for k in range(9)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert l3.status_string(99) == "unknown status"


def test_default_patch_matches_section_4_3():
    for w, h in ((500, 375), (1079, 720), (1080, 720), (1920, 1080), (1921, 1080), (2048, 1024),
                 (3840, 2160)):
        assert l3.default_patch(w, h) == oracle.patch_rule(w, h)


def test_product_encoder_matches_oracle_bytes():
    """l3_encode_cpu is separate code from the oracle; both must produce the same file."""
    images = synth.config1() + synth.config2(2) + [
        synth.voronoi_scene(3, 300, 200), synth.uniform_bytes(4, 129, 70),
        np.zeros((40, 40, 3), np.uint8), synth.gradient_noise(5, 1, 9, 2.0),
        synth.gradient_noise(6, 9, 1, 2.0)]
    for im in images:
        for patch in (0, 1, 7, 32, 64, 128, 255):
            if patch in (1, 7) and im.size > 30000:
                continue
            a = l3.encode_cpu(im, patch)
            assert a == oracle.encode(im, patch), (im.shape, patch)
            assert len(a) <= l3.encode_bound(im.shape[1], im.shape[0], patch)
            info = l3.peek_header(a)
            n = patch or oracle.patch_rule(im.shape[1], im.shape[0])
            assert (info.width, info.height, info.patch) == (im.shape[1], im.shape[0], n)
            assert info.header_bytes == 13 + 12 * info.patches_per_channel


def test_product_encoder_original_filter_matches_oracle_bytes():
    """The ablation baseline's encoder (original Paeth filter, Section 5.5) against the oracle."""
    images = synth.config1() + [synth.voronoi_scene(3, 300, 200), synth.uniform_bytes(4, 129, 70),
                                synth.gradient_noise(5, 1, 9, 2.0), synth.gradient_noise(6, 9, 1, 2.0)]
    for im in images:
        for patch in (0, 7, 32, 128):
            if patch == 7 and im.size > 30000:
                continue
            a = l3.encode_cpu(im, patch, original_filter=True)
            assert a == oracle.encode(im, patch, predictor=oracle.PREDICTOR_ORIGINAL), (im.shape, patch)
            assert len(a) <= l3.encode_bound(im.shape[1], im.shape[0], patch)


def test_normalized_values_match_the_oracle_and_torch():
    """l3_normalized_values (what the fused kernels look pixels up in) against the oracle's
    epilogue on a 1 x 256 image holding every byte value, and against PyTorch CPU ops; the
    constants reach binary16 subnormals, ties, overflow to infinity and negative values."""
    import torch
    ramp = np.arange(256, dtype=np.uint8)[None, :, None].repeat(3, 2)
    cases = [(synth.IMAGENET_MEAN, synth.IMAGENET_STD), ((0.0, 0.5, 1.0), (1.0, 0.25, 4.0)),
             ((0.5, 0.5, 0.5), (1e-5, 7e-6, 1.5e-5)),            # binary16 overflows to infinity
             ((0.0, 0.0, 0.0), (16777216.0, 65536.0 * 3, 5e7)),  # binary16 subnormals and zero
             ((0.3, 0.7, 0.1), (-0.2, 1e3, 1024.0)), ((1e-3, 2.0, -1.0), (3.0, 0.1, 1e-2))]
    rng = np.random.default_rng(5)
    for _ in range(40):
        cases.append((tuple(rng.uniform(-1, 2, 3)), tuple(10.0 ** rng.uniform(-6, 8, 3))))
    for mean, stdv in cases:
        for dtype, tdt in ((l3.BF16, torch.bfloat16), (l3.FP16, torch.float16)):
            got = l3.normalized_values(mean, stdv, dtype)
            want = oracle.crop_normalize(ramp, 0, 0, False, 256, 1, mean, stdv, dtype)[:, 0, :]
            assert np.array_equal(got, want), (mean, stdv, dtype)
            v = torch.arange(256, dtype=torch.float32)
            for c in range(3):
                y = (v / 255.0 - torch.tensor(mean[c], dtype=torch.float32)) / torch.tensor(stdv[c], dtype=torch.float32)
                ref = y.to(tdt).view(torch.int16).numpy().view(np.uint16)
                assert np.array_equal(got[c], ref), (mean, stdv, dtype, c)
    m = (ctypes.c_float * 3)(0, 0, 0)
    out = (ctypes.c_uint16 * 768)()
    lib = ctypes.CDLL(l3.library_path())
    assert lib.l3_normalized_values(m, m, 2, out) == 1 and lib.l3_normalized_values(None, m, 0, out) == 1


def test_encode_cpu_errors():
    lib = ctypes.CDLL(l3.library_path())
    lib.l3_encode_cpu.restype = ctypes.c_int
    img = np.zeros((4, 4, 3), np.uint8)
    out = np.zeros(16, np.uint8)
    n = ctypes.c_size_t()
    u8p = ctypes.POINTER(ctypes.c_uint8)
    args = lambda cap, stride=12, w=4: (img.ctypes.data_as(u8p), ctypes.c_uint32(w),
                                        ctypes.c_uint32(4), ctypes.c_size_t(stride),
                                        ctypes.c_uint8(0), out.ctypes.data_as(u8p),
                                        ctypes.c_size_t(cap), ctypes.byref(n))
    assert lib.l3_encode_cpu(*args(16)) == 5          # buffer too small
    assert lib.l3_encode_cpu(*args(16, stride=11)) == 1
    assert lib.l3_encode_cpu(*args(16, w=0)) == 1
    assert l3.encode_bound(0, 5) == 0


def test_peek_header_rejects_bad_files():
    f = bytearray(oracle.encode(synth.cosine_field(7, 100, 70), 32))
    p = 4 * 3

    def code(buf):
        with pytest.raises(l3.L3Error) as e:
            l3.peek_header(bytes(buf))
        return e.value.code

    assert code(f[:12]) == 3
    assert code(f[:13 + 12 * p - 1]) == 3
    g = bytearray(f); g[1] = 0x34
    assert code(g) == 2
    for pos in (4, 8):
        g = bytearray(f); g[pos:pos + 4] = b"\0\0\0\0"
        assert code(g) == 4
    g = bytearray(f); g[12] = 0
    assert code(g) == 4
    g = bytearray(f); struct.pack_into("<I", g, 13, 1)            # first offset not 0
    assert code(g) == 4
    g = bytearray(f); struct.pack_into("<I", g, 13 + 8, struct.unpack_from("<I", f, 13 + 4)[0])
    assert code(g) == 4                                           # not strictly increasing
    g = bytearray(f); struct.pack_into("<I", g, 13 + 4 * (3 * p - 1), 0x7FFFFFF0)
    assert code(g) == 4                                           # beyond the data section
    assert code(f[:13 + 12 * p + struct.unpack_from("<I", f, 13 + 4 * (3 * p - 1))[0] + 2]) == 4
    assert l3.peek_header(bytes(f)).patches_per_channel == p


def test_context_needs_a_gpu_and_says_so():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(l3.L3Error) as e:
        l3.Context(0)
    assert e.value.code == 7


def test_header_is_plain_c99(tmp_path):
    """include/l3.h and include/l3_ablation.h compile as C99 with every warning on (no GPU, no
    HIP header needed): the ABI has no C++ in it."""
    import subprocess
    src = tmp_path / "use_headers.c"
    src.write_text('#include "l3.h"\n#include "l3_ablation.h"\n'
                   'int use(void) { l3_info i; l3_item it; l3_crop c; l3_encode_item e;\n'
                   '  (void)i; (void)it; (void)c; (void)e; return (int)L3_ERR_DEVICE + (int)L3_LAYOUT_CHW + '
                   '(int)L3_FP16 + L3_ABLATION_DIAGONAL; }\n')
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                    "-I", os.path.join(ROOT, "include"), str(src)], check=True)
