"""Do the oracle's pins have teeth?

Each case below plants one plausible mistake in a *copy* of the oracle's source (a
wrong sign, a swapped operand, a changed tie order, another bit order, a dropped
term ...), builds that copy with the oracle's own compiler flags and runs the pin
tests of tests/test_oracle_pins.py and tests/test_oracle_original_paeth.py against
it in a child process.  The pins must fail for every planted mistake: a mistake that
survives them would mean that the oracle could be wrong in that way unnoticed.
Many of the mistakes are self-consistent (encoder and decoder changed together), so
that a round trip alone cannot see them.

Everything here runs on the CPU; nothing of the product is involved.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "l3_oracle.cpp")
PIN_FILES = [os.path.join(HERE, "test_oracle_pins.py"),
             os.path.join(HERE, "test_oracle_original_paeth.py")]

# name -> list of (text in the oracle, replacement, how often the text occurs)
#
# Not in the list, because they change nothing: the order in which a tie between
# top-left and top-right is broken, and exchanging those two operands.  Their
# distances to the reference value TL + TR - T are |TR - T| and |TL - T|; these are
# equal only if TL = TR (same value either way) or if TL and TR lie symmetrically
# about T, and then the reference value is T itself and T wins.  The same holds for
# left and top in the original filter.
MISTAKES = {
    # Section 4.2, the predictor
    "reference value with T and TR exchanged":
        [("int ref = tl + tr - t;", "int ref = tl + t - tr;", 1)],
    "tie between top-left and top goes to top":
        [("if (d_tl <= d_tr && d_tl <= d_t) return tl;", "if (d_tl <= d_tr && d_tl < d_t) return tl;", 1)],
    "tie between top-right and top goes to top":
        [("if (d_tr <= d_t) return tr;", "if (d_tr < d_t) return tr;", 1)],
    "border columns predict 0 instead of the pixel above":
        [("if (x == 0 || x + 1 >= pw) return above[x];", "if (x == 0 || x + 1 >= pw) return 0;", 1)],
    "residual is prediction minus pixel":
        [("resid[x] = (uint8_t)(cur[x] - predict_at(above.data(), x, pw));",
          "resid[x] = (uint8_t)(predict_at(above.data(), x, pw) - cur[x]);", 1),
         ("out[r * ostride + x] = (uint8_t)(pred + resid[r * rstride + x]);",
          "out[r * ostride + x] = (uint8_t)(pred - resid[r * rstride + x]);", 1)],
    # Section 4.2, base-delta
    "residuals of every row taken as unsigned":
        [("int v = (r == 0) ? (int)resid[x] : (int)(int8_t)resid[x];", "int v = (int)resid[x];", 2)],
    "a constant row still gets 1 bit per delta":
        [("unsigned width = bit_length((unsigned)(hi - lo));",
          "unsigned width = bit_length((unsigned)(hi - lo) >> 1) + 1;", 1)],
    "base before width in the row record":
        [("bw.put(width, 4);\n        bw.put((uint32_t)lo & 0xFFu, 8);",
          "bw.put((uint32_t)lo & 0xFFu, 8);\n        bw.put(width, 4);", 1),
         ("uint32_t width = br.get(4);\n        uint32_t base = br.get(8);",
          "uint32_t base = br.get(8);\n        uint32_t width = br.get(4);", 1)],
    "bits fill a byte from its most significant end":
        [("bytes[nbits >> 3] |= (uint8_t)(1u << (nbits & 7));",
          "bytes[nbits >> 3] |= (uint8_t)(0x80u >> (nbits & 7));", 1),
         ("uint32_t bit = (bytes[pos >> 3] >> (pos & 7)) & 1u;",
          "uint32_t bit = (bytes[pos >> 3] >> (7 - (pos & 7))) & 1u;", 1)],
    "a field's most significant bit goes first":
        [("if ((value >> i) & 1u)", "if ((value >> (width - 1 - i)) & 1u)", 1),
         ("v |= bit << i;", "v |= bit << (width - 1 - i);", 1)],
    "delta is stored without subtracting the base":
        [("bw.put((uint32_t)(v - lo), width);", "bw.put((uint32_t)v, width);", 1),
         ("resid[r * stride + x] = (uint8_t)(base + delta);", "resid[r * stride + x] = (uint8_t)(delta);", 1)],
    # Section 4.3, the file
    "header integers big-endian":
        [("return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) |\n           ((uint32_t)p[3] << 24);",
          "return (uint32_t)p[3] | ((uint32_t)p[2] << 8) | ((uint32_t)p[1] << 16) |\n           ((uint32_t)p[0] << 24);", 1),
         ("p[0] = (uint8_t)v;\n    p[1] = (uint8_t)(v >> 8);\n    p[2] = (uint8_t)(v >> 16);\n    p[3] = (uint8_t)(v >> 24);",
          "p[3] = (uint8_t)v;\n    p[2] = (uint8_t)(v >> 8);\n    p[1] = (uint8_t)(v >> 16);\n    p[0] = (uint8_t)(v >> 24);", 1)],
    "offsets interleaved by channel instead of one array per channel":
        [("uint64_t flat = (uint64_t)c * patches + (uint64_t)ty * px + tx;",
          "uint64_t flat = ((uint64_t)ty * px + tx) * 3 + c;", 1),
         ("uint64_t flat = (uint64_t)c * patches + (uint64_t)py * info.px + px;",
          "uint64_t flat = ((uint64_t)py * info.px + px) * 3 + c;", 1)],
    "patch size rule: 1080x720 still gets 32":
        [("if (pixels < (uint64_t)1080 * 720) return 32;", "if (pixels <= (uint64_t)1080 * 720) return 32;", 1)],
    "patch size rule: 1920x1080 already gets 128":
        [("if (pixels <= (uint64_t)1920 * 1080) return 64;", "if (pixels < (uint64_t)1920 * 1080) return 64;", 1)],
    # the original Paeth filter of the ablation baseline
    "original filter: reference value with the wrong sign":
        [("int ref = left + top - top_left;", "int ref = left - top + top_left;", 1)],
    # the fused epilogue
    "bf16 rounds halves up":
        [("if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) ++upper;",
          "if (lower >= 0x8000u) ++upper;", 1)],
    "fp16 rounds halves up":
        [("if (rest > half || (rest == half && (kept & 1))) ++h;", "if (rest >= half) ++h;", 1)],
    "pixels scaled by 1/256":
        [("(float)v / 255.0f", "(float)v / 256.0f", 1)],
    "multiplied by the standard deviation":
        [("float y = centred / stdv[c];", "float y = centred * stdv[c];", 1)],
    "mirror flag inverted":
        [("uint32_t sx = flip ? (uint32_t)x0 + crop_w - 1 - j : (uint32_t)x0 + j;",
          "uint32_t sx = flip ? (uint32_t)x0 + j : (uint32_t)x0 + crop_w - 1 - j;", 1)],
}

DRIVER = """
import sys
sys.path.insert(0, {root!r})
sys.path.insert(0, {tests!r})
import oracle.build as b
b.OUT = {lib!r}          # the binding loads whatever this names
b.build = None           # and must not build over it
import pytest
sys.exit(pytest.main(["-x", "-q", "-p", "no:cacheprovider", "--no-header"] + {args!r}))
"""


def _plant(name, workdir):
    text = open(SRC).read()
    for old, new, count in MISTAKES[name]:
        assert text.count(old) == count, f"{name}: the oracle's text changed, update this case"
        text = text.replace(old, new)
    d = os.path.join(workdir, "m%02d" % list(MISTAKES).index(name))
    os.makedirs(d)
    src = os.path.join(d, "l3_oracle.cpp")
    open(src, "w").write(text)
    lib = os.path.join(d, "libl3_oracle.so")
    subprocess.run(["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared",
                    "-I", os.path.join(ROOT, "oracle"), "-o", lib, src], check=True)
    return lib


BRUTE = "test_brute_force_tiny_images"     # the slow pin: only for what the quick ones let through


def _pins_pass(lib, brute=False):
    args = PIN_FILES + ["-k", BRUTE if brute else "not " + BRUTE]
    code = DRIVER.format(root=ROOT, tests=HERE, lib=lib, args=args)
    env = dict(os.environ, OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-c", code], stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True, env=env, cwd=ROOT)
    return r.returncode == 0, r.stdout[-1500:]


def test_unchanged_copy_passes(tmp_path):
    """The harness itself: a copy with nothing planted passes every pin."""
    MISTAKES["(nothing)"] = []
    try:
        lib = _plant("(nothing)", str(tmp_path))
    finally:
        del MISTAKES["(nothing)"]
    ok, tail = _pins_pass(lib)
    assert ok, tail


def test_every_planted_mistake_fails_a_pin(tmp_path):
    names = list(MISTAKES)
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        libs = list(pool.map(lambda n: _plant(n, str(tmp_path)), names))
        results = list(pool.map(_pins_pass, libs))
        slow = [k for k, (ok, _) in enumerate(results) if ok]
        for k, res in zip(slow, pool.map(lambda k: _pins_pass(libs[k], True), slow)):
            results[k] = res
    survivors = [n for n, (ok, _) in zip(names, results) if ok]
    print("caught only by the brute-force pin:", [names[k] for k in slow])
    assert not survivors, f"no pin notices: {survivors}"
    # a failing run must have failed in a test, not in collection or start-up
    for n, (ok, tail) in zip(names, results):
        assert " failed" in tail, (n, tail)
