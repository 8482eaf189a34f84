"""Writes tests/golden/compratio_report.md: the two synthetic columns (Random, Black) of the
paper's Table "compratio" (arxiv 2208.08711 Section 5.2) reproduced with the oracle encoder, for
every patch size, beside the closed forms.  Calls only oracle/ and paper_2208_08711_amd.synth
(the seeded input generator, which holds no codec arithmetic).

    python tests/golden/make_compratio_report.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2208_08711_amd import synth  # noqa: E402

W, H = 1920, 1080
RAW = W * H * 3


def closed_form(n, bits_per_pixel, floor_bits=0):
    """File size when every row of every patch has the same delta width."""
    px, py = -(-W // n), -(-H // n)
    total = 13 + 12 * px * py
    for j in range(py):
        ph = min(n, H - j * n)
        for i in range(px):
            pw = min(n, W - i * n)
            total += 3 * -(-(ph * (12 + pw * max(bits_per_pixel, floor_bits))) // 8)
    return total


def main():
    random_image = synth.uniform_bytes(424242, W, H)
    black = np.zeros((H, W, 3), np.uint8)
    lines = ["# Random and Black columns of the paper's Table \"compratio\" (Section 5.2)", "",
             "Raw size %d bytes (1920 x 1080 x 3, the paper's 5.93 MB).  The paper prints ratios only:" % RAW,
             "Random 1.02, Black 0.13.  Sizes below are what the oracle encoder writes "
             "(`oracle.encode`), beside the", "closed form for a constant delta width "
             "(13-byte header + 12 bytes of offsets per patch + per patch",
             "ceil(rows x (12 + width x bits) / 8) bytes).", "",
             "| content | N | oracle file (bytes) | closed form | compressed / raw | paper |",
             "|---|---|---|---|---|---|"]
    for name, im, bits, paper in (("Random (uniform bytes, seed 424242)", random_image, 8, "1.02"),
                                  ("Black (all zero)", black, 0, "0.13")):
        for n in (32, 64, 128):
            f = oracle.encode(im, n)
            assert np.array_equal(oracle.decode(f), im)
            rule = " (the rule's N for FHD)" if n == 64 else ""
            lines.append("| %s | %d%s | %d | %d | %.4f | %s |" % (name, n, rule, len(f), closed_form(n, bits),
                                                                  len(f) / RAW, paper if n == 64 else ""))
    lines += ["",
              "Random: with N = 64, the patch size the rule of Section 4.3 gives an FHD image, the ratio is",
              "1.0244, which prints as the paper's 1.02; N = 32 would print 1.05 and N = 128 1.01, and padding",
              "every row to a byte would give 1.03.  The column therefore confirms the 12-bit row record",
              "(4-bit width + 8-bit base), rows packed without padding, and N = 64 for FHD.",
              "",
              "Black: with zero-width rows (the literal \"minimum number of bits\", 12 bits per row) the ratio is",
              "%.4f; with a floor of one bit per delta it would be %.4f (closed form, N = 64).  The paper prints"
              % (closed_form(64, 0) / RAW, closed_form(64, 0, 1) / RAW),
              "0.13, which neither reading gives (0.13 would need about 1.04 bytes per 8 pixels).  Open",
              "discrepancy: the format reading keeps zero-width rows; nothing is pinned to the Black column.", ""]
    with open(os.path.join(HERE, "compratio_report.md"), "w") as fh:
        fh.write("\n".join(lines))
    print("\n".join(lines))


if __name__ == "__main__":
    main()
