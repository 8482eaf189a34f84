"""Device-side paths that ordinary parity inputs do not reach: patch offsets that only the
kernel sees as damaged, damaged streams for every patch size and output mode, and a batch
built so that every one of the 2^24 (top-left, top, top-right) triples goes through the
kernel's predictor (arxiv 2208.08711 Section 4.2).  All inputs are fixed."""
import numpy as np
import pytest

import oracle
from paper_2208_08711_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from test_gpu_parity import l3, ctx, upload_files  # noqa: E402,F401  (fixtures and helper)

POISON = 0xCD


def _decode(l3, ctx, dfiles, infos, layout, pad=5):
    outs = []
    for inf in infos:
        w, h = inf.width, inf.height
        shape = (h, 3 * w + pad) if layout == "hwc" else (3, h, w + pad)
        outs.append(torch.full(shape, POISON, dtype=torch.uint8, device="cuda"))
    strides = [(3 * inf.width if layout == "hwc" else inf.width) + pad for inf in infos]
    status = torch.full((len(infos),), 0x55, dtype=torch.int32, device="cuda")
    l3.decode_batch(ctx, dfiles, infos, outs, l3.LAYOUT_HWC if layout == "hwc" else l3.LAYOUT_CHW,
                    status=status, row_strides=strides)
    torch.cuda.synchronize()
    res = []
    for t, inf in zip(outs, infos):
        a = t.cpu().numpy()
        w = inf.width
        if layout == "hwc":
            assert (a[:, 3 * w:] == POISON).all(), "wrote outside the image rows"
            res.append(a[:, :3 * w].reshape(inf.height, w, 3))
        else:
            assert (a[:, :, w:] == POISON).all(), "wrote outside the image rows"
            res.append(a[:, :, :w].transpose(1, 2, 0))
    return res, status.cpu().numpy()


@pytest.mark.parametrize("patch", [32, 64, 128])
@pytest.mark.parametrize("layout", ["hwc", "chw"])
def test_offsets_damaged_after_the_host_check(l3, ctx, patch, layout):
    """The host validates its own copy of a file; the kernel reads the offset arrays from
    device memory.  Here the device copy differs: one offset far beyond the data section, one
    pair in decreasing order.  The kernel must flag the image (bit 2), keep every access
    inside the file and the image's rows, and leave the neighbours of the batch intact."""
    images = [synth.cosine_field(8100 + k, 300, 200) for k in range(4)]
    files = [oracle.encode(im, patch) for im in images]
    infos = [l3.peek_header(f) for f in files]          # from the undamaged bytes
    bad = [bytearray(f) for f in files]
    p = infos[1].patches_per_channel
    k = min(3, 3 * p - 2)
    bad[1][13 + 4 * k:13 + 4 * k + 4] = (0xFFFFFFF0).to_bytes(4, "little")      # beyond the data
    k2 = 3 * p - 2
    a = int.from_bytes(bad[3][13 + 4 * k2:13 + 4 * k2 + 4], "little")
    bad[3][13 + 4 * (k2 + 1):13 + 4 * (k2 + 1) + 4] = (a - 1).to_bytes(4, "little")  # end before start
    dfiles, keep = upload_files([bytes(b) for b in bad])
    got, status = _decode(l3, ctx, dfiles, infos, layout)
    assert status[0] == 0 and status[2] == 0
    assert status[1] & 4 and status[3] & 4
    assert np.array_equal(got[0], images[0]) and np.array_equal(got[2], images[2])


@pytest.mark.parametrize("patch", [32, 64, 128])
@pytest.mark.parametrize("layout", ["hwc", "chw"])
def test_damaged_streams_every_patch_size_and_layout(l3, ctx, patch, layout):
    """A width field above 8 (bit 0) and a stream cut short (bit 1), for every patch size, in
    the interleaved layout and in the planar one (which for N = 128 writes rows directly)."""
    images = [synth.cosine_field(8200 + k, 280, 150) for k in range(4)]
    files = [bytearray(oracle.encode(im, patch)) for im in images]
    info = l3.peek_header(bytes(files[0]))
    hdr = info.header_bytes
    files[1][hdr] = (files[1][hdr] & 0xF0) | 0x0B            # width 11 in the first row record
    files[3] = files[3][:-(patch // 2 + 9)]                   # the last patch loses its tail
    files = [bytes(f) for f in files]
    infos = [l3.peek_header(f) for f in files]                # both still pass the host check
    dfiles, keep = upload_files(files)
    got, status = _decode(l3, ctx, dfiles, infos, layout)
    assert status[0] == 0 and status[2] == 0
    assert status[1] & 1
    assert status[3] & 2
    assert np.array_equal(got[0], images[0]) and np.array_equal(got[2], images[2])
    diff = got[1] != images[1]
    diff[0:patch, 0:patch, 0] = False                         # damage stays inside its patch
    assert not diff.any()
    ph, pw = 150 - (150 - 1) // patch * patch, 280 - (280 - 1) // patch * patch
    diff = got[3] != images[3]
    diff[150 - ph:, 280 - pw:, 2] = False                     # the last patch of the last channel
    assert not diff.any()


@pytest.mark.parametrize("patch", [32, 64, 128])
def test_damaged_streams_fused_path(l3, ctx, patch):
    """The same two kinds of damage through the crop / mirror / normalise call: status words
    set, the clean images of the batch bit-exact, nothing written outside the tensor."""
    images = [synth.cosine_field(8300 + k, 280, 250) for k in range(4)]
    files = [bytearray(oracle.encode(im, patch)) for im in images]
    hdr = l3.peek_header(bytes(files[0])).header_bytes
    files[1][hdr] = (files[1][hdr] & 0xF0) | 0x0E
    files[3] = files[3][:-(patch // 2 + 9)]
    files = [bytes(f) for f in files]
    infos = [l3.peek_header(f) for f in files]
    dfiles, keep = upload_files(files)
    crops = [(0, 0, 0), (0, 0, 1), (30, 20, 1), (280 - 224, 250 - 224, 0)]
    raw = torch.full((4 * 3 * 224 * 224 + 64,), -1, dtype=torch.int16, device="cuda")
    out = raw[32:32 + 4 * 3 * 224 * 224].view(4, 3, 224, 224)
    status = torch.full((4,), 0x55, dtype=torch.int32, device="cuda")
    l3.decode_crop_normalize_batch(ctx, dfiles, infos, crops, 224, 224, synth.IMAGENET_MEAN,
                                   synth.IMAGENET_STD, out, status=status)
    torch.cuda.synchronize()
    st = status.cpu().numpy()
    assert st[0] == 0 and st[2] == 0 and st[1] & 1 and st[3] & 2
    r = raw.cpu().numpy()
    assert (r[:32] == -1).all() and (r[-32:] == -1).all()
    got = out.cpu().numpy().view(np.uint16)
    for i in (0, 2):
        x0, y0, flip = crops[i]
        want = oracle.crop_normalize(images[i], x0, y0, flip, 224, 224, synth.IMAGENET_MEAN,
                                     synth.IMAGENET_STD, 0)
        assert np.array_equal(got[i], want)


def test_every_neighbour_triple_through_the_kernel(l3, ctx):
    """All 2^24 combinations of (top-left, top, top-right) as the row above an interior pixel.
    Even rows carry the triples, 42 per 128-pixel patch row, centred on interior columns; odd
    rows are random bytes predicted from them.  numpy first confirms that the rows above the
    odd rows' interior pixels cover all 2^24 triples; then every byte must decode."""
    width, n = 4096, 128
    per_row = (width // n) * 42                              # triples per image row and channel
    rows = -(-(1 << 24) // (3 * per_row))                    # designed rows (three channels share the work)
    height = 2 * rows
    t = np.arange(3 * rows * per_row, dtype=np.int64) % (1 << 24)
    tri = np.stack([(t >> 16) & 255, (t >> 8) & 255, t & 255], axis=1).astype(np.uint8)
    tri = tri.reshape(3, rows, width // n, 42 * 3)           # [channel][row][patch][126 pixels]
    designed = np.zeros((3, rows, width // n, n), np.uint8)
    designed[..., :126] = tri
    designed[..., 126:] = 77
    im = np.empty((height, width, 3), np.uint8)
    im[0::2] = designed.reshape(3, rows, width).transpose(1, 2, 0)
    im[1::2] = synth.uniform_bytes(8400, width, rows)
    # coverage, from the image itself: the row above every interior pixel of the odd rows
    seen = np.zeros(1 << 24, dtype=bool)
    above = im[0::2].astype(np.int64)
    interior = np.ones(width, dtype=bool)
    interior[0::n] = False
    interior[n - 1::n] = False
    xs = np.nonzero(interior)[0]
    for c in range(3):
        a = above[:, :, c]
        seen[((a[:, xs - 1] << 16) | (a[:, xs] << 8) | a[:, xs + 1]).ravel()] = True
    assert seen.all(), "the designed rows do not cover every triple"
    f = oracle.encode(im, n)
    info = l3.peek_header(f)
    dfiles, keep = upload_files([f])
    out = torch.zeros((height, 3 * width), dtype=torch.uint8, device="cuda")
    status = torch.ones(1, dtype=torch.int32, device="cuda")
    l3.decode_batch(ctx, dfiles, [info], [out], status=status)
    torch.cuda.synchronize()
    assert int(status[0]) == 0
    assert np.array_equal(out.cpu().numpy().reshape(im.shape), im)
