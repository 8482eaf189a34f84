"""GPU parity: the HIP decoder, called through the C ABI, against the CPU oracle,
byte for byte, on the same seeded inputs (arxiv 2208.08711 Sections 4.2-4.4)."""
import numpy as np
import pytest

import oracle
from paper_2208_08711_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def l3():
    import paper_2208_08711_amd as mod
    assert torch.cuda.is_available(), "these tests need the GPU"
    return mod


@pytest.fixture(scope="module")
def ctx(l3):
    c = l3.Context(0)
    yield c
    c.close()


def upload_files(files, misalign=True):
    """All files in one device buffer, each at a deliberately odd offset."""
    offs, pos = [], 0
    for k, f in enumerate(files):
        pos = (pos + 63) // 64 * 64 + ((1 + 3 * k) % 16 if misalign else 0)
        offs.append(pos)
        pos += len(f)
    host = np.zeros(pos + 64, dtype=np.uint8)
    for o, f in zip(offs, files):
        host[o:o + len(f)] = np.frombuffer(f, dtype=np.uint8)
    dev = torch.from_numpy(host).cuda()
    return [dev[o:o + len(f)] for o, f in zip(offs, files)], dev


def gpu_decode(l3, ctx, files, layout="hwc", poison=0xCD, pad_cols=0):
    infos = [l3.peek_header(f) for f in files]
    dfiles, keep = upload_files(files)
    outs, strides = [], []
    for inf in infos:
        w, h = inf.width, inf.height
        if layout == "hwc":
            t = torch.full((h, 3 * w + pad_cols), poison, dtype=torch.uint8, device="cuda")
            strides.append(3 * w + pad_cols)
        else:
            t = torch.full((3, h, w + pad_cols), poison, dtype=torch.uint8, device="cuda")
            strides.append(w + pad_cols)
        outs.append(t)
    status = torch.full((len(files),), 0x55, dtype=torch.int32, device="cuda")
    l3.decode_batch(ctx, dfiles, infos, outs, l3.LAYOUT_HWC if layout == "hwc" else l3.LAYOUT_CHW,
                    status=status, row_strides=strides)
    torch.cuda.synchronize()
    res = []
    for t, inf in zip(outs, infos):
        a = t.cpu().numpy()
        w, h = inf.width, inf.height
        if layout == "hwc":
            if pad_cols:
                assert (a[:, 3 * w:] == poison).all(), "wrote outside the image rows"
            res.append(a[:, :3 * w].reshape(h, w, 3))
        else:
            if pad_cols:
                assert (a[:, :, w:] == poison).all(), "wrote outside the image rows"
            res.append(a[:, :, :w].transpose(1, 2, 0))
    return res, status.cpu().numpy()


def check_batch(l3, ctx, images, patch=0, layout="hwc", width_mode=0, pad_cols=0):
    files = [oracle.encode(im, patch, width_mode) for im in images]
    got, status = gpu_decode(l3, ctx, files, layout, pad_cols=pad_cols)
    for k, (g, f, im) in enumerate(zip(got, files, images)):
        want = oracle.decode(f)
        assert np.array_equal(want, im)
        bad = np.argwhere(g != want)
        assert bad.size == 0, (k, im.shape, patch, layout, bad[:5], len(bad))
    assert (status == 0).all(), status


# ---------------------------------------------------------------------------

def test_config1_single_64x64(l3, ctx):
    """configs[0]: one 64x64 gradient+noise image, N = 32."""
    check_batch(l3, ctx, synth.config1(), layout="hwc")
    check_batch(l3, ctx, synth.config1(), layout="chw")


EDGE = [(1, 1), (2, 1), (1, 2), (3, 5), (4, 4), (5, 3), (31, 33), (33, 31), (32, 32), (63, 65),
        (65, 63), (127, 3), (129, 127), (130, 129), (257, 40), (40, 257), (450, 337)]


@pytest.mark.parametrize("patch", [32, 64, 128])
@pytest.mark.parametrize("layout", ["hwc", "chw"])
def test_edge_shapes(l3, ctx, patch, layout):
    """Ragged tails in both directions, one-pixel images, widths not a multiple of the
    pixels per lane, for every patch size of the GPU path; rows padded so that writes
    outside the image would be seen."""
    images = []
    for k, (w, h) in enumerate(EDGE):
        images.append(synth.cosine_field(700 + k, w, h))
        images.append(synth.uniform_bytes(800 + k, w, h))
    check_batch(l3, ctx, images, patch=patch, layout=layout, pad_cols=5)


def test_degenerate_content(l3, ctx):
    """All-zero, all-255, checkerboards (mod-256 wrap), constant rows (width 0)."""
    h, w = 70, 150
    yy, xx = np.mgrid[0:h, 0:w]
    images = [np.zeros((h, w, 3), np.uint8), np.full((h, w, 3), 255, np.uint8),
              (((yy + xx) & 1) * 255).astype(np.uint8)[:, :, None].repeat(3, 2),
              ((yy & 1) * 255).astype(np.uint8)[:, :, None].repeat(3, 2),
              (xx * 3 % 256).astype(np.uint8)[:, :, None].repeat(3, 2),
              (yy * 5 % 256).astype(np.uint8)[:, :, None].repeat(3, 2)]
    for patch in (32, 64, 128):
        check_batch(l3, ctx, images, patch=patch)


def test_non_canonical_streams(l3, ctx):
    """Streams with non-minimal widths (always 8; minimal + 1) decode identically."""
    images = [synth.cosine_field(31, 200, 150), synth.voronoi_scene(32, 260, 140)]
    for mode in (1, 2):
        for patch in (32, 128):
            check_batch(l3, ctx, images, patch=patch, width_mode=mode)


def test_default_patch_rule_sizes(l3, ctx):
    """One image per class of the patch-size rule, default N."""
    images = [synth.cosine_field(41, 500, 375), synth.voronoi_scene(42, 1280, 720),
              synth.gradient_noise(43, 1920, 1080, 3.0), synth.voronoi_scene(44, 2048, 1024)]
    files = [oracle.encode(im) for im in images]
    assert [f[12] for f in files] == [32, 64, 64, 128]
    check_batch(l3, ctx, images)


def test_config2_variable_batch(l3, ctx):
    """configs[1] at 24 images: variable sizes in one call, N = 32."""
    check_batch(l3, ctx, synth.config2(24))
    check_batch(l3, ctx, synth.config2(5), layout="chw")


def test_config4_mixed_compressibility(l3, ctx):
    """configs[3] at one image per half: 3840x2160, compressible and incompressible."""
    images = [synth.gradient_noise(4000, 3840, 2160, 2.0, span=255.0),
              synth.uniform_bytes(4004, 3840, 2160)]
    check_batch(l3, ctx, images)


def test_config3_full_batch_bench_configuration(l3, ctx):
    """configs[2] at full size, the launch the benchmark times: 32 images of 2048x1024,
    N = 128, every byte compared."""
    check_batch(l3, ctx, synth.config3(32))


def test_config2_full_batch_bench_configuration(l3, ctx):
    """configs[1] at full size, as the benchmark launches it: 256 images of 400-500 x 300-375 in
    one call (descriptor table pulled from pinned memory, N = 32), every byte compared."""
    check_batch(l3, ctx, synth.config2(256))


def test_config4_full_batch_bench_configuration(l3, ctx):
    """configs[3] at full size: 8 images of 3840x2160, four compressible and four random."""
    check_batch(l3, ctx, synth.config4(8))


def test_config5_full_batch_bench_configuration(l3, ctx):
    """configs[4] at full size: the 256-image batch through the fused window / mirror /
    normalise path, bf16, every element compared."""
    shapes = synth.config2_shapes(256)
    tensor_case(l3, ctx, synth.config2(256), synth.config5_crops(shapes), 224, 0)


@pytest.mark.parametrize("layout", ["hwc", "chw"])
def test_seeded_random_shapes_one_call(l3, ctx, layout):
    """120 images of seeded random size (1..400 x 1..260), content kind and patch size
    (32 / 64 / 128, forty of each: above the 32 per class that fit the kernel arguments, so the
    descriptor-table route with three launches) in one call, padded output rows."""
    gen = synth.Stream(0xC0FFEE, 7)
    images, patches = [], []
    for k in range(120):
        w = int(gen.integers(1, 400)[0])
        h = int(gen.integers(1, 260)[0])
        kind = int(gen.integers(0, 3)[0])
        if kind == 0:
            im = synth.gradient_noise(5000 + k, w, h, 3.0)
        elif kind == 1:
            im = synth.cosine_field(5000 + k, w, h)
        elif kind == 2:
            im = synth.voronoi_scene(5000 + k, w, h, sites=6)
        else:
            im = synth.uniform_bytes(5000 + k, w, h)
        images.append(im)
        patches.append((32, 64, 128)[k % 3])
    files = [oracle.encode(im, p) for im, p in zip(images, patches)]
    got, status = gpu_decode(l3, ctx, files, layout, pad_cols=3)
    assert (status == 0).all(), status
    for k, (g, im) in enumerate(zip(got, images)):
        assert np.array_equal(g, im), (k, im.shape, patches[k])


def test_all_patch_sizes_all_modes(l3, ctx):
    """Every patch size of the GPU path in all three output modes on a mix of shapes."""
    images = [synth.cosine_field(900 + k, w, h) for k, (w, h) in
              enumerate([(450, 337), (129, 127), (33, 70), (1, 1), (260, 131)])]
    images.append(synth.uniform_bytes(950, 300, 200))
    for patch in (32, 64, 128):
        check_batch(l3, ctx, images, patch=patch, layout="hwc", pad_cols=3)
        check_batch(l3, ctx, images, patch=patch, layout="chw", pad_cols=3)
    im = synth.cosine_field(960, 300, 260)
    for patch in (32, 64, 128):
        crops = [(0, 0, 0), (76, 36, 1), (37, 19, 1), (5, 30, 0)]
        tensor_case(l3, ctx, [im] * len(crops), crops, 224, 0, patch=patch)


@pytest.mark.parametrize("flat", ["1", "0"])
def test_units_across_patch_rows(l3, flat, monkeypatch):
    """Shapes whose patch rows do not fill whole work units, so that the library numbers the
    units in flat order and a unit's patches lie in several patch rows (down to one patch per
    row); with and without a shorter last patch row; both layouts, padded rows.  The same
    with the flat order switched off (the switch is read when a context is created)."""
    monkeypatch.setenv("L3_FLAT_ORDER", flat)
    ctx = l3.Context(0)
    shapes = [(40, 300), (32, 257), (70, 129), (33, 64), (450, 337), (97, 96), (200, 33), (130, 260),
              (1, 3000), (3, 1025)]
    images = [synth.cosine_field(1400 + k, w, h) for k, (w, h) in enumerate(shapes)]
    for patch in (32, 64, 128):
        for layout in ("hwc", "chw"):
            check_batch(l3, ctx, images, patch=patch, layout=layout, pad_cols=5)
    ctx.close()


def test_large_image_and_odd_output_address(l3, ctx):
    """A 5760x3840 image (the largest size in the paper's Table "compratio") with the
    default N = 128, decoded into a buffer that starts at an odd address with an odd
    row stride; and a 1-row-high, very wide image."""
    for im in (synth.voronoi_scene(970, 5760, 3840, sites=60), synth.cosine_field(971, 9000, 1)):
        f = oracle.encode(im)
        info = l3.peek_header(f)
        h, w = im.shape[:2]
        stride = 3 * w + 7
        dfiles, keep = upload_files([f])
        raw = torch.full((h * stride + 64,), 0xCD, dtype=torch.uint8, device="cuda")
        out = raw[3:3 + h * stride]
        status = torch.ones(1, dtype=torch.int32, device="cuda")
        l3.decode_batch(ctx, dfiles, [info], [out], status=status, row_strides=[stride])
        torch.cuda.synchronize()
        a = raw.cpu().numpy()
        assert (a[:3] == 0xCD).all() and (a[3 + h * stride:] == 0xCD).all()
        rows = a[3:3 + h * stride].reshape(h, stride)
        assert (rows[:, 3 * w:] == 0xCD).all()
        assert np.array_equal(rows[:, :3 * w].reshape(h, w, 3), im)
        assert int(status[0]) == 0


def test_mixed_patch_sizes_in_one_call(l3, ctx):
    images = [synth.cosine_field(51, 300, 200), synth.cosine_field(52, 300, 200),
              synth.cosine_field(53, 300, 200)]
    files = [oracle.encode(im, n) for im, n in zip(images, (128, 32, 64))]
    got, status = gpu_decode(l3, ctx, files)
    for g, im in zip(got, images):
        assert np.array_equal(g, im)
    assert (status == 0).all()


def test_damaged_streams_are_flagged_and_contained(l3, ctx):
    """A width field above 8 and a patch cut short set the image's status word; the
    other images of the batch decode cleanly; nothing is written outside the rows."""
    images = [synth.cosine_field(61 + k, 200, 120) for k in range(4)]
    files = [bytearray(oracle.encode(im, 32)) for im in images]
    hdr = 13 + 12 * (7 * 4)
    files[1][hdr] = (files[1][hdr] & 0xF0) | 0x0D            # width 13 in the first row record
    files[3] = files[3][:-40]                                 # last patches lose their tail
    # the host validator accepts both (offsets are still consistent)
    got, status = gpu_decode(l3, ctx, [bytes(f) for f in files], pad_cols=7)
    assert status[0] == 0 and status[2] == 0
    assert status[1] & 1
    assert status[3] & 2
    assert np.array_equal(got[0], images[0]) and np.array_equal(got[2], images[2])
    # damage stays inside its patch: every other patch of image 1 is intact
    diff = got[1] != images[1]
    diff[0:32, 0:32, 0] = False
    assert not diff.any()


def test_host_errors_enqueue_nothing(l3, ctx):
    im = synth.cosine_field(71, 100, 80)
    f = oracle.encode(im, 16)                                  # N = 16: not a GPU patch size
    info = l3.peek_header(f)
    dfiles, keep = upload_files([f])
    out = torch.zeros((80, 300), dtype=torch.uint8, device="cuda")
    with pytest.raises(l3.L3Error) as e:
        l3.decode_batch(ctx, dfiles, [info], [out])
    assert e.value.code == 6
    f = oracle.encode(im, 32)
    info = l3.peek_header(f)
    dfiles, keep = upload_files([f])
    with pytest.raises(l3.L3Error) as e:                       # stride too small
        l3.decode_batch(ctx, dfiles, [info], [out], row_strides=[299])
    assert e.value.code == 1
    torch.cuda.synchronize()
    assert int(out.sum()) == 0
    l3.decode_batch(ctx, [], [], [])                           # n = 0 is fine


def test_many_calls_reuse_slots(l3, ctx):
    """More calls in flight than staging slots (batches of 300 images go through the pinned
    descriptor tables); results stay correct."""
    images = [synth.cosine_field(1800 + k, 40 + (k % 9), 35 + (k % 4)) for k in range(300)]
    files = [oracle.encode(im) for im in images]
    infos = [l3.peek_header(f) for f in files]
    dfiles, keep = upload_files(files)
    outs = [[torch.zeros((im.shape[0], im.shape[1] * 3), dtype=torch.uint8, device="cuda")
             for im in images] for _ in range(12)]
    for rep in range(12):
        l3.decode_batch(ctx, dfiles, infos, outs[rep])
    torch.cuda.synchronize()
    for rep in range(12):
        for t, im in zip(outs[rep], images):
            assert np.array_equal(t.cpu().numpy().reshape(im.shape), im)


def test_two_contexts_two_streams_and_one_context_on_alternating_streams(l3, ctx):
    """Calls of two contexts on two streams, enqueued alternately without waiting, and then
    one context switching between the two streams from call to call; batches of 5 images
    (descriptors inside the small kernel-argument block), of 40 (the large block) and of 300
    (descriptor table through the staging slots); the fused path as well, whose table of
    normalised values is kept across calls.  Every output is checked."""
    small = [synth.cosine_field(1300 + k, 200 + 7 * k, 90 + 5 * k) for k in range(5)]
    large = [synth.gradient_noise(1320 + k, 40 + k, 33 + (k % 7), 2.0) for k in range(40)]
    huge = [synth.gradient_noise(1700 + k, 33 + (k % 5), 34 + (k % 3), 2.0) for k in range(300)]
    other = l3.Context(0)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    try:
        work = []
        for images in (small, large, huge):
            files = [oracle.encode(im, 32) for im in images]
            infos = [l3.peek_header(f) for f in files]
            dfiles, keep = upload_files(files)
            work.append((images, infos, dfiles, keep))
        torch.cuda.synchronize()
        results = []
        for rep in range(10):
            for which, (images, infos, dfiles, keep) in enumerate(work):
                # first half: each context keeps its stream; second half: one context, both streams
                c = (ctx, other)[(rep + which) % 2] if rep < 5 else ctx
                st = streams[(rep + which) % 2]
                outs = [torch.full((im.shape[0], im.shape[1] * 3), 0xEE, dtype=torch.uint8, device="cuda")
                        for im in images]
                status = torch.full((len(images),), 0x55, dtype=torch.int32, device="cuda")
                st.wait_stream(torch.cuda.current_stream())      # the fills above
                print(f"two streams: rep={rep} images={len(images)}", flush=True)
                l3.decode_batch(c, dfiles, infos, outs, status=status, stream=st)
                results.append((images, outs, status))
        # the fused path from both streams with different constants each time
        files = [oracle.encode(im, 32) for im in small]
        infos = [l3.peek_header(f) for f in files]
        dfiles, keep2 = upload_files(files)
        crops = [(3 * k, 2 * k, k & 1) for k in range(len(small))]
        fused = []
        for rep in range(6):
            mean = [0.1 * rep, 0.5, 0.25]
            stdv = [0.5, 0.2 + 0.1 * rep, 1.0]
            out = torch.full((len(small), 3, 64, 64), -1, dtype=torch.int16, device="cuda")
            st = streams[rep % 2]
            st.wait_stream(torch.cuda.current_stream())
            l3.decode_crop_normalize_batch(ctx, dfiles, infos, crops, 64, 64, mean, stdv, out,
                                           dtype=l3.BF16, stream=st)
            fused.append((mean, stdv, out))
        torch.cuda.synchronize()
        for images, outs, status in results:
            assert (status.cpu().numpy() == 0).all()
            for t, im in zip(outs, images):
                assert np.array_equal(t.cpu().numpy().reshape(im.shape), im)
        for mean, stdv, out in fused:
            got = out.cpu().numpy().view(np.uint16)
            for i, (im, (x0, y0, flip)) in enumerate(zip(small, crops)):
                want = oracle.crop_normalize(im, x0, y0, flip, 64, 64, mean, stdv, 0)
                assert np.array_equal(got[i], want), (mean, stdv, i)
    finally:
        other.close()


# ---------------------------------------------------------------------------
# fused crop + flip + normalise (configs[4])

def tensor_case(l3, ctx, images, crops, crop, dtype, patch=0, mean=None, stdv=None):
    mean = synth.IMAGENET_MEAN if mean is None else mean
    stdv = synth.IMAGENET_STD if stdv is None else stdv
    files = [oracle.encode(im, patch) for im in images]
    infos = [l3.peek_header(f) for f in files]
    dfiles, keep = upload_files(files)
    n = len(files)
    out = torch.full((n, 3, crop, crop), -1, dtype=torch.int16, device="cuda")
    status = torch.zeros(n, dtype=torch.int32, device="cuda")
    l3.decode_crop_normalize_batch(ctx, dfiles, infos, crops, crop, crop, mean, stdv, out,
                                   dtype=dtype, status=status)
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16)
    assert (status.cpu().numpy() == 0).all()
    ftype = torch.bfloat16 if dtype == 0 else torch.float16
    for i, (im, (x0, y0, flip)) in enumerate(zip(images, crops)):
        want = oracle.crop_normalize(oracle.decode(files[i]), x0, y0, flip, crop, crop, mean, stdv,
                                     dtype)
        a = torch.from_numpy(got[i].view(np.int16)).view(ftype).float()
        b = torch.from_numpy(want.view(np.int16)).view(ftype).float()
        assert float((a - b).abs().max()) <= 1e-3          # the stated tolerance
        assert np.array_equal(got[i], want)                # and in fact identical bits


def test_fused_crop_normalize_config5(l3, ctx):
    """configs[4] at 32 images: 224x224 window, mirror with p = 0.5, bf16 NCHW;
    tolerance 1e-3 absolute on the 16-bit values (they are bit-identical)."""
    n = 32
    shapes = synth.config2_shapes(n)
    images = synth.config2(n)
    crops = synth.config5_crops(shapes)
    tensor_case(l3, ctx, images, crops, 224, 0)
    tensor_case(l3, ctx, images[:6], crops[:6], 224, 1)


def test_fused_call_with_more_images_than_the_argument_block_holds(l3, ctx):
    """300 small images: the descriptors go through the table in device memory, the normalised
    values still through the kernel's arguments; both output types, mirrored and not."""
    images = [synth.gradient_noise(5200 + k, 40 + (k % 9), 36 + (k % 4), 2.0) for k in range(300)]
    crops = [(k % 9, k % 5, k & 1) for k in range(300)]
    tensor_case(l3, ctx, images, crops, 32, 0, patch=32)
    tensor_case(l3, ctx, images, crops, 32, 1, patch=32, mean=(0.3, 0.4, 0.5), stdv=(0.5, 0.25, 2.0))


def test_fused_constants_change_between_calls(l3, ctx):
    """The normalisation table is kept between calls: ten calls on one context that
    alternate between three sets of constants and the two output types must each use
    their own."""
    im = synth.cosine_field(83, 260, 240)
    crops = [(3, 5, 0), (20, 10, 1)]
    sets = [(synth.IMAGENET_MEAN, synth.IMAGENET_STD), ((0.5, 0.5, 0.5), (0.25, 0.5, 1.0)),
            ((0.0, 0.1, 0.9), (1.0, 2.0, 0.125))]
    for k in range(10):
        mean, stdv = sets[k % 3]
        tensor_case(l3, ctx, [im, im], crops, 224, k % 2, mean=mean, stdv=stdv)


def test_fused_crop_edges(l3, ctx):
    """Windows touching every image border, whole-image window, larger patch sizes."""
    im = synth.cosine_field(81, 300, 260)
    for patch in (32, 64, 128):
        crops = [(0, 0, 0), (300 - 224, 260 - 224, 1), (0, 260 - 224, 1), (300 - 224, 0, 0),
                 (37, 19, 1)]
        tensor_case(l3, ctx, [im] * len(crops), crops, 224, 0, patch=patch)
    small = synth.cosine_field(82, 50, 40)
    files_crop = [(0, 0, 1)]
    # whole image as the window
    f = oracle.encode(small, 32)
    info = l3.peek_header(f)
    dfiles, keep = upload_files([f])
    out = torch.zeros((1, 3, 40, 50), dtype=torch.int16, device="cuda")
    l3.decode_crop_normalize_batch(ctx, dfiles, [info], files_crop, 50, 40, synth.IMAGENET_MEAN,
                                   synth.IMAGENET_STD, out)
    torch.cuda.synchronize()
    want = oracle.crop_normalize(small, 0, 0, 1, 50, 40, synth.IMAGENET_MEAN, synth.IMAGENET_STD, 0)
    assert np.array_equal(out.cpu().numpy().view(np.uint16)[0], want)


@pytest.mark.parametrize("count", [5, 40])
def test_decode_batch_replayed_from_a_captured_graph(l3, ctx, count):
    """Batches of at most 256 images carry their descriptors in the kernel arguments (a small
    block up to 32 images, a large one beyond) and allocate nothing once the context is warm,
    so the call can be captured into a HIP graph.  Every replay (with eager work and
    synchronisation between them) must give the eager result."""
    images = [synth.voronoi_scene(3300 + k, 100 + 7 * (k % 9), 70 + 3 * (k % 11), sites=9) for k in range(count)]
    files = [oracle.encode(im) for im in images]
    infos = [l3.peek_header(f) for f in files]
    dfiles, keep = upload_files(files)
    outs = [torch.zeros((im.shape[0], im.shape[1] * 3), dtype=torch.uint8, device="cuda") for im in images]
    status = torch.full((len(files),), 9, dtype=torch.int32, device="cuda")
    batch = l3.PreparedBatch(dfiles, infos, outs)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        l3.decode_batch_prepared(ctx, batch, status=status, stream=side)      # warm, eager
    torch.cuda.synchronize()
    want = [t.cpu().numpy().copy() for t in outs]
    for w_, im in zip(want, images):
        assert np.array_equal(w_.reshape(im.shape), im)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        l3.decode_batch_prepared(ctx, batch, status=status, stream=torch.cuda.current_stream())
    for rep in range(4):
        for t in outs:
            t.fill_(rep + 1)                 # eager work between the replays
        status.fill_(5)
        torch.cuda.synchronize()
        print(f"graph replay {rep}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert (status.cpu().numpy() == 0).all()
        for t, w_ in zip(outs, want):
            assert np.array_equal(t.cpu().numpy(), w_)


def test_fused_call_replayed_from_a_captured_graph(l3, ctx):
    """Under stream capture the fused call records the build of its table into the graph (a
    table of its own), so that replays stand alone: between the replays eager fused calls
    with other constants run on the same context, and every replay must give the eager
    result of its own constants."""
    n = 12
    shapes = synth.config2_shapes(n)
    images = synth.config2(n)
    crops = synth.config5_crops(shapes)
    files = [oracle.encode(im) for im in images]
    infos = [l3.peek_header(f) for f in files]
    dfiles, keep = upload_files(files)
    mean, stdv = (0.4, 0.5, 0.6), (0.2, 0.3, 0.4)
    batch = l3.PreparedCropBatch(dfiles, infos, crops, mean, stdv)
    out = torch.zeros((n, 3, 224, 224), dtype=torch.int16, device="cuda")
    other = torch.zeros((n, 3, 224, 224), dtype=torch.int16, device="cuda")
    status = torch.full((n,), 9, dtype=torch.int32, device="cuda")
    want = np.stack([oracle.crop_normalize(im, x0, y0, flip, 224, 224, mean, stdv, 0)
                     for im, (x0, y0, flip) in zip(images, crops)])
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        l3.decode_crop_normalize_batch_prepared(ctx, batch, 224, 224, out, status=status, stream=side)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint16), want)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        l3.decode_crop_normalize_batch_prepared(ctx, batch, 224, 224, out, status=status,
                                                stream=torch.cuda.current_stream())
    for rep in range(4):
        out.fill_(rep + 1)
        status.fill_(5)
        # an eager call with other constants in between (five changes walk through every slot)
        l3.decode_crop_normalize_batch(ctx, dfiles, infos, crops, 224, 224, (0.1 * rep, 0.2, 0.3),
                                       (1.0, 0.5 + rep, 0.25), other)
        torch.cuda.synchronize()
        print(f"fused graph replay {rep}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert (status.cpu().numpy() == 0).all()
        assert np.array_equal(out.cpu().numpy().view(np.uint16), want)


def _decode_many_small(l3, ctx, images):
    """Thousands of tiny images in one call: one output buffer, one slot of 64 bytes each."""
    files = [oracle.encode(im, 32) for im in images]
    infos = [l3.peek_header(f) for f in files]
    dfiles, keep = upload_files(files, misalign=False)
    n = len(files)
    out = torch.full((n, 64), 0x5A, dtype=torch.uint8, device="cuda")
    outs = [out[i] for i in range(n)]
    status = torch.full((n,), 3, dtype=torch.int32, device="cuda")
    l3.decode_batch(ctx, dfiles, infos, outs, status=status)
    torch.cuda.synchronize()
    assert int(status.abs().sum()) == 0
    return out.cpu().numpy()


def test_every_pair_of_values_in_a_column(l3, ctx):
    """All 65,536 (top, bottom) byte pairs as 1 x 2 images (three different pairings in the
    three channels): the modulo-256 arithmetic of base, delta and predictor for every value."""
    a, b = np.meshgrid(np.arange(256, dtype=np.uint8), np.arange(256, dtype=np.uint8), indexing="ij")
    a, b = a.ravel(), b.ravel()
    images = []
    for i in range(a.size):
        im = np.empty((2, 1, 3), np.uint8)
        im[0, 0] = (a[i], b[i], 255 - a[i])
        im[1, 0] = (b[i], a[i], b[i])
        images.append(im)
    got = _decode_many_small(l3, ctx, images)
    want = np.stack([im.reshape(-1) for im in images])
    assert np.array_equal(got[:, :6], want)
    assert (got[:, 6:] == 0x5A).all()


def test_predictor_grid_on_the_gpu(l3, ctx):
    """3 x 2 images: the upper row over the value grid {0, 1, 127, 128, 129, 200, 254, 255}^3,
    the pixel below its centre over all 256 values (131,072 images): every kind of neighbour
    ordering, tie and wrap goes through the packed predictor."""
    grid = np.array([0, 1, 127, 128, 129, 200, 254, 255], dtype=np.uint8)
    images = []
    for tl in grid:
        for t in grid:
            for tr in grid:
                for v in range(256):
                    im = np.empty((2, 3, 3), np.uint8)
                    im[0, :, 0] = (tl, t, tr)
                    im[0, :, 1] = (tr, tl, t)
                    im[0, :, 2] = (t, tr, tl)
                    im[1, :, 0] = (tl, v, tr)
                    im[1, :, 1] = (v, 255 - v, v)
                    im[1, :, 2] = (tr, (v + 128) & 255, t)
                    images.append(im)
    got = _decode_many_small(l3, ctx, images)
    want = np.stack([im.reshape(-1) for im in images])
    assert np.array_equal(got[:, :18], want)
    assert (got[:, 18:] == 0x5A).all()


def test_abi_from_plain_c():
    """tests/native/abi_roundtrip.c (built with gcc as C99 next to the library): encode on the
    host, decode on the GPU through the C ABI with nothing but the HIP runtime beside it."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native", "abi_roundtrip.bin")
    assert os.path.exists(exe), "build first: python -c 'import __graft_entry__ as g; g.build()'"
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(run.stdout, run.stderr, flush=True)
    assert run.returncode == 0, (run.returncode, run.stderr)
    assert "abi_roundtrip ok" in run.stdout
