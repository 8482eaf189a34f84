"""Load + Decode (arxiv 2208.08711 Section 3.1: a batch is loaded from storage into host memory,
then decoded; Section 5.3 measures the two together): L3 files written to a directory are read
into pinned staging buffers, copied to the GPU on a copy stream and decoded on a second stream,
double-buffered over several batches.  Every decoded byte is compared with the oracle."""
import os

import numpy as np
import pytest

import oracle
from paper_2208_08711_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_files_to_pinned_to_device_to_pixels(tmp_path):
    import paper_2208_08711_amd as l3
    assert torch.cuda.is_available(), "this test needs the GPU"
    batches = []
    for b in range(4):                                        # four batches of mixed shapes
        images = synth.config2(6)[b:b + 5] + [synth.voronoi_scene(9100 + b, 1280, 720),
                                              synth.voronoi_scene(9200 + b, 2048, 1024)]
        names = []
        for k, im in enumerate(images):
            name = os.path.join(tmp_path, "b%d_%d.l3" % (b, k))
            with open(name, "wb") as fh:
                fh.write(oracle.encode(im))
            names.append(name)
        batches.append((images, names))
    cap = max(sum(os.path.getsize(nm) + 64 for nm in names) for _, names in batches)
    pinned = [torch.empty(cap, dtype=torch.uint8, pin_memory=True) for _ in range(2)]
    device = [torch.empty(cap, dtype=torch.uint8, device="cuda") for _ in range(2)]
    copied = [torch.cuda.Event() for _ in range(2)]
    decoded = [torch.cuda.Event() for _ in range(2)]
    copy_stream, decode_stream = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = l3.Context(0)
    results = []
    try:
        for b, (images, names) in enumerate(batches):
            s = b % 2
            if b >= 2:
                decoded[s].synchronize()                      # the staging pair is free again
            # Load: file bytes into the pinned buffer, each file at an odd offset
            host = pinned[s].numpy()
            offs, infos, pos = [], [], 0
            for k, nm in enumerate(names):
                pos = (pos + 63) // 64 * 64 + (1 + 2 * k) % 16
                with open(nm, "rb") as fh:
                    data = fh.read()
                host[pos:pos + len(data)] = np.frombuffer(data, dtype=np.uint8)
                infos.append(l3.peek_header(data))           # header parse on the host
                offs.append((pos, len(data)))
                pos += len(data)
            with torch.cuda.stream(copy_stream):
                device[s][:pos].copy_(pinned[s][:pos], non_blocking=True)
                copied[s].record(copy_stream)
            decode_stream.wait_event(copied[s])
            dfiles = [device[s][o:o + ln] for o, ln in offs]
            outs = [torch.zeros((im.shape[0], im.shape[1] * 3), dtype=torch.uint8, device="cuda")
                    for im in images]
            status = torch.full((len(images),), 0x55, dtype=torch.int32, device="cuda")
            l3.decode_batch(ctx, dfiles, infos, outs, status=status, stream=decode_stream)
            decoded[s].record(decode_stream)
            results.append((outs, status))
        torch.cuda.synchronize()
    finally:
        ctx.close()
    for (images, names), (outs, status) in zip(batches, results):
        assert (status.cpu().numpy() == 0).all()
        for im, nm, t in zip(images, names, outs):
            with open(nm, "rb") as fh:
                want = oracle.decode(fh.read())
            assert np.array_equal(want, im)
            assert np.array_equal(t.cpu().numpy().reshape(im.shape), want)
