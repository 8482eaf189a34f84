"""Decode beside compute (arxiv 2208.08711 Section 4.4, decoding and gradient computing on separate
streams): a Cityscapes-shaped batch is decoded on one stream while a matrix-multiply loop runs on a
second stream of the same, default priority.  Every decoded byte is compared with the oracle, and
the products with the ones computed alone."""
import numpy as np
import pytest

import oracle
from paper_2208_08711_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_decode_beside_a_matmul_loop():
    import paper_2208_08711_amd as l3
    assert torch.cuda.is_available(), "this test needs the GPU"
    n = 8                                                    # images of 2048 x 1024, N = 128
    images = synth.config3(n)
    files = [oracle.encode(im) for im in images]
    assert all(f[12] == 128 for f in files)
    infos = [l3.peek_header(f) for f in files]
    dfiles = [torch.from_numpy(np.frombuffer(f, dtype=np.uint8).copy()).cuda() for f in files]
    rounds = 6
    outs = [[torch.zeros((1024, 2048 * 3), dtype=torch.uint8, device="cuda") for _ in files]
            for _ in range(rounds)]
    status = torch.full((rounds, n), 0x55, dtype=torch.int32, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(11)
    a = torch.randn((4096, 4096), device="cuda", dtype=torch.bfloat16, generator=gen)
    b = torch.randn((4096, 4096), device="cuda", dtype=torch.bfloat16, generator=gen)
    alone = a @ b
    torch.cuda.synchronize()
    compute, decode = torch.cuda.Stream(), torch.cuda.Stream()       # default priorities
    ctx = l3.Context(0)
    try:
        products = []
        with torch.cuda.stream(compute):
            for _ in range(40):
                products.append(a @ b)
        for r in range(rounds):                                       # enqueued while the loop runs
            l3.decode_batch(ctx, dfiles, infos, outs[r], status=status[r], stream=decode)
        with torch.cuda.stream(compute):
            for _ in range(20):
                products.append(a @ b)
        torch.cuda.synchronize()
    finally:
        ctx.close()
    assert (status.cpu().numpy() == 0).all()
    want = [oracle.decode(f) for f in files]
    for r in range(rounds):
        for t, w, im in zip(outs[r], want, images):
            assert np.array_equal(w, im)
            assert np.array_equal(t.cpu().numpy().reshape(w.shape), w), r
    for p in (products[0], products[20], products[-1]):
        assert torch.allclose(p.float(), alone.float(), rtol=2e-2, atol=1.0)
