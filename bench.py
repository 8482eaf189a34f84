#!/usr/bin/env python3
"""Benchmark of the L3 batch decoder on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cityscapes|imagenet|uhd]

A step is one l3_decode_batch call over one batch of synthetic images whose
compressed files are already resident in HBM: the whole hot path (descriptor
upload, stream staging, base-delta unpacking, inverse filter, RGB store).  The
default workload is the Cityscapes-shaped batch the headline metric is quoted on
(32 images of 2048x1024, N = 128).  Several input/output buffer sets are rotated
so that consecutive steps do not hit in the last-level cache.

Prints one JSON line.  `roofline` is the HBM view the target is stated in:
(file bytes read + decoded bytes written) per launch divided by the launch time
measured with events on the launch stream, against 8 TB/s; `cpu_baseline` is the CPU oracle decoding the same files on the
host cores (a reported baseline, not a target).
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
VALU_ISSUE_PER_S = 256 * 4 * 2.4e9 / 4      # wave instructions per second: 1024 SIMDs, one per 4 cycles
KERNEL_SOURCES = ("paper_2208_08711_amd/csrc/l3_device.hip", "paper_2208_08711_amd/csrc/l3_gfx950.h",
                  "paper_2208_08711_amd/csrc/l3_kernel_parts.h")


def kernel_source_stamp():
    """Hash of the decode kernel's sources: counter summaries under profiles/ carry the stamp of
    the sources they were measured with, and count only while it still matches."""
    import hashlib
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def read_counters(workload):
    """Per-launch counters of the decode kernel from the committed rocprofv3 summary of this
    workload (profiles/l3_decode_kernel_<workload>_counters.txt, written by the profile run):
    HBM bytes (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy) and SQ_INSTS_VALU.  None if there
    is no summary or if it was measured with other kernel sources than the ones in the tree."""
    path = os.path.join(ROOT, "profiles", "l3_decode_kernel_%s_counters.txt" % workload)
    if not os.path.exists(path):
        return None
    vals = {}
    with open(path) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if "=" in line:
                k, v = line.split("=", 1)
                vals[k.strip()] = v.strip()
    if vals.get("kernel_source_stamp") != kernel_source_stamp():
        return None
    return vals


def make_workload(name, batch=0):
    from paper_2208_08711_amd import synth
    if name == "cityscapes":
        n = batch or 32
        return synth.config3(n), ("Cityscapes-shaped: %d RGB images 2048x1024, Voronoi regions + texture, "
                                  "N=128" % n)
    if name == "cityscapes044":
        n = batch or 32
        return [synth.cosine_field(3500 + k, 2048, 1024, sigma=0.93) for k in range(n)], (
            "Cityscapes-sized at the paper's compression ratio: %d RGB images 2048x1024, smooth cosine "
            "field + noise sigma 0.93 (compressed/raw 0.44 as in the paper's Table compratio), N=128" % n)
    if name == "fhd":
        n = batch or 32
        return synth.config3(n, width=1920, height=1080), ("FHD: %d RGB images 1920x1080, Voronoi regions + "
                                                           "texture, N=64" % n)
    if name == "kitti":
        n = batch or 64
        return synth.config3(n, width=1024, height=720), ("KITTI-shaped: %d RGB images 1024x720, Voronoi regions "
                                                          "+ texture, N=32" % n)
    if name == "imagenet":
        return synth.config2(256), "ImageNet-shaped: 256 RGB images 400-500 x 300-375, cosine field + noise, N=32"
    if name == "train224":
        return synth.config2(256), ("Fused training-input path: the ImageNet-shaped batch of 256, seeded 224x224 "
                                    "window + mirror + per-channel normalise to bf16 NCHW, N=32")
    if name == "uhd":
        return synth.config4(8), "UHD stress: 8 RGB images 3840x2160, half compressible, half random, N=128"
    raise SystemExit(f"unknown workload {name}")


def measure_load_decode(torch, l3, ctx, images, files, infos, stream):
    """Host-resident files -> H2D copy on a side stream -> decode, two buffer sets."""
    n = len(files)
    offs, pos = [], 0
    for f in files:
        offs.append(pos)
        pos = (pos + len(f) + 63) // 64 * 64
    blob = torch.empty(pos, dtype=torch.uint8, pin_memory=True)
    hb = blob.numpy()
    for o, f in zip(offs, files):
        hb[o:o + len(f)] = np.frombuffer(f, dtype=np.uint8)
    copy_stream = torch.cuda.Stream()
    sets = []
    for _ in range(2):
        dev = torch.empty(pos, dtype=torch.uint8, device="cuda")
        dfiles = [dev[o:o + len(f)] for o, f in zip(offs, files)]
        outs = [torch.empty((im.shape[0], im.shape[1] * 3), dtype=torch.uint8, device="cuda")
                for im in images]
        sets.append({"dev": dev, "batch": l3.PreparedBatch(dfiles, infos, outs), "outs": outs,
                     "copied": torch.cuda.Event(), "decoded": torch.cuda.Event()})

    def run(steps):
        for k in range(steps):
            s = sets[k % 2]
            copy_stream.wait_event(s["decoded"])          # the set's previous decode has read it
            with torch.cuda.stream(copy_stream):
                s["dev"].copy_(blob, non_blocking=True)
                s["copied"].record(copy_stream)
            stream.wait_event(s["copied"])
            l3.decode_batch_prepared(ctx, s["batch"], stream=stream)
            s["decoded"].record(stream)

    for s in sets:
        s["decoded"].record(stream)
    run(4)
    torch.cuda.synchronize()
    steps = 40
    t0 = time.perf_counter()
    run(steps)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    for t, im in zip(sets[(steps - 1) % 2]["outs"], images):
        if not np.array_equal(t.cpu().numpy().reshape(im.shape), im):
            raise SystemExit("bench.py: pipeline output differs from the input images")
    result = {"ms_per_batch": dt * 1e3, "images_per_s": n / dt,
              "file_bytes_per_batch": sum(map(len, files)), "h2d_GBps": pos / dt / 1e9,
              "note": "files in pinned host memory, one H2D copy per batch on a second stream, "
                      "double-buffered against the decode"}

    # The same with the files read from a directory first (one file per image, read by a
    # pool of threads into two pinned staging buffers, so reading batch k+1 overlaps the
    # copy and decode of batch k).  The files were just written, so the reads are served
    # by the page cache: this is the file-system path, not a storage device's bandwidth.
    import tempfile
    with tempfile.TemporaryDirectory(prefix="l3_bench_") as tmp:
        paths = []
        for k, f in enumerate(files):
            paths.append(os.path.join(tmp, "%05d.l3" % k))
            with open(paths[-1], "wb") as fh:
                fh.write(f)
        stages = [torch.empty(pos, dtype=torch.uint8, pin_memory=True) for _ in range(2)]
        views = [memoryview(st.numpy()) for st in stages]
        workers = min(16, os.cpu_count() or 1)

        def read_one(args):
            k, which = args
            with open(paths[k], "rb", buffering=0) as fh:
                got = fh.readinto(views[which][offs[k]:offs[k] + len(files[k])])
            if got != len(files[k]):
                raise SystemExit("bench.py: short read")

        with ThreadPoolExecutor(max_workers=workers) as pool:
            def run_disk(steps):
                for k in range(steps):
                    s = sets[k % 2]
                    s["copied"].synchronize()       # the staging buffer's last copy has left it
                    list(pool.map(read_one, [(i, k % 2) for i in range(n)]))
                    copy_stream.wait_event(s["decoded"])
                    with torch.cuda.stream(copy_stream):
                        s["dev"].copy_(stages[k % 2], non_blocking=True)
                        s["copied"].record(copy_stream)
                    stream.wait_event(s["copied"])
                    l3.decode_batch_prepared(ctx, s["batch"], stream=stream)
                    s["decoded"].record(stream)

            for s in sets:
                s["outs"][0].zero_()
            run_disk(4)
            torch.cuda.synchronize()
            steps = 20
            t0 = time.perf_counter()
            run_disk(steps)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / steps
        for t, im in zip(sets[(steps - 1) % 2]["outs"], images):
            if not np.array_equal(t.cpu().numpy().reshape(im.shape), im):
                raise SystemExit("bench.py: file pipeline output differs from the input images")
    result["from_files"] = {"ms_per_batch": dt * 1e3, "images_per_s": n / dt,
                            "read_GBps": sum(map(len, files)) / dt / 1e9, "reader_threads": workers,
                            "note": "one file per image in a temporary directory, page cache warm"}
    return result


def measure_ablation(torch, l3, ctx, images, files, infos, stream, patch, product_ms):
    """The four decoder variants of Section 5.5 (plain kernels, one wave per patch and
    channel), each checked against the input images, plus two of them with the patches
    of an image taken one after another."""
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
        files_orig = list(pool.map(lambda im: l3.encode_cpu(im, patch, original_filter=True), images))
    sets = {}
    for custom, fl in ((False, files_orig), (True, files)):
        dfiles = [torch.from_numpy(np.frombuffer(f, dtype=np.uint8).copy()).cuda() for f in fl]
        finfos = [l3.peek_header(f) for f in fl]
        outs = [torch.empty((im.shape[0], im.shape[1] * 3), dtype=torch.uint8, device="cuda")
                for im in images]
        sets[custom] = (l3.PreparedBatch(dfiles, finfos, outs), outs, sum(map(len, fl)))
    PB, CF, SP = l3.ABLATION_PIXEL_BD, l3.ABLATION_CUSTOM_FILTER, l3.ABLATION_SERIAL_PATCHES
    DG = l3.ABLATION_DIAGONAL
    variants = [("baseline: original filter, one lane per patch for both stages", 0),
                ("+pixel-wise base-delta", PB),
                ("+custom filter", CF),
                ("+pixel-wise base-delta +custom filter", PB | CF),
                ("+pixel-wise base-delta, original filter along anti-diagonals (not in the paper)", PB | DG),
                ("baseline, patches of an image in turn", SP),
                ("+both, patches of an image in turn", PB | CF | SP)]
    rows = []
    for name, v in variants:
        batch, outs, _ = sets[bool(v & CF)]
        for t in outs:
            t.zero_()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        l3.ablation_decode_batch(ctx, batch, v, stream=stream)       # uploads the table, warms up
        torch.cuda.synchronize()
        for k in (0, len(images) - 1):
            if not np.array_equal(outs[k].cpu().numpy().reshape(images[k].shape), images[k]):
                raise SystemExit("bench.py: ablation variant %d decoded wrong pixels" % v)
        e0.record(stream)
        l3.ablation_decode_batch(ctx, batch, v, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        first = e0.elapsed_time(e1)
        reps = int(max(1, min(50, 300.0 / max(first, 1e-3))))
        e0.record(stream)
        for _ in range(reps):
            l3.ablation_decode_batch(ctx, batch, v, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        rows.append({"variant": name, "flags": v, "ms_per_batch": e0.elapsed_time(e1) / reps, "reps": reps})
    base = rows[0]["ms_per_batch"]
    for r in rows:
        r["normalized"] = r["ms_per_batch"] / base
    return {"variants": rows, "tuned_decoder_ms": product_ms,
            "file_bytes": {"original_filter": sets[False][2], "custom_filter": sets[True][2]},
            "note": "plain kernels of l3_ablation_decode_batch; normalised to the baseline as in the "
                    "paper's figure; the tuned decoder is l3_decode_batch on the same batch"}


def measure_encode(torch, l3, ctx, images, files, stream, patch):
    """l3_encode_batch on the workload's images; the files must equal l3_encode_cpu's."""
    n = len(images)
    dimgs = [torch.from_numpy(np.ascontiguousarray(im)).cuda() for im in images]
    caps = [l3.encode_bound(im.shape[1], im.shape[0], patch) for im in images]
    dfiles = [torch.empty(c, dtype=torch.uint8, device="cuda") for c in caps]
    lens = torch.zeros(n, dtype=torch.int64, device="cuda")
    status = torch.zeros(n, dtype=torch.int32, device="cuda")
    for _ in range(3):
        l3.encode_batch(ctx, dimgs, dfiles, lens, patch=patch, status=status, stream=stream)
    torch.cuda.synchronize()
    reps = 20
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        l3.encode_batch(ctx, dimgs, dfiles, lens, patch=patch, status=status, stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    if int(status.abs().sum()) != 0:
        raise SystemExit("bench.py: encoder reported a status")
    got = lens.cpu().tolist()
    for i in (0, n // 2, n - 1):
        if dfiles[i][:got[i]].cpu().numpy().tobytes() != files[i]:
            raise SystemExit("bench.py: GPU-encoded file differs from the CPU encoder's")
    raw = sum(im.size for im in images)
    out = sum(got)
    return {"ms_per_batch": ms, "images_per_s": n / (ms * 1e-3), "raw_GBps": raw / (ms * 1e-3) / 1e9,
            "hbm_fraction": (raw + out) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "note": "three kernels per call: strip (filter, row min/max, bit packing into per-patch "
                    "slots), layout (prefix sum of the patch sizes), compact (slots to the file)"}


def measure_overlap(torch, step, stream, steps, decode_alone_ms):
    """Decode steps on `stream`, a bf16 GEMM loop on a second stream (both default priority):
    each alone, and the rates of both while both streams have work.  The decode steps are
    enqueued in chunks with an event behind each; the chunks that lie entirely inside the GEMM
    loop's interval give the decode rate beside compute, the interval itself the GEMM rate
    beside decoding (the decode stream is given enough steps to outlast the loop)."""
    side = torch.cuda.Stream()
    m = 8192
    a = torch.randn((m, m), dtype=torch.bfloat16, device="cuda")
    b = torch.randn((m, m), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((m, m), dtype=torch.bfloat16, device="cuda")

    def gemms(k):
        with torch.cuda.stream(side):
            for _ in range(k):
                torch.matmul(a, b, out=out)

    gemms(60)                    # long enough for the clocks to settle under this load too
    torch.cuda.synchronize()
    g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    g0.record(side)
    gemms(60)
    g1.record(side)
    torch.cuda.synchronize()
    gemm_alone_ms = g0.elapsed_time(g1) / 60
    n_gemm, chunk = 150, 5
    # decode steps: several times what fits beside the loop even if decoding kept its full speed
    n_chunks = max(40, int(1.5 * n_gemm * gemm_alone_ms / (decode_alone_ms * chunk)) // 8)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_chunks + 1)]
    g0.record(side)
    gemms(n_gemm)
    g1.record(side)
    marks[0].record(stream)
    for c in range(n_chunks):
        for k in range(chunk):
            step(c * chunk + k)
        marks[c + 1].record(stream)
    torch.cuda.synchronize()
    gemm_span = g0.elapsed_time(g1)
    inside = [marks[c].elapsed_time(marks[c + 1]) / chunk for c in range(n_chunks)
              if g0.elapsed_time(marks[c]) >= 0.0 and g0.elapsed_time(marks[c + 1]) <= gemm_span]
    outlasted = g0.elapsed_time(marks[n_chunks]) > gemm_span
    beside = sum(inside) / len(inside) if inside else None
    return {"compute": "torch.matmul bf16 %dx%dx%d on a second stream, default priority" % (m, m, m),
            "gemms": n_gemm, "decode_steps_enqueued": n_chunks * chunk,
            "decode_steps_inside_the_gemm_loop": len(inside) * chunk,
            "decode_stream_outlasted_the_gemm_loop": outlasted,
            "decode_ms_per_step_alone": decode_alone_ms,
            "decode_ms_per_step_beside_compute": beside,
            "gemm_ms_alone": gemm_alone_ms,
            "gemm_ms_beside_decode": gemm_span / n_gemm,
            "gemm_TFLOPs_alone": 2.0 * m ** 3 / (gemm_alone_ms * 1e-3) / 1e12}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--workload", default="cityscapes",
                    help="cityscapes (default, the configuration the metric is quoted on), cityscapes044 "
                         "(same shape, content at the paper's Cityscapes compression ratio), fhd, kitti, "
                         "imagenet, uhd, train224")
    ap.add_argument("--sets", type=int, default=4, help="rotating buffer sets")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="after the timed steps also run 5 plain device copies of BYTES bytes "
                         "(a kernel of known traffic, to scale rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--patch", type=int, default=0,
                    help="encode the workload with this patch size instead of the paper's rule "
                         "(32, 64 or 128; for the patch-size sweep)")
    ap.add_argument("--load-pipeline", action="store_true",
                    help="also time Load+Decode: the files start in pinned host memory, are copied "
                         "to the GPU on a second stream and decoded, double-buffered (the paper's "
                         "data-preparation measurement, Section 5.3, with host RAM as the source)")
    ap.add_argument("--batch", type=int, default=0, metavar="N",
                    help="cityscapes workload only: number of images per batch (default 32, the "
                         "configuration the metric is quoted on)")
    ap.add_argument("--layout", default="hwc", choices=("hwc", "chw"),
                    help="output layout of the plain decode (the headline is hwc)")
    ap.add_argument("--no-settle", action="store_true",
                    help="skip the extra untimed warm-up that waits for the clocks to settle")
    ap.add_argument("--ablation", action="store_true",
                    help="also time the decoder variants of the paper's ablation (Section 5.5): "
                         "original or custom filter, one lane or one lane per pixel for base-delta, "
                         "with and without patch-level parallelism")
    ap.add_argument("--encode", action="store_true",
                    help="also time l3_encode_batch on the same images (pixels resident in HBM) "
                         "and check its files against l3_encode_cpu's")
    ap.add_argument("--overlap-gemm", action="store_true",
                    help="also time the decode steps while a bf16 GEMM loop runs on a second "
                         "stream of default priority (Section 4.4 of the paper: decode beside "
                         "the training step's compute), and the GEMM loop alone")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (decode needs no exchange between GPUs: "
              "each GPU would decode its own shard of the batch); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2208_08711_amd as l3

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (there is no CPU fallback)")

    # one thread per host core, but never more than the 16 a one-GPU machine grants its jobs
    host_cores = os.cpu_count() or 1
    cores = min(host_cores, 16)
    images, label = make_workload(args.workload, args.batch)
    with ThreadPoolExecutor(cores) as pool:
        files = list(pool.map(lambda im: l3.encode_cpu(im, args.patch), images))
    if args.patch:
        label += " [patch size forced to %d]" % args.patch
    n = len(files)
    file_bytes = sum(len(f) for f in files)
    decoded_bytes = sum(im.size for im in images)
    compressed_over_raw = round(file_bytes / decoded_bytes, 4)

    ctx = l3.Context(0)
    infos = [l3.peek_header(f) for f in files]
    fused = args.workload == "train224"
    sets = []
    if fused:
        from paper_2208_08711_amd import synth
        crops = synth.config5_crops([(im.shape[1], im.shape[0]) for im in images])
        for s in range(args.sets):
            dfiles = [torch.from_numpy(np.frombuffer(f, dtype=np.uint8).copy()).cuda() for f in files]
            out = torch.empty((n, 3, 224, 224), dtype=torch.bfloat16, device="cuda")
            sets.append((l3.PreparedCropBatch(dfiles, infos, crops, synth.IMAGENET_MEAN,
                                              synth.IMAGENET_STD), out))

        def step(k):
            batch, out = sets[k % args.sets]
            l3.decode_crop_normalize_batch_prepared(ctx, batch, 224, 224, out, dtype=l3.BF16,
                                                    stream=stream)
    else:
        for s in range(args.sets):
            dfiles = [torch.from_numpy(np.frombuffer(f, dtype=np.uint8).copy()).cuda() for f in files]
            if args.layout == "chw":
                outs = [torch.empty((3, im.shape[0], im.shape[1]), dtype=torch.uint8, device="cuda")
                        for im in images]
                sets.append((l3.PreparedBatch(dfiles, infos, outs, layout=l3.LAYOUT_CHW), outs))
            else:
                outs = [torch.empty((im.shape[0], im.shape[1] * 3), dtype=torch.uint8, device="cuda")
                        for im in images]
                sets.append((l3.PreparedBatch(dfiles, infos, outs), outs))

        def step(k):
            l3.decode_batch_prepared(ctx, sets[k % args.sets][0], stream=stream)

    stream = torch.cuda.current_stream()
    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    # Untimed: the GPU's clocks keep rising for a few hundred launches after an idle
    # spell (the same kernel goes from 105 to 87 us over ~400 launches), so warm-up goes
    # on in blocks of 100 steps until two blocks in a row take the same time within 1 %.
    settle_steps, last = 0, None
    if not args.no_settle:
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(30):
            s0.record(stream)
            for k in range(100):
                step(k)
            s1.record(stream)
            torch.cuda.synchronize()
            settle_steps += 100
            now = s0.elapsed_time(s1)
            if last is not None and abs(now - last) <= 0.01 * last:
                break
            last = now

    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for k in range(args.steps):
        step(k)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = ev0.elapsed_time(ev1)

    # the result of the last steps must be the cropped, mirrored, normalised images
    if fused:
        got = sets[0][1].cpu()
        mean = torch.tensor(synth.IMAGENET_MEAN, dtype=torch.float32)[:, None, None]
        stdv = torch.tensor(synth.IMAGENET_STD, dtype=torch.float32)[:, None, None]
        for i in (0, n // 2, n - 1):
            x0, y0, flip = crops[i]
            win = torch.from_numpy(images[i][y0:y0 + 224, x0:x0 + 224].copy())
            if flip:
                win = win.flip(1)
            want = ((win.permute(2, 0, 1).to(torch.float32) / 255.0 - mean) / stdv).to(torch.bfloat16)
            if not torch.equal(got[i], want):
                raise SystemExit("bench.py: fused output differs from the expected tensor")
        # bytes of this path: the 16-bit tensor written; read: the header and offset arrays
        # plus the streams of the patches that intersect the window; decoded (for the
        # arithmetic count): the rows of those patches down to the window's last row
        decoded_bytes = n * 3 * 224 * 224 * 2
        file_bytes, fused_decoded = 0, 0
        for f, inf, (x0, y0, flip) in zip(files, infos, crops):
            npx, w, h = int(inf.patch), int(inf.width), int(inf.height)
            tx, ty = -(-w // npx), -(-h // npx)
            p = tx * ty
            offs = np.frombuffer(f, dtype="<u4", count=3 * p, offset=13).astype(np.int64)
            ends = np.append(offs[1:], len(f) - int(inf.header_bytes))
            file_bytes += int(inf.header_bytes)
            for j in range(y0 // npx, (y0 + 223) // npx + 1):
                rows = min(npx, h - j * npx, y0 + 224 - j * npx)
                for i in range(x0 // npx, (x0 + 223) // npx + 1):
                    k = j * tx + i
                    file_bytes += int(sum(ends[c * p + k] - offs[c * p + k] for c in range(3)))
                    fused_decoded += 3 * rows * min(npx, w - i * npx)
    else:
        for s in range(args.sets):
            for t, im in zip(sets[s][1], images):
                got = t.cpu().numpy()
                got = got.transpose(1, 2, 0) if args.layout == "chw" else got.reshape(im.shape)
                if not np.array_equal(got, im):
                    raise SystemExit("bench.py: decoded output differs from the input images")

    if args.copy_calibration:
        src = torch.ones(args.copy_calibration, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    # a plain device-to-device copy on the same stream: the practical ceiling beside the 8 TB/s
    csrc = torch.ones(1 << 28, dtype=torch.uint8, device="cuda")
    cdst = torch.empty_like(csrc)
    for _ in range(3):
        cdst.copy_(csrc)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record(stream)
    for _ in range(10):
        cdst.copy_(csrc)
    c1.record(stream)
    torch.cuda.synchronize()
    copy_gbps = 2 * csrc.numel() * 10 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del csrc, cdst

    ms_per_step = wall * 1e3 / args.steps
    launch_ms = gpu_ms / args.steps
    algo_bytes = file_bytes + decoded_bytes
    patch = int(infos[0].patch)
    counters = read_counters(args.workload)
    traffic, valu = None, None
    if counters:
        if "fetch_bytes_per_launch" in counters and "write_bytes_per_launch" in counters:
            traffic = int(counters["fetch_bytes_per_launch"]) + int(counters["write_bytes_per_launch"])
        if "sq_insts_valu_per_launch" in counters:
            insts = float(counters["sq_insts_valu_per_launch"])
            # measured wave instructions of the vector ALU against what 1024 SIMDs can issue
            # during one launch at the nominal 2.4 GHz (one instruction per SIMD per 4 cycles)
            valu = {"sq_insts_valu_per_launch": insts,
                    "issue_fraction_at_2.4GHz": insts / (VALU_ISSUE_PER_S * launch_ms * 1e-3),
                    "insts_per_256_decoded_bytes": insts / ((fused_decoded if fused else decoded_bytes) / 256.0),
                    "kernel_source_stamp": counters.get("kernel_source_stamp")}
    result = {
        "metric": "decoded images/s",
        "value": n / (ms_per_step * 1e-3),
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_steps": settle_steps,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": label, "batch": n,
                   "layout": "NCHW bf16" if fused else args.layout.upper() + " uint8",
                   "buffer_sets_rotated": args.sets,
                   "compressed_over_raw": compressed_over_raw},
        "decoded_GBps": decoded_bytes / (ms_per_step * 1e-3) / 1e9,
        "hbm_fraction": algo_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        # The fraction the target is stated in: algorithmic bytes (files read + output written)
        # per launch over the launch time (events on the launch stream) over 8 TB/s.  `traffic`
        # and `valu` come from the committed rocprofv3 counter summary of this workload and are
        # null when the kernel sources have changed since it was taken.
        "roofline": {"bound": "hbm",
                     "achieved": algo_bytes / (launch_ms * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": algo_bytes / (launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "traffic": traffic,
                     "kernel": ("l3_decode_kernel_args<%d, 4, %s, %d>" % (
                                    patch, "TENSOR" if fused else args.layout.upper(), 32 if n <= 32 else 256)
                                if n <= 256 else
                                "l3_decode_kernel<%d, 4, %s>" % (patch, "TENSOR" if fused else args.layout.upper())),
                     "launch_ms": launch_ms,
                     "algorithmic_bytes_per_launch": algo_bytes,
                     "device_copy_GBps": copy_gbps,
                     "valu": valu},
    }

    if args.overlap_gemm:
        result["overlap"] = measure_overlap(torch, step, stream, args.steps, ms_per_step)
    if args.load_pipeline and not fused:
        result["load_decode"] = measure_load_decode(torch, l3, ctx, images, files, infos, stream)
    if args.ablation and not fused:
        result["ablation"] = measure_ablation(torch, l3, ctx, images, files, infos, stream,
                                              args.patch, result["roofline"]["launch_ms"])
    if args.encode:
        result["encode"] = measure_encode(torch, l3, ctx, images, files, stream, args.patch)

    if not args.no_cpu_baseline:
        import oracle                  # the only use of the oracle here: the reported CPU baseline
        sample = files if args.workload != "imagenet" else files[:128]
        sample_bytes = sum(images[i].size for i in range(len(sample)))
        oracle.decode(sample[0])                               # warm-up
        single = sample[:max(1, len(sample) // (4 if args.workload == "imagenet" else 1))]
        t = time.perf_counter()
        for f in single:
            oracle.decode(f)
        one = (time.perf_counter() - t) / len(single)
        many = float("inf")
        with ThreadPoolExecutor(cores) as pool:
            for _ in range(3):                                 # best of three passes
                t = time.perf_counter()
                list(pool.map(oracle.decode, sample))
                many = min(many, time.perf_counter() - t)
        result["cpu_baseline"] = {
            "value": len(sample) / many, "unit": "images/s", "cores": cores, "host_cpu_count": host_cores,
            "kind": "oracle",
            "sample": f"{len(sample)} images of the same batch, best of three passes over {cores} "
                      f"threads (one image per task); single thread over {len(single)} images: "
                      f"{1.0 / one:.2f} images/s",
            "decoded_GBps": sample_bytes / many / 1e9,
            "single_thread_images_per_s": 1.0 / one,
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
