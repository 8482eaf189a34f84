"""The decode kernels' own source (paper_2208_08711_amd/csrc/l3_device.hip with its host
planning) compiled for the host and run on host threads, one per GPU thread
(tests/native/kernel_cpu), under AddressSanitizer + UBSan and under ThreadSanitizer, on ragged
shapes of every patch size, layout and the fused path: every byte against the oracle, every
buffer of exactly the promised size (so an access outside one ends the run), every pair of
accesses to LDS ordered by a barrier.  No GPU; the same cases run on the GPU in
tests/test_gpu_parity.py."""
import os
import struct
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import oracle
from paper_2208_08711_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/llvm/bin/clang++"
SOURCES = [os.path.join(ROOT, "tests", "native", "kernel_cpu", "kernel_cpu_main.cpp"),
           os.path.join(ROOT, "paper_2208_08711_amd", "csrc", "l3_host.cpp")]
MEAN, STD = synth.IMAGENET_MEAN, synth.IMAGENET_STD


def build(tmp, name, flags, kernel_source=None):
    exe = os.path.join(tmp, name)
    if kernel_source:
        flags = [*flags, f'-DL3_KERNEL_SOURCE="{kernel_source}"']
    subprocess.run([CLANG, "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-pthread", *flags,
                    "-I", os.path.join(ROOT, "tests", "native", "kernel_cpu"),
                    "-I", os.path.join(ROOT, "include"),
                    "-I", os.path.join(ROOT, "paper_2208_08711_amd", "csrc"),
                    "-x", "c++", *SOURCES, "-o", exe], check=True)
    return exe


@pytest.fixture(scope="module")
def exes(tmp_path_factory):
    if not os.path.exists(CLANG):
        pytest.skip("no clang++ with sanitizer runtimes")
    tmp = str(tmp_path_factory.mktemp("kernel_cpu"))
    with ThreadPoolExecutor(2) as pool:      # the two builds side by side
        asan = pool.submit(build, tmp, "kernel_cpu_asan", ["-fsanitize=address,undefined",
                                                            "-fno-sanitize-recover=undefined"])
        tsan = pool.submit(build, tmp, "kernel_cpu_tsan", ["-fsanitize=thread"])
        return {"asan": asan.result(), "tsan": tsan.result(), "tmp": tmp}


def write_case(path, mode, images, patch, crops=None, crop=(0, 0), dtype=0, pad_cols=5):
    """mode 0: interleaved, 1: planar, 2: fused call, 3: the fused call that allocates nothing."""
    files = [oracle.encode(im, patch) for im in images]
    with open(path, "wb") as f:
        f.write(struct.pack("<5I3f3f2I", 0x434B334C, mode, len(images), crop[0], crop[1], *MEAN, *STD,
                            dtype, pad_cols))
        tensor = []
        for k, (im, fl) in enumerate(zip(images, files)):
            assert np.array_equal(oracle.decode(fl), im)
            f.write(struct.pack("<Q", len(fl)))
            f.write(fl)
            x0, y0, flip = crops[k] if crops else (0, 0, 0)
            f.write(struct.pack("<iiI", x0, y0, flip))
            if mode == 0:
                want = im.tobytes()
            elif mode == 1:
                want = np.ascontiguousarray(im.transpose(2, 0, 1)).tobytes()
            else:
                tensor.append(oracle.crop_normalize(im, x0, y0, flip, crop[0], crop[1], MEAN, STD, dtype))
                continue
            f.write(struct.pack("<Q", len(want)))
            f.write(want)
        if mode >= 2:
            want = np.stack(tensor).astype(np.uint16).tobytes()
            f.write(struct.pack("<Q", len(want)))
            f.write(want)


def execute(exe, case):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               TSAN_OPTIONS="halt_on_error=1")
    return subprocess.run([exe, case], capture_output=True, text=True, env=env, timeout=900)


def run(exe, case):
    r = execute(exe, case)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert r.stdout.startswith("ok"), r.stdout


SHAPES = [(1, 1), (2, 1), (3, 5), (5, 3), (33, 31), (63, 65), (65, 34), (130, 40), (257, 9), (129, 66)]


def ragged_images(seed):
    out = []
    for k, (w, h) in enumerate(SHAPES):
        out.append(synth.cosine_field(seed + k, w, h) if k % 2 else synth.uniform_bytes(seed + k, w, h))
    return out


@pytest.mark.parametrize("patch", [32, 64, 128])
@pytest.mark.parametrize("mode", [0, 1])
def test_pixel_modes_under_address_and_ub_sanitizers(exes, patch, mode):
    case = os.path.join(exes["tmp"], f"px_{patch}_{mode}.bin")
    write_case(case, mode, ragged_images(900 + patch), patch)
    run(exes["asan"], case)


@pytest.mark.parametrize("patch", [32, 64, 128])
def test_fused_path_under_address_and_ub_sanitizers(exes, patch):
    images = [synth.cosine_field(40 + k, 70 + 9 * k, 50 + 7 * k) for k in range(4)]
    crops = [(0, 0, 0), (7, 3, 1), (79 - 40, 57 - 33, 0), (31, 17, 1)]
    for mode, dtype in ((2, 0), (3, 1)):
        case = os.path.join(exes["tmp"], f"fused_{patch}_{mode}.bin")
        write_case(case, mode, images, patch, crops=crops, crop=(40, 33), dtype=dtype)
        run(exes["asan"], case)


def test_more_than_256_images_go_through_the_descriptor_table(exes):
    images = [synth.uniform_bytes(3000 + k, 1 + k % 7, 1 + k % 5) for k in range(260)]
    case = os.path.join(exes["tmp"], "many.bin")
    write_case(case, 0, images, 32)
    run(exes["asan"], case)
    # the fused kernel of that kind takes its descriptors from the table in device memory and
    # its normalised values from the tail of its arguments
    images = [synth.uniform_bytes(3100 + k, 20 + k % 7, 18 + k % 5) for k in range(260)]
    case = os.path.join(exes["tmp"], "many_fused.bin")
    write_case(case, 2, images, 32, crops=[(k % 5, k % 3, k & 1) for k in range(260)], crop=(16, 15))
    run(exes["asan"], case)


@pytest.mark.parametrize("patch,mode", [(32, 0), (64, 0), (128, 0), (128, 1), (32, 2)])
def test_lds_protocol_under_thread_sanitizer(exes, patch, mode):
    """Rings, parked rows and the table are handed between waves through LDS with one workgroup
    barrier per period and wave-level fences: ThreadSanitizer sees every access of every lane."""
    images = [synth.cosine_field(70, 140, 75), synth.uniform_bytes(71, 66, 40)]
    case = os.path.join(exes["tmp"], f"tsan_{patch}_{mode}.bin")
    if mode == 2:
        write_case(case, 2, images, patch, crops=[(10, 5, 1), (3, 2, 0)], crop=(50, 30))
    else:
        write_case(case, mode, images, patch)
    run(exes["tsan"], case)


def test_planted_mistakes_are_seen(exes):
    """The tool has teeth: copies of the kernel source with one mistake each -- a granule
    fetched beyond the stream's last one, the period's barrier left out, a store one word too
    far -- are built the same way, and each run ends in the report that names the mistake (an
    access outside a buffer, a data race, a byte that differs from the oracle's)."""
    src = open(os.path.join(ROOT, "paper_2208_08711_amd", "csrc", "l3_device.hip")).read()
    images = [synth.cosine_field(70, 140, 75), synth.uniform_bytes(71, 66, 40)]
    case = os.path.join(exes["tmp"], "planted.bin")
    write_case(case, 0, images, 64)
    plants = [
        ("overread", "asan", "if (at < limit) v =", "if (at < limit + 32) v =", "heap-buffer-overflow"),
        ("nobarrier", "tsan", "are parked: write them out */\n            __syncthreads();",
         "are parked: write them out */", "data race"),
        ("overwrite", "asan", "reinterpret_cast<global_u32x3_any*>(row + column)",
         "reinterpret_cast<global_u32x3_any*>(row + column + 4)", "MISMATCH"),
    ]
    def build_plant(plant):
        name, kind, old, new, report = plant
        assert src.count(old) == 1, name
        path = os.path.join(exes["tmp"], f"l3_device_{name}.hip")
        with open(path, "w") as f:
            f.write(src.replace(old, new))
        flags = (["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"] if kind == "asan"
                 else ["-fsanitize=thread"])
        return build(exes["tmp"], f"kernel_cpu_{name}", flags, kernel_source=path)

    with ThreadPoolExecutor(3) as pool:
        built = list(pool.map(build_plant, plants))
    for (name, kind, old, new, report), exe in zip(plants, built):
        r = execute(exe, case)
        assert r.returncode != 0 and report in r.stderr, (name, r.returncode, r.stderr[-1500:])
