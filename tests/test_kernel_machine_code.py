"""The decode kernels as compiled: hipcc's gfx950 machine code (text, `-S`, the library's own
flags) is run by an interpreter on the CPU (tests/native/isa_interp/interp.py) for launches
recorded by the host build of the same source (tests/native/kernel_cpu): every global access
inside the launch's buffers, every LDS access aligned and inside the workgroup's allocation,
every buffer afterwards identical to the host build's, which the harness has compared with the
oracle.  And in the optimised IR every loop of every decode kernel still has a way out.  (A
kernel can be right as source and wrong as compiled; these are the checks for that.)  No GPU."""
import os
import re
import struct
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2208_08711_amd import synth

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import test_kernel_cpu_build as host_build   # noqa: E402  (case writer, harness build)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
DEVICE_SOURCE = os.path.join(ROOT, "paper_2208_08711_amd", "csrc", "l3_device.hip")
INTERP = os.path.join(ROOT, "tests", "native", "isa_interp", "interp.py")
# the library's flags (paper_2208_08711_amd/build.py), device side only
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off", "-Xclang", "-target-feature",
         "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2208_08711_amd", "csrc"),
         "-x", "hip", DEVICE_SOURCE, "--cuda-device-only"]


@pytest.fixture(scope="module")
def built(tmp_path_factory):
    if not os.path.exists(HIPCC) or not os.path.exists(host_build.CLANG):
        pytest.skip("needs hipcc and clang++")
    tmp = str(tmp_path_factory.mktemp("machine_code"))
    asm, ir = os.path.join(tmp, "l3_device.s"), os.path.join(tmp, "l3_device.ll")
    with ThreadPoolExecutor(3) as pool:      # the three builds side by side
        jobs = [pool.submit(subprocess.run, [HIPCC, *FLAGS, "-S", "-o", asm], check=True),
                pool.submit(subprocess.run, [HIPCC, *FLAGS, "-emit-llvm", "-S", "-o", ir], check=True),
                pool.submit(host_build.build, tmp, "kernel_cpu_plain", [])]
        harness = [j.result() for j in jobs][2]
    return {"tmp": tmp, "asm": open(asm).read(), "ir": open(ir).read(), "harness": harness}


def kernel_text(asm, n, mode, kind):
    if kind == 0:
        name = "_ZN12_GLOBAL__N_116l3_decode_kernelILi%dELi4ELi%dEEE" % (n, mode)
    else:
        name = "_ZN12_GLOBAL__N_121l3_decode_kernel_argsILi%dELi4ELi%dELi%dEEE" % (n, mode, 32 if kind == 1 else 256)
    m = re.search(r"^" + re.escape(name) + r"\S*: +; @", asm, flags=re.M)
    assert m, name
    return asm[m.start():asm.index(".end_amdhsa_kernel", m.start())]


def record_and_interpret(built, tag, mode, images, patch, **kw):
    rec = os.path.join(built["tmp"], tag)
    os.makedirs(rec)
    case = os.path.join(rec, "case.bin")
    host_build.write_case(case, mode, images, patch, **kw)
    r = subprocess.run([built["harness"], case], capture_output=True, text=True, timeout=600,
                       env=dict(os.environ, L3CPU_RECORD=rec))
    assert r.returncode == 0 and r.stdout.startswith("ok"), (r.stdout, r.stderr[-2000:])
    launches = sorted(f for f in os.listdir(rec) if f.startswith("launch_"))
    assert launches
    out = []
    for name in launches:
        path = os.path.join(rec, name)
        n, kmode, kind = struct.unpack("<3i", open(path, "rb").read(12))
        text = os.path.join(rec, name + ".s")
        with open(text, "w") as f:
            f.write(kernel_text(built["asm"], n, kmode, kind))
        r = subprocess.run([sys.executable, INTERP, text, path, os.path.join(rec, "after.bin")],
                           capture_output=True, text=True, timeout=900)
        assert r.returncode == 0, (tag, name, r.stdout[-1500:], r.stderr[-1500:])
        assert "buffers that differ from the host build's: 0 of" in r.stdout, r.stdout[-500:]
        assert "LDS accesses out of range: 0" in r.stdout
        out.append((path, text))
    return out


def small_images(seed):
    return [synth.cosine_field(seed, 70, 37), synth.uniform_bytes(seed + 1, 33, 66), synth.uniform_bytes(seed + 2, 5, 3)]


@pytest.mark.parametrize("patch", [32, 64, 128])
@pytest.mark.parametrize("mode", [0, 1])
def test_pixel_kernels_as_compiled(built, patch, mode):
    record_and_interpret(built, f"px_{patch}_{mode}", mode, small_images(300 + patch), patch)


@pytest.mark.parametrize("patch,dtype", [(32, 0), (64, 1)])
def test_fused_kernels_as_compiled(built, patch, dtype):
    images = [synth.cosine_field(50 + k, 70 + 9 * k, 50 + 7 * k) for k in range(2)]
    record_and_interpret(built, f"fused_{patch}", 2, images, patch, crops=[(7, 3, 1), (20, 11, 0)],
                         crop=(40, 33), dtype=dtype)


def test_descriptor_table_kernel_as_compiled_and_a_short_buffer_is_seen(built):
    """More than 256 images go through the kernel that reads descriptors from device memory.  The
    same recorded launch with one file's buffer cut short by its last granule must end in the
    interpreter's report of the load that leaves the buffer: the bounds check has teeth."""
    images = [synth.uniform_bytes(3000 + k, 1 + k % 3, 1 + k % 2) for k in range(257)]
    (launch, text), = record_and_interpret(built, "table", 0, images, 32)
    blob = open(launch, "rb").read()
    (kn,) = struct.unpack_from("<Q", blob, 24)
    at = 32 + kn
    (count,) = struct.unpack_from("<Q", blob, at)
    at += 8
    out, cut = [blob[:at]], False
    for _ in range(count):
        addr, n = struct.unpack_from("<QQ", blob, at)
        data = blob[at + 16:at + 16 + n]
        at += 16 + n
        if not cut and 32 <= n <= 64 and n % 16 == 0 and data[:4] != b"\xa5\xa5\xa5\xa5" and b"L3\x00\x01" in data[:20]:
            n -= 16
            data = data[:n]
            cut = True
        out.append(struct.pack("<QQ", addr, n) + data)
    assert cut
    short = launch + ".short"
    with open(short, "wb") as f:
        f.write(b"".join(out))
    r = subprocess.run([sys.executable, INTERP, text, short], capture_output=True, text=True, timeout=900)
    assert r.returncode != 0 and "outside every buffer" in r.stdout, r.stdout[-800:]


def test_every_loop_of_every_decode_kernel_keeps_an_exit(built):
    """In the optimised IR of each decode kernel, every loop (every back edge's natural loop) has
    an edge that leaves it.  A loop that lost its exit test in the optimiser runs past its bound
    on the GPU and writes rows that do not exist."""
    lines = built["ir"].split("\n")
    seen = 0
    k = 0
    while k < len(lines):
        if lines[k].startswith("define") and "l3_decode_kernel" in lines[k]:
            name = re.search(r"@(\S+?)\(", lines[k]).group(1)
            j = k
            while lines[j] != "}":
                j += 1
            blocks, cur = {}, None
            for line in lines[k:j + 1]:
                m = re.match(r"^(\d+):", line)
                if m:
                    cur = int(m.group(1))
                    blocks[cur] = []
                elif cur is not None:
                    blocks[cur].append(line)
            succ = {}
            for b, ls in blocks.items():
                term = [x for x in ls if x.strip().startswith(("br ", "ret", "switch", "unreachable"))]
                succ[b] = [int(x) for x in re.findall(r"label %(\d+)", term[-1])] if term else []
            pred = {}
            for b, ss in succ.items():
                for s in ss:
                    pred.setdefault(s, []).append(b)
            for b, ss in succ.items():
                for h in ss:
                    if h <= b:          # a back edge: blocks are numbered in layout order
                        loop, stack = {h}, [b]
                        while stack:
                            x = stack.pop()
                            if x not in loop:
                                loop.add(x)
                                stack += pred.get(x, [])
                        assert any(s not in loop for x in loop for s in succ[x]), (name, h, b)
                        seen += 1
            k = j
        k += 1
    assert seen >= 27 * 2    # 27 kernels, each with at least the period loop and the status loop
