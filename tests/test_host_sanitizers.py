"""The library's host code under AddressSanitizer and UBSan (CPU only): the CPU
encoders, the encode bound and the header validator of
paper_2208_08711_amd/csrc/l3_host.cpp, driven by tests/native/host_sanitize.cpp with
exact-size heap buffers, truncated files and damaged headers."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-static-libasan",
                    "-I" + os.path.join(ROOT, "include"),
                    "-I" + os.path.join(ROOT, "paper_2208_08711_amd", "csrc"), "-o", exe,
                    os.path.join(HERE, "native", "host_sanitize.cpp"),
                    os.path.join(ROOT, "paper_2208_08711_amd", "csrc", "l3_host.cpp")], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    word, cases = r.stdout.split()
    assert word == "ok" and int(cases) > 100000
