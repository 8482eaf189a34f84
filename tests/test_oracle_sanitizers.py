"""The oracle itself under AddressSanitizer and UBSan (CPU only): oracle/l3_oracle.cpp driven by
tests/native/oracle_sanitize.cpp with exact-size heap buffers, round trips on edge shapes for
every patch size, width mode and predictor, truncated and damaged files, and the crop /
normalise epilogue on windows touching every border."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-static-libasan",
                    "-I" + os.path.join(ROOT, "oracle"), "-o", exe,
                    os.path.join(HERE, "native", "oracle_sanitize.cpp"),
                    os.path.join(ROOT, "oracle", "l3_oracle.cpp")], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    word, cases = r.stdout.split()
    assert word == "ok" and int(cases) > 2000
