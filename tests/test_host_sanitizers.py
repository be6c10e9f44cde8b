"""AddressSanitizer + UndefinedBehaviorSanitizer build of the code that does index
arithmetic on caller arrays on the host: the library's host logic
(csrc/host_logic.cpp: planners, replica lists, coverage, tiling) and the C oracle,
driven by tests/host_fuzz.cpp on thousands of random instances.  CPU only; the
sanitizers cover host code (the GPU pass is compiled without them)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]


@pytest.mark.skipif(not (os.path.exists(HIPCC) and shutil.which("gcc")), reason="needs hipcc and gcc")
def test_host_logic_and_oracle_under_asan_ubsan(tmp_path):
    oracle_o = tmp_path / "eep_oracle.o"
    subprocess.run(["gcc", "-std=c99", "-O1", "-g", "-ffp-contract=off", *SAN, "-c",
                    os.path.join(ROOT, "oracle", "eep_oracle.c"), "-o", str(oracle_o)], check=True)
    exe = tmp_path / "host_fuzz"
    objs = [str(oracle_o)]
    for src in (os.path.join(ROOT, "paper_2605_10670_amd", "csrc", "host_logic.cpp"),
                os.path.join(ROOT, "tests", "host_fuzz.cpp")):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-std=c++17", "-O1", "-g", *SAN,
                        "-fno-gpu-sanitize", "-I", os.path.join(ROOT, "include"),
                        "-I", os.path.join(ROOT, "paper_2605_10670_amd", "csrc"), "-c", src,
                        "-o", obj], check=True)
        objs.append(obj)
    subprocess.run([HIPCC, *SAN, "-fno-gpu-sanitize", *objs, "-lm", "-o", str(exe)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe), "4000"], env=env, capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert run.stdout.strip().endswith("ok 4000")
