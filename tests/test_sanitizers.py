"""AddressSanitizer + UndefinedBehaviorSanitizer build of the C oracle and of the host side of the library (every .cc
file: scheme loader and verifier, cost model, argument checks), exercised by tests/sanitize_driver.cc without a GPU.
Kernel launchers are left unresolved at link time on purpose: no checked path reaches a launch."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_06057_amd", "csrc")
GEN = os.path.join(CSRC, "generated")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_oracle_and_host_library_under_asan_and_ubsan(tmp_path):
    if not os.path.exists(os.path.join(GEN, "registry.cc")):
        from paper_2605_06057_amd.gen.generate import generate
        generate(GEN)
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-g", "-O1", "-fno-omit-frame-pointer"]
    exe = str(tmp_path / "sanitize_driver")
    oracle_o = str(tmp_path / "oracle.o")
    subprocess.check_call(["gcc", "-std=c11", "-fopenmp", "-c", os.path.join(ROOT, "oracle", "lcma_oracle.c"), "-o", oracle_o] + san)
    host = [os.path.join(CSRC, f) for f in ("api.cc", "scheme.cc", "model.cc", "unfused.cc", "fp8_api.cc", "plane_gemm.cc")]
    host.append(os.path.join(GEN, "registry.cc"))
    cmd = ["g++", "-std=c++17", "-I", CSRC, "-I", GEN, os.path.join(ROOT, "tests", "sanitize_driver.cc")] + host + [oracle_o] + san + \
          ["-fopenmp", "-static-libasan", "-Wl,--unresolved-symbols=ignore-all", "-o", exe]
    subprocess.check_call(cmd)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    r = subprocess.run([exe, str(tmp_path)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitize driver ok" in r.stdout
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr
