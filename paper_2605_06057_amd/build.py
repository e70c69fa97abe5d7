"""Builds liblcma.so: runs the kernel generator, compiles every translation unit for gfx950
with hipcc and links them.  Usage: python -m paper_2605_06057_amd.build [--force] [-j N]"""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys
import time

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
GEN = os.path.join(CSRC, "generated")
LIB = os.path.join(PKG, "liblcma.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-I", CSRC, "-I", GEN, "-Wno-unused-command-line-argument"]
COMMON += os.environ.get("LCMA_EXTRA_FLAGS", "").split()  # e.g. -D switches of timing experiments


def _newer(target: str, deps: list[str]) -> bool:
    if not os.path.exists(target):
        return False
    t = os.path.getmtime(target)
    return all(os.path.getmtime(d) <= t for d in deps)


def _compile(src: str, obj: str, deps: list[str], force: bool) -> str:
    if not force and _newer(obj, [src] + deps):
        return f"up to date  {os.path.basename(src)}"
    t0 = time.time()
    flags = COMMON + (DEVICE_FLAGS if src.endswith(".hip") else ["-x", "c++"])
    cmd = [HIPCC] + flags + ["-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "is not a recognized feature" not in l)
    if r.returncode:
        raise RuntimeError(f"{' '.join(cmd)}\n{err}")
    return f"compiled {time.time() - t0:5.1f}s  {os.path.basename(src)}" + (("\n" + err) if err.strip() else "")


def build(force: bool = False, jobs: int | None = None, verbose: bool = True) -> str:
    from .gen.generate import generate

    hips = generate(GEN)
    headers = [os.path.join(CSRC, h) for h in ("lcma_device.hpp", "lcma_prepare_b.hpp", "lcma_combine_h.hpp", "lcma_params.h", "host_common.h", "lcma_fp8.hpp", "lcma_plane_gemm.hpp")]
    headers.append(os.path.join(PKG, "..", "include", "lcma.h"))
    headers.append(os.path.join(GEN, "builtin_schemes.inc"))
    units = [(h, h[:-4] + ".o") for h in hips]
    for name in ("api.cc", "scheme.cc", "model.cc", "unfused.cc", "lcma_aux.hip", "lcma_static.hip", "lcma_fp8.hip", "fp8_api.cc", "lcma_plane_gemm.hip", "plane_gemm.cc"):
        units.append((os.path.join(CSRC, name), os.path.join(GEN, os.path.splitext(name)[0] + ".o")))
    units.append((os.path.join(GEN, "registry.cc"), os.path.join(GEN, "registry.o")))
    jobs = jobs or min(8, os.cpu_count() or 1)
    with cf.ThreadPoolExecutor(jobs) as ex:
        for msg in ex.map(lambda u: _compile(u[0], u[1], headers, force), units):
            if verbose:
                print(msg, flush=True)
    objs = [o for _, o in units]
    if force or not _newer(LIB, objs):
        tmp = LIB + f".tmp{os.getpid()}"
        subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs)
        os.replace(tmp, LIB)
        if verbose:
            print(f"linked {LIB}", flush=True)
    return LIB


if __name__ == "__main__":
    j = None
    if "-j" in sys.argv:
        j = int(sys.argv[sys.argv.index("-j") + 1])
    build(force="--force" in sys.argv, jobs=j)
