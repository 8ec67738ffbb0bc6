"""Builds liblava.so (the HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2509_09754_amd.build              the library the tests and benchmarks load
    python -m paper_2509_09754_amd.build --sanitize   _build/liblava_san.so: the same sources with the HOST
                                                      side under AddressSanitizer + UBSan (device code is
                                                      built as usual); load it by pointing LAVA_LIBRARY at it,
                                                      with the sanitizer runtime this prints preloaded

Objects go to _build/ (ignored by git); the shared library lands next to this file so that it
travels with the source tree.  hipcc cross-compiles without a GPU present.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD_DIR = os.path.join(ROOT, "_build")
LIB_PATH = os.path.join(HERE, "liblava.so")

SOURCES = ["lava_api.hip", "k_sweep.hip", "k_select.hip", "k_compact.hip", "k_budgets.hip", "k_decode.hip", "k_probe.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # packed-FP32 VALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA results go straight to VGPRs (no v_accvgpr_read per accumulator element in the epilogues)
    "-mllvm", "-amdgpu-mfma-vgpr-form",
]


def _compile(src: str, extra: list[str], suffix: str = "") -> str:
    obj = os.path.join(BUILD_DIR, os.path.splitext(src)[0] + suffix + ".o")
    cmd = [HIPCC, *COMMON_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


# host-side sanitizers: every -fsanitize= sits directly behind an -Xarch_host, so the device pass never sees it
SANITIZE_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                  "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
SAN_LIB_PATH = os.path.join(BUILD_DIR, "liblava_san.so")


def build_library(extra_flags: list[str] | None = None, verbose: bool = True, sanitize: bool = False) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    extra = list(extra_flags or [])
    out, suffix = LIB_PATH, ""
    if sanitize:
        extra += SANITIZE_FLAGS
        out, suffix = SAN_LIB_PATH, ".san"
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(lambda s: _compile(s, extra, suffix), SOURCES))
    link_extra = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                  "-shared-libsan"] if sanitize else []
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *link_extra, *objs, "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    if verbose:
        print(f"built {out}")
        if sanitize:
            print("run with: LD_PRELOAD=" + sanitizer_runtime() + " LAVA_LIBRARY=" + out +
                  " ASAN_OPTIONS=detect_leaks=0 python -m pytest tests/test_boundary.py -q")
    return out


def sanitizer_runtime() -> str:
    """The shared AddressSanitizer runtime of the compiler that built the library (to be preloaded into python)."""
    res = subprocess.run([HIPCC, "--print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = res.stdout.strip()
    if not os.path.isabs(path):
        res = subprocess.run(["/opt/rocm/lib/llvm/bin/clang", "--print-file-name=libclang_rt.asan-x86_64.so"],
                             capture_output=True, text=True)
        path = res.stdout.strip()
    return path


if __name__ == "__main__":
    args = sys.argv[1:]
    san = "--sanitize" in args
    build_library([a for a in args if a != "--sanitize"], sanitize=san)
