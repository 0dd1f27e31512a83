"""Builds libpurekv.so (HIP, gfx950 only) in-tree with hipcc.  Run as `python -m paper_2510_25600_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libpurekv.so")
SOURCES = ["api.hip", "plan.cpp", "prefill.hip", "importance.hip", "select.hip", "compact.hip", "decode.hip", "rank.hip", "calib.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build_library(verbose: bool = True) -> str:
    """Compiles every source and links the shared library; always recompiles."""
    objs = []
    build_dir = os.path.join(HERE, "_build")
    os.makedirs(build_dir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(build_dir, src.rsplit(".", 1)[0] + ".o")
        objs.append(obj)
        cmd = [HIPCC, *FLAGS, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n{out}", file=sys.stderr)
        elif verbose and out.strip():
            print(f"[build] {src}:\n{out}")
    if failed:
        raise RuntimeError("hipcc failed")
    link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH]
    subprocess.run(link, check=True)
    if verbose:
        print(f"[build] wrote {LIB_PATH}")
    return LIB_PATH


def build_host_sanitized(verbose: bool = True) -> str:
    """Host code under AddressSanitizer + UndefinedBehaviorSanitizer: rebuilds the planner (plan.cpp) and the C ABI's
    host half (api.hip: validation, plan life cycle, inspection) with the sanitizers on the HOST side only, links
    them with the library's other objects (built if missing) into _build/san/libpurekv_san.so, and builds
    tests/host_sanitizer_driver.cpp against it.  Returns the path of the driver executable; it needs no GPU.
        python -m paper_2510_25600_amd.build --sanitize && paper_2510_25600_amd/_build/san/host_sanitizer_driver"""
    build_dir = os.path.join(HERE, "_build")
    san_dir = os.path.join(build_dir, "san")
    os.makedirs(san_dir, exist_ok=True)
    others = [s for s in SOURCES if s not in ("api.hip", "plan.cpp")]
    if not all(os.path.exists(os.path.join(build_dir, s.rsplit(".", 1)[0] + ".o")) for s in others):
        build_library(verbose=False)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    objs = [os.path.join(build_dir, s.rsplit(".", 1)[0] + ".o") for s in others]
    procs = []
    for src in ("api.hip", "plan.cpp"):
        obj = os.path.join(san_dir, src.rsplit(".", 1)[0] + ".o")
        objs.append(obj)
        cmd = [HIPCC, *FLAGS, *san, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, pr in procs:
        out, _ = pr.communicate()
        if pr.returncode != 0:
            raise RuntimeError(f"sanitized build of {src} failed:\n{out}")
    lib = os.path.join(san_dir, "libpurekv_san.so")
    clangxx = os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "lib", "llvm", "bin", "clang++")
    if not os.path.exists(clangxx):
        clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    rt_dir = os.path.dirname(subprocess.check_output([clangxx, "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip())
    host_san = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-shared-libsan",
                f"-Wl,-rpath,{rt_dir}"]
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *host_san, *objs, "-o", lib], check=True)
    exe = os.path.join(san_dir, "host_sanitizer_driver")
    subprocess.run([clangxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", *host_san, "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), lib, f"-Wl,-rpath,{san_dir}", "-o", exe],
                   check=True)
    if verbose:
        print(f"[build] wrote {lib} and {exe}")
    return exe


if __name__ == "__main__":
    if "--sanitize" in sys.argv:
        build_host_sanitized()
    else:
        build_library()
