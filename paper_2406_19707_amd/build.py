"""Builds libinfinigen_hip.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libinfinigen_hip.so")
SOURCES = ["ig_api.hip", "k_scan.hip", "k_project.hip", "k_kv.hip", "k_layer.hip", "k_equalize.hip", "k_index.hip", "k_skew.hip", "ig_host.cpp"]
HIPCC = "/opt/rocm/bin/hipcc"
# packed-fp32 instruction selection is switched off for every device compile
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if src.endswith(".hip"):
        cmd = [HIPCC, *COMMON, *DEVICE_FLAGS, "-c", path, "-o", obj]
    else:
        cmd = [HIPCC, *COMMON, "-x", "c++", "-c", path, "-o", obj]
    subprocess.check_call(cmd)
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs])
    if verbose:
        print("built", LIB)
    return LIB


HOST_SANITIZED = ["ig_api.hip", "ig_host.cpp"]      # the files whose host code checks and computes


def sanitizer_runtime() -> str:
    """Path of the shared AddressSanitizer runtime of hipcc's clang (to be preloaded by a process
    that loads the host-sanitized library)."""
    clang = subprocess.check_output([HIPCC, "--hip-path=/opt/rocm", "-print-file-name=libclang_rt.asan-x86_64.so"],
                                    text=True).strip()
    if os.path.isabs(clang) and os.path.exists(clang):
        return clang
    import glob
    hits = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not hits:
        raise FileNotFoundError("libclang_rt.asan-x86_64.so not found under /opt/rocm")
    return hits[-1]


def build_host_sanitized(out_dir: str) -> str:
    """Second copy of the library whose HOST code (argument checks, offline skewing, partial index,
    CPU-side speculation) is instrumented with AddressSanitizer and UndefinedBehaviorSanitizer;
    device code and the kernel launch files are the ordinary objects of build().  For the CPU test
    suite only."""
    os.makedirs(out_dir, exist_ok=True)
    san = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
    objs = []
    for src in SOURCES:
        plain = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
        if src not in HOST_SANITIZED:
            if not os.path.exists(plain):
                _compile(src)
            objs.append(plain)
            continue
        obj = os.path.join(out_dir, os.path.splitext(src)[0] + ".o")
        path = os.path.join(CSRC, src)
        if src.endswith(".hip"):
            host = [f for flag in san for f in ("-Xarch_host", flag)]
            cmd = [HIPCC, "-O1", "-g", *COMMON[1:], *DEVICE_FLAGS, *host, "-c", path, "-o", obj]
        else:
            cmd = [HIPCC, "-O1", "-g", *COMMON[1:], *san, "-x", "c++", "-c", path, "-o", obj]
        subprocess.check_call(cmd)
        objs.append(obj)
    lib = os.path.join(out_dir, "libinfinigen_hip.so")
    subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-shared-libsan", *san, "-o", lib, *objs])
    return lib


if __name__ == "__main__":
    build(verbose=True)
