"""Build libng.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2410_16029_amd.build`."""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libng.so")
SOURCES = ["ng_api.hip", "k_elementwise.hip", "k_gemm_f32.hip", "k_gemm_bf16.hip", "k_refresh.hip", "k_skinny.hip",
           "k_microbench.hip"]

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def source_hash() -> str:
    """Hash of everything the library is compiled from (kernel sources, internal and public headers)."""
    import hashlib

    h = hashlib.sha256()
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h")))
    files.append(os.path.join(ROOT, "include", "ng.h"))
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def built_hash():
    """source_hash() as it was when libng.so was last built here, or None."""
    try:
        return open(os.path.join(HERE, "_build", "source_hash.txt")).read().strip()
    except OSError:
        return None


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _compile(src: str, objdir: str, extra) -> str:
    obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, res.stdout, res.stderr))
    return obj


def build(verbose: bool = True, extra=()) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, objdir, list(extra)), SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (res.stdout, res.stderr))
    with open(os.path.join(objdir, "source_hash.txt"), "w") as f:
        f.write(source_hash() + "\n")
    if verbose:
        print("built", LIB)
    return LIB


def build_host_sanitizer(verbose: bool = True) -> str:
    """The library with AddressSanitizer + UndefinedBehaviorSanitizer on its HOST side (the device code is
    compiled as usual), linked with tests/host/abi_driver.cpp into one executable: the host scheduler's
    validation, planning and bookkeeping under the sanitizers, no GPU needed.  Returns the executable."""
    objdir = os.path.join(HERE, "_build", "asan")
    os.makedirs(objdir, exist_ok=True)
    san = ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, objdir, san), SOURCES))
    exe = os.path.join(objdir, "abi_driver")
    driver = os.path.join(ROOT, "tests", "host", "abi_driver.cpp")
    cmd = [_hipcc(), "--offload-arch=gfx950", "-std=c++17", "-O1", "-g", "-fno-gpu-sanitize", "-fsanitize=address",
           "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-I" + os.path.join(ROOT, "include"),
           # the driver also sees the internal header, as plain C++
           "-I" + CSRC, "-D__HIP_PLATFORM_AMD__",
           "-I" + os.path.join(os.path.dirname(os.path.dirname(os.path.realpath(_hipcc()))), "include"),
           "-x", "c++", driver, "-x", "none", *objs, "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("sanitizer link failed:\n%s\n%s" % (res.stdout, res.stderr))
    if verbose:
        print("built", exe)
    return exe


if __name__ == "__main__":
    if sys.argv[1:] == ["--host-sanitizer"]:
        build_host_sanitizer()
    else:
        build(extra=sys.argv[1:])
