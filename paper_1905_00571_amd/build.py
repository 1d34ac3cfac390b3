"""Builds paper_1905_00571_amd/libcadnn.so from csrc/ with hipcc for gfx950.

`python -m paper_1905_00571_amd.build` (or `__graft_entry__.build()`) compiles every
translation unit and links the shared library in-tree.  Objects are cached under
`_build/` keyed by source mtime unless force=True.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")
OBJDIR = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libcadnn.so")

SOURCES = ["pack.cpp", "api.cpp", "net.cpp", "conv_tile.hip", "conv_direct.hip", "conv_linear.hip", "conv_quad.hip", "conv_stile.hip", "conv_ptile.hip", "conv_wtile.hip", "conv_depthwise.hip", "misc_kernels.hip", "dense_conv.hip", "dense_wide.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I", INCLUDE, "-I", CSRC,
]


def _newer(a: str, deps) -> bool:
    if not os.path.exists(a):
        return False
    t = os.path.getmtime(a)
    return all(os.path.getmtime(d) <= t for d in deps)


# Host-code sanitizers (the device code is compiled as always): each -fsanitize= directly
# after -Xarch_host, so that only the host pass sees it.
ASAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
              "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
ASAN_OBJDIR = os.path.join(OBJDIR, "asan")
ASAN_LIB = os.path.join(ASAN_OBJDIR, "libcadnn_asan.so")


def _compile(src: str, force: bool, asan: bool = False) -> str:
    path = os.path.join(CSRC, src)
    obj = os.path.join(ASAN_OBJDIR if asan else OBJDIR, src + ".o")
    deps = [path, os.path.join(CSRC, "internal.h"), os.path.join(INCLUDE, "cadnn.h")]
    if not force and _newer(obj, deps):
        return obj
    cmd = [HIPCC, "-x", "hip", "-c", path, "-o", obj] + FLAGS + (ASAN_FLAGS if asan else [])
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out.strip():
        sys.stderr.write(out + "\n")
    return obj


def build(force: bool = True, jobs: int = 6) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    os.replace(tmp, LIB)
    return LIB


def asan_runtime() -> str:
    """The shared AddressSanitizer runtime of the compiler that built the library (a process
    that loads the instrumented library must have it loaded first)."""
    r = subprocess.run([HIPCC, "--print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = r.stdout.strip()
    if not os.path.isabs(path):
        clang = os.path.join(os.path.dirname(os.path.dirname(HIPCC)), "lib", "llvm", "bin", "clang")
        r = subprocess.run([clang, "--print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
        path = r.stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else ""


def build_asan(force: bool = False, jobs: int = 6) -> str:
    """The same library with AddressSanitizer and UndefinedBehaviorSanitizer on its HOST code
    (packer, plan builders, net layout: index arithmetic that runs without a GPU), as
    _build/asan/libcadnn_asan.so.  CADNN_LIB_PATH makes the binding load it; the process needs
    the runtime preloaded (asan_runtime())."""
    os.makedirs(ASAN_OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, True), SOURCES))
    tmp = ASAN_LIB + f".tmp{os.getpid()}"
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-shared-libsan", "-fsanitize=address",
           "-fsanitize=undefined", "-o", tmp] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    os.replace(tmp, ASAN_LIB)
    return ASAN_LIB


if __name__ == "__main__":
    if "--asan" in sys.argv:
        print(build_asan(force="--incremental" not in sys.argv))
        print("runtime:", asan_runtime())
    else:
        print(build(force="--incremental" not in sys.argv))
