"""Builds ``libautobyte.so`` (HIP, gfx950) next to this file.  Run as a script or call :func:`build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libautobyte.so")
SOURCES = ["api.hip", "gemm_launch.hip", "gemm_big.hip", "scoring_kernels.hip", "update.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


HOST_SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-sanitize-recover=all", "-g"]


def _compile(src: str, objdir: str, extra=(), suffix: str = ".o") -> str:
    obj = os.path.join(objdir, src.replace(".hip", suffix))
    cmd = [HIPCC] + FLAGS + list(extra) + ["-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed on " + src)
    return obj


def build(verbose: bool = False) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=5) as ex:
        objs = list(ex.map(lambda s: _compile(s, objdir), SOURCES))
    tmp = LIB + ".tmp%d" % os.getpid()
    res = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                         capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("link failed")
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


def build_host_sanitized(verbose: bool = False) -> str:
    """``libautobyte_hostsan.so``: the translation units that hold the host-side argument checks and launch
    sequences (api.hip, update.hip, gemm_launch.hip) compiled with AddressSanitizer and
    UndefinedBehaviorSanitizer on the HOST side only (device code is compiled as always; GPU sanitizers are
    not used), linked with the ordinary objects of the kernel-only files.  For CPU-side checks of the ABI's
    error paths; a process that loads it needs clang's ASan runtime preloaded."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    plain = ["gemm_big.hip", "scoring_kernels.hip"]
    for src in plain:
        if not os.path.exists(os.path.join(objdir, src.replace(".hip", ".o"))):
            _compile(src, objdir)
    san = ["api.hip", "update.hip", "gemm_launch.hip"]
    with ThreadPoolExecutor(max_workers=3) as ex:
        objs = list(ex.map(lambda s: _compile(s, objdir, HOST_SANITIZE, ".san.o"), san))
    objs += [os.path.join(objdir, src.replace(".hip", ".o")) for src in plain]
    out = os.path.join(HERE, "libautobyte_hostsan.so")
    tmp = out + ".tmp%d" % os.getpid()
    res = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address",
                          "-fsanitize=undefined", "-shared-libsan", "-o", tmp] + objs, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("link of the host-sanitized library failed")
    os.replace(tmp, out)
    if verbose:
        print("built", out)
    return out


if __name__ == "__main__":
    build(verbose=True)
