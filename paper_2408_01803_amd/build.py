"""Builds libstb.so (host packer + gfx950 kernels) in-tree with g++ and hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
BUILD = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libstb.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ARCH = "gfx950"

HOST_SOURCES = ["stb_host.cpp"]
DEVICE_SOURCES = ["stb_device.hip", "stb_fast.hip", "stb_gemv24.hip", "stb_gemm.hip", "stb_pack.hip"]

HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-ffp-contract=off", "-Wall", "-pthread"]
DEVICE_FLAGS = ["-O3", "-std=c++17", "-fPIC", f"--offload-arch={ARCH}",
                "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                "-Wno-unused-command-line-argument"]


def _run(cmd):
    print("+", " ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build(verbose: bool = True) -> str:
    os.makedirs(BUILD, exist_ok=True)
    inc = ["-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
    objs, cmds = [], []
    for src in HOST_SOURCES:
        obj = os.path.join(BUILD, src + ".o")
        cmds.append(["g++", *HOST_FLAGS, *inc, "-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    for src in DEVICE_SOURCES:
        obj = os.path.join(BUILD, src + ".o")
        cmds.append([HIPCC, *DEVICE_FLAGS, *inc, "-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    # the translation units are independent: compile them side by side (five processes)
    with ThreadPoolExecutor(max_workers=len(cmds)) as pool:
        list(pool.map(_run, cmds))
    # the loads issued from asm statements must keep their distance from scalar restores (see isa_check)
    try:
        from . import isa_check
    except ImportError:                      # run as a script
        sys.path.insert(0, PKG)
        import isa_check
    dev = [os.path.join(CSRC, src) for src in DEVICE_SOURCES]
    with ThreadPoolExecutor(max_workers=len(dev)) as pool:
        found = list(pool.map(lambda src: isa_check.check_source(src, BUILD, HIPCC, [*DEVICE_FLAGS, *inc]), dev))
    for src, f in zip(DEVICE_SOURCES, found):
        for w_line, w, m_line, m, ws in f:
            if ws < 0:
                print(f"{src}: {m}: {w}", flush=True)
            else:
                print(f"{src}.s:{m_line}: '{m}' reads a scalar that '{w}' (line {w_line}) wrote {ws} wait states earlier", flush=True)
    if any(found):
        raise RuntimeError("hazard in the generated code (asm loads): see the lines above")
    tmp = LIB + ".tmp"
    _run([HIPCC, "-shared", "-fPIC", f"--offload-arch={ARCH}", "-o", tmp, *objs, "-pthread"])
    shutil.move(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
