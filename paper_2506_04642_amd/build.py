"""Compile libtadakv.so (HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtadakv.so")

# packed-fp32 instruction forms are switched off for every device translation unit
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# (source, extra flags): the quantiser is compiled without fused multiply-add contraction so
# that every binary32 operation rounds once, in the order written
UNITS = [
    ("tadakv_abi.cpp", ["-x", "hip"]),
    ("quant_append.hip", ["-ffp-contract=off"]),
    ("compressv.hip", ["-ffp-contract=off", "-save-temps=obj"]),
    ("decode_valu.hip", []),
    # matrix-instruction results go straight to ordinary vector registers; the direct-to-LDS fetches
    # are issued by hand and name M0 as clobbered, which the compiler remarks on at every use
    # (the assembly text is kept next to the object and read by verify_hand_loads after the compile)
    ("decode_mfma.hip", ["-mllvm", "-amdgpu-mfma-vgpr-form", "-Wno-inline-asm", "-save-temps=obj"]),
    ("xhead_dense.hip", []),
    ("stream_probe.hip", []),
]


def sources():
    return [os.path.join(CSRC, s) for s, _ in UNITS] + [
        os.path.join(CSRC, "tadakv_internal.h"),
        os.path.join(CSRC, "quant_wave.h"),
        os.path.join(os.path.dirname(HERE), "include", "tadakv.h"),
    ]


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile every translation unit and link the shared library.  With force=False an
    up-to-date library is kept."""
    if not force and os.path.exists(LIB):
        if all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in sources()):
            return LIB
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = []
    procs = []
    for src, extra in UNITS:
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        cmd = ["hipcc"] + COMMON + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for cmd, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
        if verbose and out.strip():
            print(out)
    # the kernels that issue loads by hand: the compiler must have left the destinations alone
    import importlib.util

    spec = importlib.util.spec_from_file_location("verify_hand_loads", os.path.join(HERE, "verify_hand_loads.py"))
    _v = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(_v)  # (by path: this file also runs as a script)

    for unit, kernel, glob in (("decode_mfma", "decode_split_mfma_kernel", True), ("compressv", "compressv_gemm_kernel", False)):
        checked = _v.verify(os.path.join(objdir, unit + "-hip-amdgcn-amd-amdhsa-gfx950.s"), kernel, glob)
        if verbose:
            print("verify_hand_loads: %s: %d kernels, %d global requests, %d LDS reads" % ((unit,) + checked))
        for f in os.listdir(objdir):
            if f.startswith(unit + "-") or f.startswith(unit + ".hip-"):
                os.remove(os.path.join(objdir, f))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
