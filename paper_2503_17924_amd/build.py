"""Builds libwlb.so (the C-ABI library) for gfx950 with hipcc, in-tree.

Run as `python -m paper_2503_17924_amd.build` or through `__graft_entry__.build()`.
hipcc cross-compiles, so no GPU is needed to build.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libwlb.so")
SOURCES = ["wlb_host.cpp", "wlb_plan.hip", "wlb_attn_fwd.hip", "wlb_attn_bwd.hip", "wlb_calib.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 instructions are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def build(verbose: bool = False, keep_asm: bool = False, lib_out: str | None = None) -> str:
    """Compiles every source and links the library (to `lib_out`, default in-tree libwlb.so).
    WLB_HIPCC_EXTRA adds compiler flags (space separated) to every compile line."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    extra = os.environ.get("WLB_HIPCC_EXTRA", "").split()
    lib_out = lib_out or LIB
    bdir = os.path.join(ROOT, "_build" if lib_out == LIB else "_build/" + os.path.basename(lib_out))
    os.makedirs(bdir, exist_ok=True)
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(bdir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if src.endswith(".cpp"):
            # host code: no fused multiply-add contraction, so the latency estimates are the same
            # doubles on every machine
            cmd[1:1] = ["-x", "hip", "-ffp-contract=off"]
        if "attn" in src:
            # kernels only: lets max() compile to bare v_max3 (no NaN quieting); the host-side
            # argument checks live in other files and keep full NaN semantics
            cmd += ["-fno-honor-nans"]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, cwd=bdir)))
        if keep_asm and src.endswith(".hip"):
            asm = [c for c in cmd if c != "-c"]
            asm[asm.index("-o") + 1] = os.path.join(bdir, os.path.splitext(src)[0] + ".s")
            asm += ["-S", "--cuda-device-only"]
            procs.append((src + " (asm)", subprocess.Popen(asm, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, cwd=bdir)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    tmp = lib_out + ".tmp"
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp]
    r = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    os.replace(tmp, lib_out)
    return lib_out


if __name__ == "__main__":
    _out = [a.split("=", 1)[1] for a in sys.argv if a.startswith("--out=")]
    print(build(verbose=True, keep_asm="--asm" in sys.argv, lib_out=os.path.abspath(_out[0]) if _out else None))
