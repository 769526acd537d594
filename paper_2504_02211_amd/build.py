"""Builds libftattn.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libftattn.so")
SOURCES = [os.path.join(PKG, "csrc", "ftattn.hip"), os.path.join(PKG, "csrc", "ftattn_perstep.hip"),
           os.path.join(PKG, "csrc", "ftattn_elementwide.hip"), os.path.join(PKG, "csrc", "ftattn_lazy.hip"),
           os.path.join(PKG, "csrc", "ftgemm.hip"), os.path.join(PKG, "csrc", "ftdecoupled.hip")]
HEADERS = [os.path.join(PKG, "csrc", "ftattn_device.h"), os.path.join(PKG, "csrc", "ftattn_main.h"),
           os.path.join(PKG, "csrc", "ftgemm_main.h"), os.path.join(ROOT, "include", "ftattn.h"),
           os.path.join(ROOT, "include", "ftgemm.h"), os.path.join(ROOT, "include", "ftdecoupled.h")]
OBJDIR = os.path.join(PKG, "_build")


def build(verbose: bool = True, extra_flags=()) -> str:
    """Compiles every HIP source for gfx950 (one hipcc process per source, side by side) and
    links the shared library; returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-value", "-Wno-unknown-attributes", "-Wno-inline-asm",
             "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"), *extra_flags]
    os.makedirs(OBJDIR, exist_ok=True)
    objs, procs = [], []
    for src in SOURCES:
        obj = os.path.join(OBJDIR, os.path.splitext(os.path.basename(src))[0] + ".o")
        cmd = [hipcc, *flags, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    failed = []
    for cmd, p in procs:
        text, _ = p.communicate()
        out = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed.append(out)
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed:\n" + "\n".join(failed))
    if verbose:
        print(" ".join(link), flush=True)
    res = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stdout)
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
