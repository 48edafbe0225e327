"""Builds libcascade_attn.so (gfx950) in-tree with hipcc.  Used by __graft_entry__.build()."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.environ.get("CASCADE_ATTN_LIB") or os.path.join(PKG, "libcascade_attn.so")

SOURCES = ["ca_meta.cpp", "ca_api.cpp", "ca_sched.cpp", "rope_cache.hip", "attn_f32.hip", "attn_bf16.hip", "mfma_peak.hip", "gemm_bf16.hip"]

# packed fp32 instructions are kept off for all device code on the test machines
DEVICE_FLAGS = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def build(verbose: bool = False, extra=(), bdir: str | None = None) -> str:
    objs = []
    bdir = bdir or os.path.join(PKG, "_build")
    os.makedirs(bdir, exist_ok=True)
    # the hand-scheduled attention main loop is emitted as an inline-assembly include
    subprocess.run([sys.executable, os.path.join(CSRC, "gen_attn_core.py"),
                    os.path.join(bdir, "attn_core_gfx950.inc")], check=True,
                   stdout=None if verbose else subprocess.DEVNULL)
    subprocess.run([sys.executable, os.path.join(CSRC, "gen_gemm_core.py"),
                    os.path.join(bdir, "gemm_core_gfx950.inc")], check=True,
                   stdout=None if verbose else subprocess.DEVNULL)
    common = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-I", os.path.join(ROOT, "include"),
              "-I", CSRC, "-I", bdir, "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"] + DEVICE_FLAGS + list(extra)
    procs = []
    for src in SOURCES:
        obj = os.path.join(bdir, src + ".o")
        cmd = [hipcc(), "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + common
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
