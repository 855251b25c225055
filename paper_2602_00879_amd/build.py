"""Builds the C-ABI library `libdes_hip.so` from csrc/ with hipcc for gfx950,
in-tree (next to this file)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdes_hip.so")
SOURCES = ["des_api.hip", "des_routing.hip", "des_ffn.hip", "des_attention.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 arithmetic is switched off (some of its forms are unreliable here)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    *(["-DDES_ROUTING_TIMESTAMPS"] if os.environ.get("DES_ROUTING_TIMESTAMPS") else []),
    *(["-DDES_FFN_STAMPS"] if os.environ.get("DES_FFN_STAMPS") else []),
    *(["-DDES_FFN_WAVES=" + os.environ["DES_FFN_WAVES"]] if os.environ.get("DES_FFN_WAVES") else []),
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("is not a recognized feature for this target", "inline asm clobber list contains reserved",
             "Reserved registers on the clobber list")
    lines = r.stderr.splitlines()
    keep = []
    skip = 0
    for l in lines:  # drop the known-harmless warnings together with their source excerpts
        if any(n in l for n in noise):
            skip = 2 if "warning" in l or "note" in l else 0
            continue
        if skip > 0 and (l.lstrip().startswith(("|", "^")) or l[:6].strip().isdigit() or " | " in l[:12]):
            skip -= 1
            continue
        skip = 0
        keep.append(l)
    err = "\n".join(keep)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)


def build(verbose: bool = False) -> str:
    """Compiles every source to an object file (in parallel) and links the library."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    cflags = [f for f in FLAGS if f != "-shared"]
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        jobs = [ex.submit(_run, [hipcc, *cflags, "-c", os.path.join(CSRC, s), "-o", o], verbose)
                for s, o in zip(SOURCES, objs)]
        for j in jobs:
            j.result()
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], verbose)
    return LIB


def device_asm(source: str, out_path: str) -> str:
    """gfx950 assembly of one source file (device side only), for checks on the
    generated code (wait states around hand-written asm, register spills)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in FLAGS if f not in ("-fPIC", "-shared")]
    cmd = [hipcc, *flags, "--cuda-device-only", "-S", os.path.join(CSRC, source), "-o", out_path]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stderr)
    return out_path


if __name__ == "__main__":
    print(build(verbose=True))
