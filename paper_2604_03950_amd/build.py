"""Build libdma_mi355x.so in-tree with hipcc for gfx950 (cross-compiles without a GPU).

    python -m paper_2604_03950_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdma_mi355x.so")
SOURCES = ["dma_api.hip", "dma_quantize.hip", "dma_attn_fwd.hip", "dma_diag.hip"]
HEADERS = ["dma_device.hpp", "dma_internal.hpp", "dma_attn_kernel.hpp", os.path.join("..", "..", "include", "dma.h")]
# (low, high) format pairs of the fused forward, as product-path ids of dma_device.hpp: dma_attn_inst.hip is compiled
# once per pair (the list mirrors the declarations in dma_attn_fwd.hip)
ATTN_PAIRS = [(2, 3), (2, 1), (2, 4), (2, 2), (3, 3), (1, 1), (4, 4), (0, 0)]
MAX_PARALLEL = 8

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-FP32 VALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def source_digest() -> str:
    """SHA-256 over the kernel sources and the public header (file names and contents, sorted by name): what a profile
    summary records so that a figure measured on one version of the kernels is not quoted for another."""
    import hashlib
    h = hashlib.sha256()
    names = sorted(n for n in os.listdir(CSRC) if n.endswith((".hip", ".hpp")))
    for path in [os.path.join(CSRC, n) for n in names] + [os.path.join(HERE, "..", "include", "dma.h")]:
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def _stale(obj: str, deps: list[str]) -> bool:
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source and link the shared library.  Returns its path."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    headers = [os.path.join(CSRC, h) for h in HEADERS]
    jobs, objs = [], []
    units = [(s, s.replace(".hip", ".o"), []) for s in SOURCES]
    units += [("dma_attn_inst.hip", f"dma_attn_inst_{lo}_{hi}.o", [f"-DDMA_LO={lo}", f"-DDMA_HI={hi}"]) for lo, hi in ATTN_PAIRS]
    for s, o, defs in units:
        src = os.path.join(CSRC, s)
        obj = os.path.join(objdir, o)
        objs.append(obj)
        if force or _stale(obj, [src] + headers):
            cmd = ["hipcc"] + HIPCC_FLAGS + defs + ["-c", src, "-o", obj]
            if verbose:
                cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
            jobs.append((o, cmd))
    failed = False
    while jobs:
        batch, jobs = jobs[:MAX_PARALLEL], jobs[MAX_PARALLEL:]
        procs = [(o, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)) for o, cmd in batch]
        for o, p in procs:
            out, _ = p.communicate()
            lines = [ln for ln in out.splitlines() if "packed-fp32-ops" not in ln]
            if p.returncode != 0 or verbose:
                print(f"--- {o}\n" + "\n".join(lines), file=sys.stderr)
            failed |= p.returncode != 0
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, check=True)
    return LIB


if __name__ == "__main__":
    if "--digest" in sys.argv:
        print(source_digest())
    else:
        print(build(force="--incremental" not in sys.argv, verbose="-v" in sys.argv))
