"""Build libsla.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libsla.so")
SOURCES = ["sla_api.hip", "sla_kernels.hip", "sla_kernels_bf16.hip", "sla_kernels_f32.hip", "sla_decode.hip",
           "sla_backward.hip", "sla_backward_f32.hip", "sla_backward_narrow.hip", "sla_backward_gdn.hip", "sla_backward_gdn_block.hip", "sla_prologue.hip", "sla_prologue_grad.hip"]
OBJ_DIR = os.path.join(_HERE, "_build")

# Packed-fp32 VALU instructions are switched off for all device code (a hipcc flag; the host pass
# prints a harmless "not a recognized feature" note).
FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(_ROOT, "include"),
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose: bool = False, extra=(), out: str = LIB, sources=None, jobs: int = 8) -> str:
    """Compile every source to an object (in parallel; always recompiles) and link them into the shared library."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    sources = list(sources or SOURCES)
    objs = [os.path.join(OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in sources]
    cmds = [[hipcc] + FLAGS + list(extra) + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(sources, objs)]
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(cmds)))) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", out], verbose)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
