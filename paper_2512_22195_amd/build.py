"""Compiles libmatkv.so (gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libmatkv.so")
OBJ_DIR = os.path.join(_HERE, "_build")

SOURCES = ["matkv_api.hip", "attn_rows.hip", "attn_mfma.hip", "attn_prefill.hip", "materialize.hip",
           "materialize_mfma.hip", "compress.hip"]

_NOISE = "is not a recognized feature for this target"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if _NOISE not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + msgs)
    if verbose and msgs.strip():
        print(msgs)


def build(verbose: bool = False, only: list[str] | None = None) -> str:
    """Compile every HIP source (one hipcc process each, side by side) and link them into
    paper_2512_22195_amd/libmatkv.so.  `only`: recompile just these sources and reuse the other
    objects of an earlier build (for work on one kernel file)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument",
             "-I", os.path.join(_ROOT, "include"), "-I", CSRC]
    objs = {s: os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES}
    todo = [s for s in SOURCES if only is None or s in only or not os.path.exists(objs[s])]
    jobs = int(os.environ.get("MAX_JOBS", "8"))
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(todo) or 1))) as ex:
        list(ex.map(lambda s: _run([hipcc] + flags + ["-c", os.path.join(CSRC, s), "-o", objs[s]], verbose), todo))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + [objs[s] for s in SOURCES], verbose)
    return LIB_PATH


if __name__ == "__main__":
    import sys
    print(build(verbose=True, only=sys.argv[1:] or None))
