"""Builds libfreekv.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2505_13109_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfreekv.so")
SOURCES = ["fkv_api.hip", "fkv_data.hip", "fkv_select.hip", "fkv_attn.hip", "fkv_wide.hip"]

# -ffp-contract=off: the arithmetic that decides page ids is written operation by operation.
# packed fp32 ops are switched off for this target.
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def build(verbose: bool = True, extra_flags=(), lib: str = LIB) -> str:
    """Compile every source for gfx950 and link `lib`.  Another `lib` (an experiment build with extra
    flags) keeps its objects beside itself, so it can be built while the product library is."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    obj_dir = CSRC if lib == LIB else os.path.dirname(os.path.abspath(lib))
    for src in SOURCES:
        obj = os.path.join(obj_dir, os.path.basename(lib) + "." + src.replace(".hip", ".o") if lib != LIB else src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l or "error" in l]
        if p.returncode != 0:
            failed = True
            print(out, file=sys.stderr)
        elif verbose and lines:
            print("\n".join(lines))
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", lib]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    build()
