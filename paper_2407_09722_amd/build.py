"""Builds libmtad.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmtad.so")
SOURCES = ["kernels_gemm.hip", "kernels_gemm_tiled.hip", "kernels_misc.hip", "kernels_attn.hip", "kernels_attn_mfma.hip", "kernels_beam.hip", "kernels_flow.hip", "mtad_abi.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _hipcc():
    for p in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if p and (os.path.sep not in p or os.path.exists(p)):
            return p
    raise RuntimeError("hipcc not found")


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False, defines=(), lib: str = LIB, objdir_name: str = "_build") -> str:
    """Compiles every source for gfx950 and links `lib`.  `defines` adds -D macros (development builds)."""
    hipcc = _hipcc()
    objdir = os.path.join(HERE, objdir_name)
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        return _run([hipcc, *FLAGS, *["-D" + d for d in defines], "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        logs = list(ex.map(one, zip(SOURCES, objs)))
    logs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]))
    if verbose:
        print("\n".join(l for l in logs if l.strip()))
    return lib


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
