"""Builds libchimera.so (gfx950) next to this file with hipcc.

    python -m paper_2107_06925_amd.build
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libchimera.so")
OBJ = os.path.join(HERE, "_build")
SOURCES = ["schedule.cpp", "stage.hip", "rowwise.hip", "reference_kernels.hip", "gemm_mfma.hip", "attention_mfma.hip", "probe.hip", "edges.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# Per-file additions.  The attention kernels work on their MFMA results with vector instructions
# in every loop step (softmax, rescaling); with the accumulators in the AGPR half of the register
# file every such touch costs a v_accvgpr move each way, a quarter of the kernels' vector
# instructions.  The VGPR form of the MFMA instructions avoids them.
EXTRA_FLAGS = {"attention_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _compile(src):
    obj = os.path.join(OBJ, src.rsplit(".", 1)[0] + ".o")
    cmd = ["hipcc", *FLAGS, *EXTRA_FLAGS.get(src, []), "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    return src, obj, r


def build(verbose=True):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(_compile, SOURCES))
    objs = []
    for src, obj, r in results:
        out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                        if "packed-fp32-ops" not in l and l.strip())
        if r.returncode:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out:
            print(out)
        objs.append(obj)
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *objs],
                       capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    return OUT


if __name__ == "__main__":
    print(build())
