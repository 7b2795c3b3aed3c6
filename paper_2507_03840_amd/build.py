"""Builds libegnn_hip.so (gfx950) in-tree with hipcc.  `python -m paper_2507_03840_amd.build`."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libegnn_hip.so")
SOURCES = ["egnn_api.hip", "egnn_api_backward.hip", "nlist.hip", "edge_radial.hip", "node_mix.hip", "tp_segsum.hip",
           "readout.hip", "layer_fused.hip", "layer_fused_lane.hip", "graph_util.hip", "tp_backward.hip", "radial_backward.hip", "readout_backward.hip",
           "so2_message.hip", "hamiltonian.hip", "partition.hip", "static_scratch.hip", "edge_pairs.hip", "radial_grid.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         # keep the compiler from forming packed fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    r = subprocess.run(cmd, cwd=CSRC, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    text = "\n".join(l for l in r.stdout.splitlines() if "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), text))
    return text


def build(verbose=True, extra_flags=()):
    _run([sys.executable, os.path.join(CSRC, "gen_tables.py")])
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        out = _run([HIPCC, *FLAGS, *extra_flags, "-c", src, "-o", obj])
        return obj, out

    with ThreadPoolExecutor(max_workers=8) as ex:
        results = list(ex.map(compile_one, SOURCES))
    for obj, out in results:
        if verbose and out.strip():
            print(out)
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *[o for o, _ in results]])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
