"""Builds the HIP library (gfx950) in-tree: paper_2605_21649_amd/libentmaxkv.so.

    python -m paper_2605_21649_amd.build

hipcc cross-compiles without a GPU.  Objects go to paper_2605_21649_amd/_build/ (not committed)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libentmaxkv.so")
SOURCES = ["api.hip", "stats.hip", "score.hip", "select_topk.hip", "select_gauss.hip", "select_box.hip", "decode.hip",
           "softmax_sparse.hip", "probe.hip"]
# packed-FP32 instructions are switched off for all device code (hipcc-only flag; the host pass warns
# that it does not know the feature, which is harmless)
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-pass-failed"]


def _compile(src, objdir):
    obj = os.path.join(objdir, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                     if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{msgs}")
    return obj, msgs


def build_library(verbose=True, jobs=8):
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        results = list(ex.map(lambda s: _compile(s, objdir), SOURCES))
    for (obj, msgs), src in zip(results, SOURCES):
        if verbose and msgs.strip():
            print(f"[{src}]\n{msgs}", file=sys.stderr)
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", OUT, *[o for o, _ in results]]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    if verbose:
        print("built", OUT)
    return OUT


if __name__ == "__main__":
    build_library()
