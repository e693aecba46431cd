"""Build libantkv.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libantkv.so")
SOURCES = ["api.hip", "encode.hip", "encode12.hip", "topk.hip", "window.hip", "prefill_attn.hip", "kmeans.hip", "anchor_score.hip", "decode12.hip", "decode_attn.hip", "rope_keys.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # keep the compiler from forming packed-FP32 VALU instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# per-file additions: the encode kernel takes maxima of finite scores only
EXTRA_FLAGS = {"encode.hip": ["-fno-honor-nans"]}


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


PROBE_SRC = "machine_limits.hip"                     # stand-alone probe of the chip's HBM / LDS / issue rates (not part of the library)
PROBE = os.path.join(HERE, "machine_limits")


def build(verbose: bool = False) -> str:
    """Compile every source, link libantkv.so, and build the stand-alone machine_limits probe beside it."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()

    def run(cmd, what):
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0 or verbose:
            sys.stderr.write(r.stdout + r.stderr)
        if r.returncode != 0:
            raise RuntimeError(what)

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        run([hipcc, *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj], f"hipcc failed on {src}")
        return obj

    def build_probe(_):
        run([hipcc, *[f for f in FLAGS if f != "-fPIC"], os.path.join(CSRC, PROBE_SRC), "-o", PROBE], f"hipcc failed on {PROBE_SRC}")

    with ThreadPoolExecutor(len(SOURCES) + 1) as ex:
        probe = ex.submit(build_probe, None)
        objs = list(ex.map(compile_one, SOURCES))
        probe.result()
    run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], "link failed")
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
