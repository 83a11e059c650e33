"""Builds libqerl_nvfp4.so (HIP, gfx950 only) in-tree with hipcc.

`python -m paper_2510_11696_amd.build` compiles every translation unit under
csrc/ and links them into paper_2510_11696_amd/libqerl_nvfp4.so.  hipcc
cross-compiles, so this works on a machine without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.environ.get("QERL_BUILD_LIB_PATH") or os.path.join(HERE, "libqerl_nvfp4.so")   # (tuning builds may go elsewhere)
if os.environ.get("QERL_BUILD_OBJ_DIR"):
    OBJ_DIR = os.environ["QERL_BUILD_OBJ_DIR"]

# -packed-fp32-ops is switched off for all device code (v_pk_*_f32 are not to
# be generated); quantize.hip additionally forbids fp contraction so that each
# fp32 operation of the scale chain is rounded on its own.
COMMON = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]
PER_FILE = {"quantize.hip": ["-ffp-contract=off"], "mx.hip": ["-ffp-contract=off"]}
# extra hipcc flags for tuning builds, e.g. QERL_EXTRA_HIPCC_FLAGS="-DQERL_TUNING_HOOKS -DQERL_STREAM_TRACE=1"
COMMON += os.environ.get("QERL_EXTRA_HIPCC_FLAGS", "").split()


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    cmd = ["hipcc", *COMMON, *PER_FILE.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout[-2000:]}\n{r.stderr[:4000]}")
    return obj


def build(verbose: bool = True, jobs: int = 6) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, sources()))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB_PATH} from {len(objs)} translation units")
    return LIB_PATH


if __name__ == "__main__":
    build()
    sys.exit(0)
