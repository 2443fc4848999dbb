"""Builds libkvq.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2502_15075_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libkvq.so")

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
          # packed-FP32 VALU forms are kept out of the generated code
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes"]
# translation unit -> extra flags.  The quantizer must round every operation once: no contraction.
UNITS = {
    "kvq_api.hip": [],
    "kvq_quant.hip": ["-ffp-contract=off"],
    "kvq_decode.hip": [],
}


def _compile(item):
    src, extra = item
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = ["hipcc", "-c", os.path.join(CSRC, src), "-o", obj] + COMMON + extra
    r = subprocess.run(cmd, capture_output=True, text=True)
    return src, r.returncode, (r.stdout + r.stderr), obj


def build_lib(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(_compile, UNITS.items()))
    objs = []
    for src, rc, log, obj in results:
        if verbose and log.strip():
            print(f"--- {src}\n{log}", file=sys.stderr)
        if rc != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{log}")
        objs.append(obj)
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
