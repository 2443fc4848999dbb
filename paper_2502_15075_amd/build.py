"""Builds libkvq.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2502_15075_amd.build`."""
from __future__ import annotations

import os
import re
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
          "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes", "-Wno-unused-function",
          "-Wno-unneeded-internal-declaration"]
# (b_K, b_V) pairs with decode kernels: kvq_decode.hip is compiled once per pair (-DKVQ_INST_BK/BV: the kernels of that
# pair) and once without (plan + dispatch), so that the instances build in parallel.
DECODE_PAIRS = [(4, 2), (2, 4), (4, 4), (8, 8), (2, 2), (8, 4), (8, 2), (4, 8), (2, 8), (16, 16),
                (3, 2), (3, 4), (3, 8), (6, 2), (6, 4), (6, 8), (1, 2), (1, 4), (1, 8),
                (1, 1), (2, 1), (3, 1), (4, 1), (6, 1), (8, 1),
                (1, 3), (2, 3), (3, 3), (4, 3), (6, 3), (8, 3), (1, 6), (2, 6), (3, 6), (4, 6), (6, 6), (8, 6),
                # one tensor unquantized (the ablations that quantize only keys or only values)
                (16, 1), (16, 2), (16, 3), (16, 4), (16, 6), (16, 8), (1, 16), (2, 16), (3, 16), (4, 16), (6, 16), (8, 16)]
# No decode kernel may use scratch memory (a register spill in the streaming loop costs more than any ring depth gains):
# the build fails on an instance that does.
def _scratch_allowed(kernel_name: str) -> int:
    return 0


# (source, object name, extra flags).  The quantizer must round every operation once: no contraction.
UNITS = [("kvq_api.hip", "kvq_api.o", []),
         ("kvq_quant.hip", "kvq_quant.o", ["-ffp-contract=off"]),
         ("kvq_decode.hip", "kvq_decode.o", [])]
UNITS += [("kvq_decode.hip", f"kvq_decode_k{bk}v{bv}.o",
           [f"-DKVQ_INST_BK={bk}", f"-DKVQ_INST_BV={bv}", "-Rpass-analysis=kernel-resource-usage"]) for bk, bv in DECODE_PAIRS]


def _compile(item):
    src, objname, extra = item
    obj = os.path.join(OBJ, objname)
    cmd = ["hipcc", "-c", os.path.join(CSRC, src), "-o", obj] + COMMON + extra
    r = subprocess.run(cmd, capture_output=True, text=True)
    log = r.stdout + r.stderr
    if r.returncode == 0 and "-Rpass-analysis=kernel-resource-usage" in extra:
        # a decode kernel that spills would wait on scratch reloads in the middle of its load pipeline: refuse it
        spills = []
        for block in re.split(r"Function Name: ", log)[1:]:
            m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", block)
            if m and int(m.group(1)) > _scratch_allowed(block.split()[0]):
                spills.append(int(m.group(1)))
        if spills:
            return objname, 1, f"{len(spills)} decode kernel(s) use scratch memory (register spills, up to {max(spills)} bytes per lane)", obj
        log = "\n".join(l for l in log.splitlines() if "remark:" not in l)
    return objname, r.returncode, log, obj


def build_lib(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        results = list(ex.map(_compile, UNITS))
    objs, failed = [], []
    for src, rc, log, obj in results:
        if verbose and log.strip():
            print(f"--- {src}\n{log}", file=sys.stderr)
        if rc != 0:
            failed.append(f"{src}:\n{log}")
        objs.append(obj)
    if failed:                                     # every failing unit is named, and the library of an earlier build goes:
        if os.path.exists(LIB):                    # nothing may load a library that the sources no longer produce
            os.remove(LIB)
        raise RuntimeError("hipcc failed on " + "\n".join(failed))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
