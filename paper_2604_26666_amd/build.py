"""Compile the HIP library for gfx950 into paper_2604_26666_amd/libfact_gemm.so.

One translation unit per tile configuration (csrc/configs.def), compiled in parallel,
plus the auxiliary kernels and the C ABI.  hipcc cross-compiles without a GPU.
"""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfact_gemm.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-I", CSRC]


def configs():
    rows = []
    with open(os.path.join(CSRC, "configs.def")) as f:
        for line in f:
            m = re.match(r"\s*FACT_CFG\(\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*\)", line)
            if m:
                rows.append(tuple(int(x) for x in m.groups()))
    return rows


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + out)
    return out


def build(jobs=None, verbose=False, extra_flags=(), lib=LIB, obj_dir=OBJ):
    """extra_flags / lib / obj_dir exist for experiments (a variant library beside the product one)."""
    OBJ = obj_dir
    LIB = lib
    FLAGS = list(globals()["FLAGS"]) + list(extra_flags)
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(8, os.cpu_count() or 1)
    units = []
    for (cid, bm, bn, wm, wn, bk, st) in configs():
        obj = os.path.join(OBJ, f"inst{cid}.o")
        units.append((obj, [HIPCC] + FLAGS + [f"-DFACT_ID={cid}", f"-DFACT_BM={bm}", f"-DFACT_BN={bn}",
                                              f"-DFACT_WM={wm}", f"-DFACT_WN={wn}", f"-DFACT_BK={bk}", f"-DFACT_STAGES={st}",
                                              "-c", os.path.join(CSRC, "inst.hip"), "-o", obj]))
    for name in ("aux_kernels", "fact_api"):
        obj = os.path.join(OBJ, name + ".o")
        units.append((obj, [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, name + ".hip"), "-o", obj]))
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for out in ex.map(lambda u: _run(u[1]), units):
            if verbose and out:
                print(out)
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [u[0] for u in units])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
