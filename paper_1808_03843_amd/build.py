"""Builds libals_gfx950.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libals_gfx950.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "hermitian.hip", "hermitian_x3.hip", "wide.hip", "wide_ldlt.hip", "wide_ldlt_bf16.hip", "wide_ldlt_f16.hip", "wide_ldlt_implicit.hip", "implicit.hip", "dual.hip", "solve.hip", "plan.hip", "metrics.hip", "transpose.hip", "peaks.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    extra = os.environ.get("ALS_EXTRA_HIPCC_FLAGS", "").split()   # e.g. -DALS_DEPTH_SLOTS=4 for tuning runs
    # the register / scratch / occupancy report of every kernel is kept beside the object: the MFMAs are
    # inline asm that the compiler cannot protect, so a kernel that spills is a kernel that may be wrong
    cmd = [HIPCC, *FLAGS, *extra, "-Rpass-analysis=kernel-resource-usage", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
    with open(obj + ".resources", "w") as fh:
        fh.write(r.stderr)
    return obj


def kernel_resources(obj_dir: str = None):
    """Parses the reports written by the last build: {kernel name: {"vgpr", "agpr", "spill", "scratch", "occupancy"}}."""
    import re
    obj_dir = obj_dir or OBJ_DIR
    out = {}
    for src in SOURCES:
        path = os.path.join(obj_dir, src.replace(".hip", ".o") + ".resources")
        if not os.path.exists(path):
            continue
        with open(path) as fh:
            text = fh.read()
        for blk in re.split(r"remark: Function Name: ", text)[1:]:
            name = blk.split(" ")[0]
            num = lambda key: int(re.search(key + r": (\d+)", blk).group(1))
            out[name] = {"vgpr": num("VGPRs"), "agpr": num("AGPRs"), "spill": num("VGPRs Spill"),
                         "scratch": num(r"ScratchSize \[bytes/lane\]"), "occupancy": num(r"Occupancy \[waves/SIMD\]")}
    return out


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "als.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, lib: str = LIB) -> str:
    if not force and not stale():
        return lib
    os.makedirs(OBJ_DIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    return lib


if __name__ == "__main__":
    print(build())
