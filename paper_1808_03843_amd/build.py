"""Builds libals_gfx950.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libals_gfx950.so")
OBJ_DIR = os.path.join(HERE, "_build")
# canary build: every hand-written MFMA waits for its operands and for its result (csrc/tiles.h, ALS_DRAINED_MFMA);
# tests/test_gpu_drained.py compares it with the production library bit for bit
LIB_DRAINED = os.path.join(HERE, "libals_gfx950_drained.so")
OBJ_DIR_DRAINED = os.path.join(HERE, "_build_drained")
SOURCES = ["api.hip", "hermitian.hip", "hermitian_x3.hip", "hermitian_x2.hip", "wide.hip", "wide_ldlt.hip", "wide_ldlt_bf16.hip", "wide_ldlt_f16.hip", "wide_ldlt_implicit.hip", "implicit.hip", "implicit16.hip", "dual.hip", "cg_short.hip", "solve.hip", "plan.hip", "metrics.hip", "transpose.hip", "peaks.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _compile(job) -> str:
    src, obj_dir, defines = job
    obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
    extra = os.environ.get("ALS_EXTRA_HIPCC_FLAGS", "").split()   # e.g. -DALS_DEPTH_SLOTS=4 for tuning runs
    # the register / scratch / occupancy report of every kernel is kept beside the object: the fp32 MFMAs are
    # inline asm that the compiler cannot protect, so a kernel that spills may be wrong
    cmd = [HIPCC, *FLAGS, *defines, *extra, "-Rpass-analysis=kernel-resource-usage", "-c", os.path.join(CSRC, src), "-o", obj]
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


def _link(lib: str, objs) -> None:
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")


def check_resources(obj_dir: str = None) -> None:
    """Raises if a kernel of the library spills registers or uses scratch memory: a spill store next to an inline-asm
    MFMA can save a register whose new value has not arrived yet, so such a build must not be loaded."""
    bad = {k: v for k, v in kernel_resources(obj_dir).items() if k.startswith("_ZN3als") and (v["spill"] or v["scratch"])}
    if bad:
        raise RuntimeError("kernels that spill or use scratch (the build is refused): "
                           + "; ".join(f"{k}: {v}" for k, v in sorted(bad.items())))


def build(force: bool = True, lib: str = LIB, drained: bool = True, obj_dir: str = OBJ_DIR) -> str:
    """Compiles every source for gfx950 and links the library; with `drained` also the canary library.
    lib / obj_dir: another place for a variant build (ALS_EXTRA_HIPCC_FLAGS), e.g. the timing variants of profiles/."""
    if not force and not stale() and (not drained or os.path.exists(LIB_DRAINED)):
        return lib
    jobs = [(src, obj_dir, []) for src in SOURCES]
    if drained:
        jobs += [(src, OBJ_DIR_DRAINED, ["-DALS_DRAINED_MFMA"]) for src in SOURCES]
        os.makedirs(OBJ_DIR_DRAINED, exist_ok=True)
    os.makedirs(obj_dir, exist_ok=True)
    # the slowest translation units first, so that they do not end up alone at the tail of the pool
    slow = {"wide.hip": 0, "wide_ldlt_implicit.hip": 1, "wide_ldlt.hip": 2, "wide_ldlt_f16.hip": 3, "wide_ldlt_bf16.hip": 4,
            "hermitian.hip": 5}
    jobs.sort(key=lambda j: slow.get(j[0], 99))
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        objs = dict(zip([(j[0], j[1]) for j in jobs], ex.map(_compile, jobs)))
    check_resources(obj_dir)
    _link(lib, [objs[(src, obj_dir)] for src in SOURCES])
    if drained:
        _link(LIB_DRAINED, [objs[(src, OBJ_DIR_DRAINED)] for src in SOURCES])
    return lib


if __name__ == "__main__":
    print(build())
