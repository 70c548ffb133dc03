"""Build libqgemm.so for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_2504_12984_amd.build [-j N]

Per-weight-type sources (de-quantiser, small-M and tiled matmul kernels) are
compiled once per weight type, in parallel, then linked into one shared library
next to this file.  Objects go to _build/ (not tracked).
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libqgemm.so")
NUM_WT = 14
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-std=c++20", "-O3", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _jobs():
    jobs = [("qg_pack.hip", None), ("qg_probe.hip", None), ("qg_api.hip", None)]
    for src in ("qg_dequant.hip", "qg_decode_gemm.hip", "qg_large.hip", "qg_large32.hip", "qg_gemv.hip"):
        jobs += [(src, wt) for wt in range(NUM_WT)]
    jobs += [("qg_a8_gemm.hip", -bits) for bits in range(1, 9)]      # int8 activations: once per code width
    jobs.append(("qg_large.hip", NUM_WT))      # the tiled kernel on weights already de-quantised (pass-through decoder)
    for src in ("qg_dequant.hip", "qg_decode_gemm.hip", "qg_large.hip"):      # codebook indices of 1..8 bits (kernel-side types 15..22)
        jobs += [(src, NUM_WT + 1 + b) for b in range(8)]
    return jobs


# The tiled kernels issue their matrix instructions through inline asm, so the
# compiler does not know when an accumulator is final and would spill or reload one
# without waiting for the matrix pipeline.  Their register budget is therefore
# checked at build time: beyond the few dwords of loop-invariant values that are parked
# across the main loop, nothing may go to scratch memory.
SPILL_CHECKED = {"qg_large.hip": 16, "qg_large32.hip": 16}    # bytes per lane allowed


def _check_scratch(stem, src, remarks):
    limit = SPILL_CHECKED[src]
    name = None
    for ln in remarks.splitlines():
        m = re.search(r"remark: (.*?) \[-Rpass-analysis", ln)
        if not m:
            continue
        text = m.group(1).strip()
        if text.startswith("Function Name:"):
            name = text.split(":", 1)[1].strip()
        elif text.startswith("ScratchSize") and name:
            used = int(text.split(":")[1])
            if used > limit:
                raise RuntimeError(f"{stem}: kernel {name} spills {used} bytes per lane to scratch "
                                   f"(limit {limit}); its accumulators are not safe to spill")


def _stem(job):
    """Object name of a job: (source, None), (source, weight-type index) or (source, -code width)."""
    src, wt = job
    return src[:-4] + ("" if wt is None else f"_wt{wt}" if wt >= 0 else f"_bits{-wt}")


def _compile(job):
    src, wt = job
    stem = _stem(job)
    obj = os.path.join(OBJ, stem + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    if wt is not None:
        cmd.insert(-4, f"-DQG_WT={wt}" if wt >= 0 else f"-DQG_BITS={-wt}")
    if src in SPILL_CHECKED:
        cmd.insert(-4, "-Rpass-analysis=kernel-resource-usage")
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        err = "\n".join(ln for ln in r.stderr.splitlines() if "packed-fp32-ops" not in ln)
        raise RuntimeError(f"hipcc failed for {stem}:\n{err}")
    if src in SPILL_CHECKED:
        _check_scratch(stem, src, r.stderr)
    lines = [ln for ln in r.stderr.splitlines() if "packed-fp32-ops" not in ln]
    if src in SPILL_CHECKED:      # drop the resource remarks and the source excerpts printed with them
        lines = [ln for ln in lines if "warning:" in ln or "error:" in ln]
    err = "\n".join(lines)
    return obj, err


def build(jobs: int | None = None, verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        results = list(ex.map(_compile, _jobs()))
    objs = [o for o, _ in results]
    if verbose:
        for _, err in results:
            if err.strip():
                print(err, file=sys.stderr)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    n = None
    if "-j" in sys.argv:
        n = int(sys.argv[sys.argv.index("-j") + 1])
    print(build(n))
