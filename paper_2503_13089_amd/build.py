"""Builds libcluscomp.so (gfx950 only) from csrc/*.hip with hipcc, in-tree."""
from __future__ import annotations

import glob
import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
LIB = os.path.join(_HERE, "libcluscomp.so")

# Packed-FP32 instruction selection is switched off for all device code (see the design notes).
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


# Kernels whose global loads are written as instructions with hand-placed waits: a register spill inside them would
# put memory operations of the compiler's own between those loads and shift what the waits count. The build reads
# the compiler's resource report for them and fails if it shows a spill or scratch memory.
NO_SPILL_KERNELS = {"layer_gemm.hip": ("gemm_frag_kernel",)}


def sources():
    return sorted(glob.glob(os.path.join(_HERE, "csrc", "*.hip")))


def _check_no_spills(src: str, report: str) -> None:
    names = NO_SPILL_KERNELS.get(os.path.basename(src), ())
    current, seen = None, set()
    for line in report.splitlines():
        if "Function Name:" in line:
            current = next((n for n in names if n in line), None)
            if current:
                seen.add(current)
        elif current and ("VGPRs Spill:" in line or "ScratchSize" in line):
            value = int(line.split(":")[-1].split("[")[0].strip())
            if value != 0:
                raise RuntimeError(f"{os.path.basename(src)}: {current} needs scratch memory or spills registers "
                                   f"({line.split('remark:')[-1].strip()}); its hand-placed memory waits assume it does not")
    missing = set(names) - seen
    if missing:
        raise RuntimeError(f"{os.path.basename(src)}: no resource report for {sorted(missing)}")


def build(verbose: bool = False) -> str:
    """Compiles every kernel and the C ABI into one shared library. Always recompiles: one hipcc per
    source file (in parallel, objects in a temporary folder), then one link."""
    noise = "is not a recognized feature for this target"

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        proc = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + err)
        src = next((a for a in cmd if a.endswith(".hip")), None)
        if src is not None and os.path.basename(src) in NO_SPILL_KERNELS:
            _check_no_spills(src, err)
            err = "\n".join(l for l in err.splitlines() if "remark:" not in l and "|" not in l[:12])
        if verbose and err.strip():
            print(err)

    with tempfile.TemporaryDirectory(prefix="cluscomp_build_") as tmp:
        objs = []
        jobs = []
        for src in sources():
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            objs.append(obj)
            report = ["-Rpass-analysis=kernel-resource-usage"] if os.path.basename(src) in NO_SPILL_KERNELS else []
            jobs.append(["hipcc", *HIPCC_FLAGS, *report, "-I", os.path.join(ROOT, "include"), "-c", src, "-o", obj])
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
            list(pool.map(run, jobs))
        run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
