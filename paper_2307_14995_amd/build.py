"""Build step: compile the gfx950 HIP sources into paper_2307_14995_amd/libltn_attn.so.

hipcc cross-compiles for gfx950 without a GPU.  The library is built in-tree so that
it travels with the source tree; it is never installed elsewhere.  Every source is
compiled to an object of its own (in parallel), then linked; the compiler's per-kernel
resource report is read back and the build fails if a kernel that relies on registers
staying put (see ``NO_SPILL``) was given scratch memory or spilled vector registers.
"""
from __future__ import annotations

import glob
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libltn_attn.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-Rpass-analysis=kernel-resource-usage",
]

# Kernels whose inline-assembly loads land in registers asynchronously (issued blocks ahead,
# waited for with explicit vmcnt counts): a spill or a stack copy between issue and wait would
# read stale data without any diagnostic, so such a build is refused.
NO_SPILL = re.compile(r"pass_bf16_kernel|pass_f32_kernel|tiled_(fwd|bwd)_bf16_kernel")


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _headers():
    return glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))


def _obj_of(src: str) -> str:
    return os.path.join(OBJ, os.path.basename(src) + ".o")


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def is_stale() -> bool:
    return _stale(LIB, sources() + _headers())


def check_resource_report(report: str) -> None:
    """Raise if a NO_SPILL kernel of this compiler report uses scratch or spilled VGPRs."""
    bad = []
    name = None
    for line in report.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            continue
        m = re.search(r"remark:\s+(ScratchSize \[bytes/lane\]|VGPRs Spill): (\d+)", line)
        if m and name and NO_SPILL.search(name) and int(m.group(2)) != 0:
            bad.append(f"{name}: {m.group(1)} = {m.group(2)}")
    if bad:
        raise RuntimeError("kernels with register-resident asynchronous loads must not spill:\n  " + "\n  ".join(bad))


def _compile(src: str, hipcc: str, verbose: bool) -> str:
    obj = _obj_of(src)
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-c", src, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n" + res.stdout + res.stderr)
    check_resource_report(res.stderr)
    with open(obj + ".resources.txt", "w") as f:       # kept beside the object for inspection
        f.write("\n".join(l for l in res.stderr.splitlines() if "remark:" in l and "Function Name" in l or
                          re.search(r"remark:\s+(VGPRs|AGPRs|ScratchSize|Occupancy|VGPRs Spill|SGPRs Spill|LDS Size)", l)))
    return obj


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 (all of them when `force`, otherwise only those
    older than a source or header) and link the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    todo = [s for s in srcs if force or _stale(_obj_of(s), [s] + _headers())]
    jobs = int(os.environ.get("MAX_JOBS", "8") or 8)
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, 16))) as pool:
        list(pool.map(lambda s: _compile(s, hipcc, verbose), todo))
    objs = [_obj_of(s) for s in srcs]
    if todo or _stale(LIB, objs):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + res.stdout + res.stderr)
    return LIB


if __name__ == "__main__":
    import sys
    print(build_library(force="--stale-only" not in sys.argv, verbose=True))
