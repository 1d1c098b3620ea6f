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


# Host-side sanitizer build (a checker's build, never what the product loads): AddressSanitizer and
# UndefinedBehaviorSanitizer on the host code only -- argument validation, plan selection, launch
# wrappers -- with the device code compiled as usual.
SAN_OBJ = os.path.join(PKG, "_build_san")
SAN_LIB = os.path.join(SAN_OBJ, "libltn_attn_san.so")
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-omit-frame-pointer", "-Xarch_host", "-fno-sanitize-recover=undefined"]


def _obj_of(src: str, objdir: str = OBJ) -> str:
    return os.path.join(objdir, os.path.basename(src) + ".o")


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


def _compile(src: str, hipcc: str, verbose: bool, objdir: str = OBJ, extra=()) -> str:
    obj = _obj_of(src, objdir)
    cmd = [hipcc] + HIPCC_FLAGS + list(extra) + ["-I", os.path.join(ROOT, "include"), "-c", src, "-o", obj]
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


def sanitizer_runtime() -> str:
    """Path of the shared AddressSanitizer runtime of the compiler that hipcc drives."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    res = subprocess.run([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = res.stdout.strip()
    if not os.path.isabs(path):
        cands = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
        path = cands[0] if cands else ""
    return path


def build_sanitized(verbose: bool = False) -> str:
    """The same sources with ASan + UBSan on the host code, linked against the shared sanitizer
    runtime, into _build_san/ (only what is stale is recompiled)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(SAN_OBJ, exist_ok=True)
    srcs = sources()
    todo = [s for s in srcs if _stale(_obj_of(s, SAN_OBJ), [s] + _headers())]
    jobs = int(os.environ.get("MAX_JOBS", "8") or 8)
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, 16))) as pool:
        list(pool.map(lambda s: _compile(s, hipcc, verbose, SAN_OBJ, SAN_FLAGS), todo))
    objs = [_obj_of(s, SAN_OBJ) for s in srcs]
    if todo or _stale(SAN_LIB, objs):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
               "-shared-libsan"] + objs + ["-o", SAN_LIB]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("sanitizer link failed:\n" + res.stdout + res.stderr)
    return SAN_LIB


if __name__ == "__main__":
    import sys
    print(build_library(force="--stale-only" not in sys.argv, verbose=True))
