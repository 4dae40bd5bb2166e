"""Builds libqsync.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2407_02327_amd.build [--force]
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libqsync.so")
SOURCES = ["api.hip", "elementwise.hip", "gemm_mfma.hip", "gemm_f32.hip", "probe.hip", "indicator.hip"]

# -ffp-contract=off: the quantizer's multiply and subtract must stay separately rounded.
# packed fp32 VALU ops are disabled for the device pass (hipcc's host pass warns that it
# does not know the feature; that is harmless).
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-mllvm", "-pragma-unroll-threshold=262144",   # the 16x16 quantize patch must unroll fully
               "-Wno-unused-command-line-argument"]


# Kernels whose LDS reads are hand-written instructions with hand-placed waits: a register spill would store a
# result before it has arrived (the compiler does not know the instruction is a memory read), so these must
# build without any scratch memory.  Checked from the compiler's resource-usage remarks at every build.
NO_SPILL = {"gemm_mfma.hip": ("gemm_nt_kernel", "gemm_nt_persistent_kernel")}


def _check_no_spill(src: str, remarks: str) -> None:
    names = NO_SPILL.get(src)
    if not names:
        return
    current = None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            current = line.split("Function Name:")[1].split()[0]
        elif "ScratchSize [bytes/lane]:" in line and current and any(n in current for n in names):
            size = int(line.split("ScratchSize [bytes/lane]:")[1].split()[0])
            if size != 0:
                raise RuntimeError(f"{src}: kernel {current} uses {size} bytes of scratch per lane (register spills); "
                                   "its hand-waited LDS reads are not safe to spill")


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; cannot build libqsync.so")


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every kernel source for gfx950 and link libqsync.so next to this file."""
    hipcc = _hipcc()
    obj_dir = os.path.join(PKG_DIR, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    inc = os.path.join(os.path.dirname(PKG_DIR), "include")
    headers += [os.path.join(inc, f) for f in os.listdir(inc) if f.endswith(".h")]
    newest_header = max(os.path.getmtime(h) for h in headers)

    def compile_one(src: str) -> str:
        src_path = os.path.join(CSRC, src)
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        stale = (force or not os.path.exists(obj)
                 or os.path.getmtime(obj) < max(os.path.getmtime(src_path), newest_header))
        if stale:
            extra = ["-Rpass-analysis=kernel-resource-usage"] if src in NO_SPILL else []
            cmd = [hipcc, *HIPCC_FLAGS, *extra, "-c", src_path, "-o", obj]
            res = subprocess.run(cmd, capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError(f"hipcc failed for {src}:\n{res.stderr}")
            _check_no_spill(src, res.stderr)
            if verbose and res.stderr.strip():
                print(res.stderr, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    return LIB_PATH


def library_is_stale() -> bool:
    """True when any kernel source or header is newer than the built library."""
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h"))]
    inc = os.path.join(os.path.dirname(PKG_DIR), "include")
    deps += [os.path.join(inc, f) for f in os.listdir(inc) if f.endswith(".h")]
    return any(os.path.getmtime(d) > built for d in deps)


def ensure_built(rebuild_if_stale: bool = False) -> str:
    """Returns the library path, compiling it first when no library is there at all.  Tests and the smoke
    check load what is built; with `rebuild_if_stale` (the benchmark) a library older than any of its
    sources is rebuilt as well, and if that is impossible (no compiler) the call fails instead of timing
    stale code."""
    if not os.path.exists(LIB_PATH) or (rebuild_if_stale and library_is_stale()):
        return build(force=True)
    return LIB_PATH


if __name__ == "__main__":
    path = build(force="--force" in sys.argv, verbose=True)
    print(path)
