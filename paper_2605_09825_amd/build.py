"""Build libmxfp4.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmxfp4.so")
SOURCES = ["api.hip", "quantize.hip", "quantize_fp8.hip", "gemm.hip"]

# -ffp-contract=off: the quantiser's fp32 butterflies must round after every operation.
# The -target-feature pair switches packed-fp32 code generation off (device pass only; the
# host pass prints a harmless "not a recognized feature" note).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-fno-fast-math", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the MXFP4 library cannot be built")
    return exe


# MXFP4_SANITIZE_HOST=1: an AddressSanitizer + UndefinedBehaviorSanitizer build of the HOST side of the library
# (argument checks, layouts, launch logic; device code is not instrumented) as libmxfp4_san.so, which the
# binding then loads instead.  Run the CPU-only tests against it with the clang ASan runtime preloaded:
#   MXFP4_SANITIZE_HOST=1 LD_PRELOAD=$(ls /opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so) \
#       ASAN_OPTIONS=detect_leaks=0 python -m pytest tests/test_abi.py -q
SANITIZE_HOST = os.environ.get("MXFP4_SANITIZE_HOST", "") not in ("", "0")
if SANITIZE_HOST:
    LIB = os.path.join(HERE, "libmxfp4_san.so")
    FLAGS = [f for f in FLAGS if f != "-O3"] + ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
                                                "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


def _run(cmd) -> str:
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    return err


def build(verbose: bool = False) -> str:
    """Compile every HIP source into paper_2605_09825_amd/libmxfp4.so (always recompiles): the sources side by
    side into objects in a scratch folder, then one link."""
    import concurrent.futures
    import tempfile
    cc = hipcc()
    compile_flags = [f for f in FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="mxfp4_build_") as tmp:
        objs = [os.path.join(tmp, s.replace(".hip", ".o")) for s in SOURCES]
        cmds = [[cc] + compile_flags + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
        with concurrent.futures.ThreadPoolExecutor(max_workers=len(cmds)) as pool:
            errs = list(pool.map(_run, cmds))
        errs.append(_run([cc] + FLAGS + objs + ["-o", LIB]))
    if verbose and any(e.strip() for e in errs):
        print("\n".join(e for e in errs if e.strip()))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
