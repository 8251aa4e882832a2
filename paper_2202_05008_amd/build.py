"""Build the gfx950 shared library (libevo_gfx950.so) in-tree with hipcc.

    python -m paper_2202_05008_amd.build

Every csrc/*.hip and csrc/*.cpp is compiled for gfx950 only and linked into one C-ABI
library next to this file.  hipcc cross-compiles, so no GPU is needed to build.
"""
import glob
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libevo_gfx950.so")

HIPCC = os.environ.get("HIPCC") or shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Wall", "-Wno-unused-function",
    # packed fp32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(os.path.dirname(HERE), "include"),
]


# Extra flags of single files.  The matrix accumulators of these kernels are consumed by vector instructions
# right after the products, so they are kept in the vector half of the register file; otherwise every value
# costs one move out of the accumulation registers before its epilogue.  Measured on one box: the
# register-resident bf16 kernel 1.61 -> 1.48 ms at 2048 observations per member (the streaming kernel
# unchanged), the cart-pole roll-out 1.38 -> 1.30 ms; the LSTM kernel does not change and the ConvNet kernel has
# no such moves, so they are left alone.
_VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form"]
FILE_FLAGS = {"policy_bf16.hip": _VGPR_FORM, "task_cartpole.hip": _VGPR_FORM, "probe.hip": _VGPR_FORM}


def _compile(src, build_dir=BUILD, extra_flags=()):
    obj = os.path.join(build_dir, os.path.basename(src) + ".o")
    cmd = [HIPCC, *FLAGS, *extra_flags, *FILE_FLAGS.get(os.path.basename(src), []), "-c", src, "-o", obj]
    if src.endswith(".cpp"):
        cmd[1:1] = ["-x", "hip"]
    if src.endswith(".c"):      # a plain C caller of the C ABI: host compiler only
        cmd = [HIPCC, "-x", "c", "-O1", "-g", *extra_flags, "-I", os.path.join(os.path.dirname(HERE), "include"),
               "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    warn = [l for l in r.stderr.splitlines() if "warning" in l and "packed-fp32-ops" not in l]
    return obj, warn


def build(verbose=True, jobs=8):
    os.makedirs(BUILD, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))
    if not srcs:
        raise RuntimeError("no sources under %s" % CSRC)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        results = list(ex.map(_compile, srcs))
    objs = [o for o, _ in results]
    if verbose:
        for _, warn in results:
            for w in warn:
                print(w, file=sys.stderr)
    tmp = LIB + ".tmp"
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    os.replace(tmp, LIB)
    if verbose:
        print("built %s from %d sources" % (LIB, len(srcs)))
    return LIB


# Host-side sanitizers (the device code is compiled as always): every -fsanitize= goes to the host pass only.
HOST_SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


def build_checked_executable(driver_c, out, build_dir, jobs=8):
    """The library's sources plus one C driver, host code under AddressSanitizer and UndefinedBehaviorSanitizer,
    linked into the executable `out` (used by the CPU tests; no GPU needed to build or to run the host paths)."""
    os.makedirs(build_dir, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = [o for o, _ in ex.map(lambda s: _compile(s, build_dir, HOST_SANITIZE), srcs)]
    drv, _ = _compile(driver_c, build_dir, ["-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined",
                                            "-fno-sanitize-recover=undefined"])
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined",
                        "-o", out, drv, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    return out


if __name__ == "__main__":
    build()
