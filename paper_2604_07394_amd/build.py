"""Build the HIP libraries in-tree for gfx950 (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "lib")

# packed fp32 VALU instructions are disabled on purpose (target feature -packed-fp32-ops)
COMMON = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]

FLUX_SOURCES = ["flux_api.hip", "kv_append.hip", "decode.hip", "prefill.hip", "router.hip", "xa_select.hip"]


def _run(cmd):
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), err))
    return err


def build_all(verbose: bool = False) -> None:
    os.makedirs(LIB, exist_ok=True)
    inc = ["-I" + os.path.join(ROOT, "include")]
    out = _run(COMMON + inc + [os.path.join(CSRC, s) for s in FLUX_SOURCES] + ["-o", os.path.join(LIB, "libflux.so")])
    if verbose and out:
        print(out)
    out = _run(COMMON + ["-ffp-contract=off", os.path.join(CSRC, "synth_fill.hip"), "-o",
                         os.path.join(LIB, "libflux_synth.so")])
    if verbose and out:
        print(out)
    build_hostcheck(verbose)


# The C ABI's host side (argument validation, workspace arithmetic, the sink / window rounding) built once more as
# plain C++ under AddressSanitizer and UndefinedBehaviorSanitizer, with launchers that report "no device", and a
# small driver that calls every entry point with ordinary and extreme arguments.  No GPU is needed to run it.
SAN = ["-O1", "-g", "-std=c++17", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"


def build_hostcheck(verbose: bool = False) -> None:
    inc = ["-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
    out = _run([CLANGXX, "-x", "c++", "-D__HIP_PLATFORM_AMD__"] + inc + SAN + ["-fPIC", "-shared",
               os.path.join(CSRC, "flux_api.hip"), os.path.join(CSRC, "hostcheck_stubs.cpp"), "-L/opt/rocm/lib", "-lamdhip64",
               "-Wl,-rpath,/opt/rocm/lib", "-o", os.path.join(LIB, "libflux_hostcheck.so")])
    out += _run([CLANGXX] + SAN + [os.path.join(CSRC, "hostcheck_main.cpp"), "-L" + LIB, "-lflux_hostcheck",
                "-Wl,-rpath,$ORIGIN", "-Wl,-rpath,/opt/rocm/lib", "-o", os.path.join(LIB, "flux_hostcheck")])
    if verbose and out:
        print(out)


if __name__ == "__main__":
    build_all(verbose=True)
    print("built", os.listdir(LIB))
