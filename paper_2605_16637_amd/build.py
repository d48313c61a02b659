"""Builds the C-ABI library ``libhx.so`` (and the benchmark's calibration kernels,
``libhx_calib.so``) from the HIP sources, in-tree, for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhx.so")
CALIB_LIB = os.path.join(HERE, "libhx_calib.so")      # the benchmark's calibration kernels, a library of their own
SOURCES = ["hx_ctx.hip", "hx_score.hip", "hx_dag.hip", "hx_plan.hip", "hx_decode.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                       # every fused multiply-add is an explicit fmaf
    # no arithmetic ever sees a NaN, so min/max need no quieting: the one NaN the library writes (the ratio of a call
    # whose node or workflow index is out of range) is chosen among integers and stored as bits, never computed with
    "-fno-honor-nans",
    # no packed fp32 instructions.  A device feature; the flag cannot be routed to the device pass alone (-Xarch_device
    # takes no option with an argument), and the host pass answers with a notice that build() drops from the log
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


# host-side AddressSanitizer + UndefinedBehaviorSanitizer (device code cannot be sanitized here): each option
# directly after -Xarch_host
HOST_SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]


def build(verbose: bool = False, out: str = LIB, extra_flags=()) -> str:
    if out == LIB:
        _compile(["hipcc", *FLAGS, "-o", CALIB_LIB, os.path.join(CSRC, "hx_calib.hip")], verbose)
    return _compile(["hipcc", *FLAGS, *extra_flags, "-o", out, *[os.path.join(CSRC, s) for s in SOURCES]], verbose, out)


def _compile(cmd, verbose, out=None) -> str:
    if verbose:
        print(" ".join(cmd))
    run = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    notice = "'-packed-fp32-ops' is not a recognized feature for this target"
    lines = run.stdout.splitlines()
    rest = [l for l in lines if notice not in l]
    if rest:
        print("\n".join(rest))
    if verbose and len(rest) != len(lines):
        print("(%d host-pass notices dropped: -packed-fp32-ops is a device feature, the host target does not know it)"
              % (len(lines) - len(rest)))
    if run.returncode:
        raise subprocess.CalledProcessError(run.returncode, cmd)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
