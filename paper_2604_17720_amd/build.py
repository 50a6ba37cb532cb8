"""Builds libflashfps.so (HIP, gfx950) in-tree with hipcc.

build(profile=True) builds libflashfps_prof.so instead: the same sources with
-DFFPS_PROFILE, whose multi-pick kernels time the phases of a round and leave
the counters in the workspace's status block (read by profile_phases.py)."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libflashfps.so")
LIB_PROFILE = os.path.join(HERE, "libflashfps_prof.so")
SOURCES = ["api.hip", "fps_wg.hip", "fps_grid.hip", "fps_stream.hip", "aux.hip"]
HEADERS = ["fps_device.h", "fps_launch.h", "fps_exchange.h"]

# -ffp-contract=off: a fused multiply-add would change the low bits of the
# squared distance and therefore the picks.
# -target-feature -packed-fp32-ops: the device pass must not form packed fp32
# instructions.  The driver hands the switch to the host pass as well, which
# does not know it and says so once per function; that line is dropped from
# the output below, and check_no_packed_fp32() proves on the device assembly
# that the device pass honoured the switch.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]
_HOST_PASS_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"
_PACKED_FP32 = re.compile(r"\bv_pk_(add|mul|fma)_f32\b")
# Integer instructions with reversed operands in their DPP form (the compiler folds a
# lane permutation into them when the permuted value is the subtrahend or the shift
# count).  The reversed subtractions were seen to permute the other operand on
# gfx950; the shifts were not tried.  The kernels avoid all of them.
_REVERSED_INT_DPP = re.compile(r"\bv_(subrev|subbrev)_(co_)?[iu]32_dpp\b|\bv_(lshlrev|lshrrev|ashrrev)_\w+_dpp\b")


def _hipcc() -> str:
    for c in ("/opt/rocm/bin/hipcc", "hipcc"):
        if os.path.sep not in c or os.path.exists(c):
            return c
    return "hipcc"


def _finish(cmd, proc) -> None:
    """Waits for a compiler process, forwards what it printed except the host
    pass's note about the device-only feature, raises on failure."""
    _, err = proc.communicate()
    for line in err.decode(errors="replace").splitlines():
        if line.strip() != _HOST_PASS_NOTE:
            print(line, file=sys.stderr)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd))


def check_no_packed_fp32(extra_flags=()) -> None:
    """Compiles the device side of every source to assembly and raises if a
    packed fp32 add, multiply or fused multiply-add was generated, or an integer
    instruction with reversed operands in DPP form."""
    procs = []
    for s in SOURCES:
        cmd = [_hipcc(), *FLAGS, *extra_flags, "--cuda-device-only", "-S", os.path.join(CSRC, s),
               "-o", "-"]
        procs.append((s, cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE)))
    for s, cmd, p in procs:
        out, err = p.communicate()
        if p.returncode != 0:
            sys.stderr.write(err.decode(errors="replace"))
            raise RuntimeError("hipcc failed: " + " ".join(cmd))
        text = out.decode(errors="replace")
        hit = _PACKED_FP32.search(text)
        if hit:
            raise RuntimeError(f"{s}: the device pass generated {hit.group(0)}; "
                               "packed fp32 instructions must stay off")
        hit = _REVERSED_INT_DPP.search(text)
        if hit:
            raise RuntimeError(f"{s}: the device pass generated {hit.group(0)}; write the operation "
                               "so that the permuted operand comes first")


def build(force: bool = True, verbose: bool = False, profile: bool = False) -> str:
    """Compile every HIP source for gfx950 and link the shared library.
    With force=False an up-to-date library is reused."""
    lib = LIB_PROFILE if profile else LIB
    extra = ["-DFFPS_PROFILE"] if profile else []
    suffix = ".prof.o" if profile else ".o"
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    deps = srcs + [os.path.join(CSRC, h) for h in HEADERS] + \
        [os.path.join(HERE, "..", "include", "flashfps.h")]
    if not force and os.path.exists(lib) and \
            all(os.path.getmtime(lib) >= os.path.getmtime(d) for d in deps):
        return lib
    objs = []
    procs = []
    for s in srcs:
        o = s[:-4] + suffix
        objs.append(o)
        cmd = [_hipcc(), *FLAGS, *extra, "-c", s, "-o", o]
        if verbose:
            print(" ".join(cmd))
        procs.append((cmd, subprocess.Popen(cmd, stderr=subprocess.PIPE)))
    for cmd, p in procs:
        _finish(cmd, p)
    check_no_packed_fp32(extra)
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    subprocess.check_call(cmd)
    return lib


if __name__ == "__main__":
    print(build(force=True, verbose=True, profile="--profile" in sys.argv[1:]))
