"""Build libabl.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libabl.so")

# every HIP translation unit: no packed-fp32 instructions (they have misbehaved on the test machines)
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-variable",
          "-Wno-unused-but-set-variable",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]

# translation unit -> extra flags.  The quantizer must round every fp32 operation on its own
# (the codes are compared bit for bit with an IEEE evaluation), so no fused multiply-add there.
UNITS = {
    "bn_kernels.hip": ["-ffp-contract=off"],
    "conv_kernels.hip": [],
    "conv_halo.hip": ["-ffp-contract=off"],
    "conv_pointwise.hip": ["-ffp-contract=off"],
    "conv_bf16.hip": [],
    "conv_image.hip": ["-ffp-contract=off"],
    "abl_api.hip": [],
    "abl_noalloc.hip": [],
    "probe_kernels.hip": [],
}


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True, only=None) -> str:
    """Compile every translation unit (or, with `only`, just the named ones, reusing the other
    object files of an earlier build) and link libabl.so."""
    cc = hipcc()
    objs = []
    procs = []
    for unit, extra in UNITS.items():
        src = os.path.join(CSRC, unit)
        obj = os.path.join(CSRC, unit.replace(".hip", ".o"))
        objs.append(obj)
        if only and unit.replace(".hip", "") not in only and os.path.exists(obj):
            continue
        cmd = [cc, *COMMON, *extra, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((unit, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for unit, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (unit, out))
        if verbose and out:
            print(out, flush=True)
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(only=[a for a in sys.argv[1:] if not a.startswith("-")] or None)
    sys.exit(0)
