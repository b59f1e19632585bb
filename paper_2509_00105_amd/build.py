"""Build the HIP library (libkvh.so) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvh.so")
SOURCES = ["kvh_api.hip", "kvh_decode.hip", "kvh_encode.hip", "kvh_transcode.hip", "kvh_loader.hip", "kvh_policy.cpp"]

# -ffp-contract=off: the codec's arithmetic fuses only where the source says fma.
# -fno-honor-nans: inputs are finite by contract; without it every min/max of a value unpacked with
# integer ops is preceded by a canonicalising v_max (sNaN quieting).
# packed-fp32-ops off: hipcc must not form v_pk_*_f32 from the scalar float code.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-fno-honor-nans",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc, *HIPCC_FLAGS, "-o", tmp, *[os.path.join(CSRC, s) for s in SOURCES]]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    out = "\n".join(ln for ln in res.stdout.splitlines() if noise not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
