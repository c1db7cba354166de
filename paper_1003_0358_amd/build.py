"""Build libdbsn.so (HIP, gfx950) in-tree with hipcc."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libdbsn.so")
SOURCES = [os.path.join(CSRC, "dbsn.hip")]
HEADERS = [os.path.join(CSRC, h) for h in ("dbsn_plan.h", "dbsn_rng.h", "dbsn_mlp_kernels.h", "dbsn_deform_kernels.h",
                                           "dbsn_persistent_kernel.h", "dbsn_batch_kernels.h",
                                           "dbsn_reduce_kernels.h", "dbsn_probe_kernels.h")] + \
          [os.path.join(ROOT, "include", "dbsn.h")]


def hipcc_command(out=LIB):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
            # keep the compiler from forming packed fp32 instructions
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            # keep identical stores in different switch cases apart: merged, they index the weight
            # registers of the persistent kernel dynamically, which sends them to scratch memory
            "-mllvm", "-simplifycfg-sink-common=false",
            "-I", os.path.join(ROOT, "include"), "-I", CSRC, *SOURCES, "-o", out]


def build(verbose=False):
    cmd = hipcc_command()
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


def up_to_date():
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    return all(os.path.getmtime(f) <= t for f in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build(verbose=True))
