"""Build the benchmark's measurement aid and its comparison program in-tree for gfx950.

Separate from the library's build: a failure here never fails the product."""

from __future__ import annotations

import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2511_06605_amd import build as dl_build  # noqa: E402

AID_LIB = os.path.join(HERE, "libdl_benchaid.so")
# the runtime's batched copy call under the ROCm installation's own HIP runtime
RUNTIME_BATCH = os.path.join(HERE, "dl_runtime_batch")


def build(verbose: bool = False) -> str:
    """The timing loops (linked against the library, which must have been built) and the comparison program."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    pkg = dl_build.HERE
    dl_build._run([hipcc, *dl_build.HIPCC_FLAGS, os.path.join(HERE, "dl_benchaid.hip"), "-L" + pkg, "-ldmalatte",
                   "-Wl,-rpath,$ORIGIN/../paper_2511_06605_amd", "-ldl", "-o", AID_LIB], verbose)
    rocm_lib = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(hipcc))), "lib")
    dl_build._run([hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wall", "-Wextra", "-Xclang", "-target-feature",
                   "-Xclang", "-packed-fp32-ops", os.path.join(HERE, "dl_runtime_batch.hip"),
                   "-Wl,-rpath," + rocm_lib, "-o", RUNTIME_BATCH], verbose)
    return AID_LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
