"""Compile the HIP sources into paper_2508_10395_amd/libxquant.so for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libxquant.so")
SOURCES = ["api.hip", "quantize.hip", "cl_accumulate.hip", "prepare_weights.hip", "remat_attn.hip",
           "latent_project.hip"]
HEADERS = ["common.hpp", "remat_layout.hpp", "unpack.hpp", "remat_common.hpp", "remat_epilogues.hpp", "remat_launch.hpp"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def needs_build():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, h) for h in HEADERS]
    deps.append(os.path.join(HERE, "..", "include", "xquant.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=True, verbose=False):
    """Build the library.  force=False skips when the library is newer than its sources."""
    if not force and not needs_build():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *sources(), "-o", LIB]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l)      # the host pass does not know the device feature
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
