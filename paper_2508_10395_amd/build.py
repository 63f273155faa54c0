"""Compile the HIP sources into paper_2508_10395_amd/libxquant.so for gfx950."""
import hashlib
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libxquant.so")
SOURCES = ["api.hip", "quantize.hip", "cl_accumulate.hip", "prepare_weights.hip", "remat_attn.hip",
           "remat_attn16.hip", "latent_project.hip"]
HEADERS = ["common.hpp", "remat_layout.hpp", "unpack.hpp", "remat_common.hpp", "remat_epilogues.hpp", "remat_launch.hpp"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function",
         # the LDS-DMA asm names M0 in its clobber list; M0 is a reserved register, which clang remarks on
         "-Wno-inline-asm"]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


STAMP = os.path.join(HERE, "libxquant.srchash")      # digest of the sources the library was built from


def _deps():
    deps = sources() + [os.path.join(CSRC, h) for h in HEADERS]
    deps.append(os.path.join(HERE, "..", "include", "xquant.h"))
    return deps


def source_digest():
    """SHA-256 over the flags and every source and header, in a fixed order (file times do not survive every copy)."""
    h = hashlib.sha256(" ".join(FLAGS).encode())
    for d in _deps():
        h.update(os.path.basename(d).encode())
        with open(d, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def needs_build():
    """True when there is no library, or it was built from other sources than the ones in the tree."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as f:
        return f.read().strip() != source_digest()


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l)      # the host pass does not know the device feature
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(force=True, verbose=False):
    """Build the library.  force=False skips when the library was built from the sources in the tree.
    The translation units are compiled side by side (objects under _build/, which is not committed), then linked."""
    if not force and not needs_build():
        return LIB
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]
    objs = [os.path.join(objdir, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
        list(pool.map(lambda so: _run([hipcc, *compile_flags, "-c", so[0], "-o", so[1]], verbose), zip(sources(), objs)))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], verbose)
    with open(STAMP, "w") as f:
        f.write(source_digest() + "\n")
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
