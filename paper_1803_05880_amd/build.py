"""Build libgg.so (the C-ABI library) in-tree with hipcc for gfx950."""
import glob
import hashlib
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libgg.so")
DIGEST_PATH = LIB_PATH + ".digest"      # digest of the sources the library on disk was built from

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    "-ffp-contract=off",            # every fp32 operation rounded on its own
    "-fno-gpu-flush-denormals-to-zero",   # denormals kept
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall",
    "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))


def source_digest():
    """sha256 over everything that determines the library: HIP sources, headers, compiler flags.
    The library reports the digest it was built from (gg_build_id)."""
    h = hashlib.sha256()
    h.update("\0".join(HIPCC_FLAGS).encode())
    files = sources() + sorted(glob.glob(os.path.join(HERE, "csrc", "*.h"))) + \
        sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    for path in files:
        h.update(os.path.basename(path).encode() + b"\0")
        h.update(open(path, "rb").read())
    return h.hexdigest()


def build_library(verbose=False):
    """Compile every HIP source into paper_1803_05880_amd/libgg.so.  Always compiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    digest = source_digest()
    cmd = [hipcc] + HIPCC_FLAGS + ['-DGG_BUILD_ID="%s"' % digest, "-I", os.path.join(ROOT, "include"),
                                   "-I", os.path.join(HERE, "csrc"), "-o", LIB_PATH] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed with exit code %d" % res.returncode)
    if verbose and res.stderr.strip():
        sys.stderr.write(res.stderr)
    with open(DIGEST_PATH, "w") as f:
        f.write(digest + "\n")
    return LIB_PATH


C_DRIVER_SRC = os.path.join(ROOT, "tests", "c_abi", "driver.c")
C_DRIVER_BIN = os.path.join(ROOT, "tests", "c_abi", "driver")


def build_c_driver(verbose=False):
    """Compile the plain-C caller of the ABI (tests/c_abi/driver.c) with gcc against libgg.so."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
           "-I", os.path.join(ROOT, "include"), C_DRIVER_SRC, "-o", C_DRIVER_BIN, "-L", HERE, "-lgg",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath,$ORIGIN/../../paper_1803_05880_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("gcc failed with exit code %d" % res.returncode)
    return C_DRIVER_BIN


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_c_driver(verbose=True))
