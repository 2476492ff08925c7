"""Builds libpp.so (the gfx950 HIP library) in-tree with hipcc."""
import glob
import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
# PP_LIBPP selects another build of the library (experiments); the default is the in-tree one
LIB_PATH = os.environ.get("PP_LIBPP") or os.path.join(_PKG, "libpp.so")

HIPCC_FLAGS = [
    "-shared", "-fPIC", "--offload-arch=gfx950", "-O3", "-std=c++17",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(_PKG, "csrc", "*.hip")))


def build_libpp(verbose=False):
    """Compile every HIP source under csrc/ into paper_2204_10562_amd/libpp.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(_ROOT, "include"),
                                   "-I", os.path.join(_PKG, "csrc")] + sources() + ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB_PATH


if __name__ == "__main__":
    print(build_libpp(verbose=True))
