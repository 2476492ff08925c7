"""Builds libpp.so (the gfx950 HIP library) in-tree with hipcc."""
import glob
import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
# PP_LIBPP selects another build of the library (experiments); the default is the in-tree one
LIB_PATH = os.environ.get("PP_LIBPP") or os.path.join(_PKG, "libpp.so")

HIPCC_FLAGS = [
    "-fPIC", "--offload-arch=gfx950", "-O3", "-std=c++17",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]
OBJ_DIR = os.path.join(_ROOT, "_build")


def sources():
    return sorted(glob.glob(os.path.join(_PKG, "csrc", "*.hip")))


def _headers():
    return glob.glob(os.path.join(_PKG, "csrc", "*.h")) + glob.glob(os.path.join(_ROOT, "include", "*.h"))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build_libpp(verbose=False, incremental=False):
    """Compile every HIP source under csrc/ (one hipcc per file, side by side) and link them
    into paper_2204_10562_amd/libpp.so.  incremental=True keeps objects newer than their
    source and every header."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    inc = ["-I", os.path.join(_ROOT, "include"), "-I", os.path.join(_PKG, "csrc")]
    newest_header = max(os.path.getmtime(h) for h in _headers())
    jobs, objs = [], []
    for src in sources():
        obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        fresh = (incremental and os.path.exists(obj)
                 and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header))
        if not fresh:
            jobs.append([hipcc, "-c"] + HIPCC_FLAGS + inc + [src, "-o", obj])
    workers = max(1, min(len(jobs), os.cpu_count() or 1, 8))
    with ThreadPoolExecutor(workers) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "-shared"] + HIPCC_FLAGS + objs + ["-o", LIB_PATH], verbose)
    return LIB_PATH


CALIB_PATH = os.path.join(_PKG, "libpp_calib.so")


def build_calib(verbose=False):
    """Compile the benchmark's calibration kernels (csrc/calib/) into libpp_calib.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    src = os.path.join(_PKG, "csrc", "calib", "pp_calib.hip")
    _run([hipcc, "-shared"] + HIPCC_FLAGS + [src, "-o", CALIB_PATH], verbose)
    return CALIB_PATH


if __name__ == "__main__":
    import sys
    print(build_libpp(verbose=True, incremental="--incremental" in sys.argv))
    print(build_calib(verbose=True))
