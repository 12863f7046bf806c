"""Build libbnn.so for gfx950 with hipcc, in-tree (paper_2301_05126_amd/libbnn.so)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ_DIR = os.path.join(ROOT, "_build", "libbnn")
LIB = os.path.join(PKG, "libbnn.so")

# (source, extra defines, object name)
UNITS = [("bnn_api.hip", [], "bnn_api.o"), ("bgemm.hip", [], "bgemm.o"), ("bconv.hip", [], "bconv.o"),
         ("bconv_small.hip", [], "bconv_small.o"),
         ("first_layer.hip", [], "first_layer.o"), ("elementwise.hip", [], "elementwise.o"),
         ("host_tools.hip", [], "host_tools.o")]
# the convolution kernels: per channel-word width, the 256 x 128 tile (part 1, slowest) apart
UNITS = [("bconv_inst.hip", [f"-DBNN_CONV_WPH={w}", "-DBNN_CONV_PART=1"], f"bconv_wph{w}_big.o")
         for w in (4, 2, 16, 8, 1)] + UNITS
UNITS += [("bconv_inst.hip", [f"-DBNN_CONV_WPH={w}", "-DBNN_CONV_PART=0"], f"bconv_wph{w}.o") for w in (1, 2, 4, 8, 16)]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # keep hipcc from forming packed-fp32 VALU ops (integer path; flag kept for all HIP code)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _compile(unit):
    src, defines, objname = unit
    obj = os.path.join(OBJ_DIR, objname)
    cmd = [HIPCC] + FLAGS + defines + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False) -> str:
    """Compile every HIP source and link the shared library.  Always recompiles."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(UNITS))) as ex:
        objs = list(ex.map(_compile, UNITS))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
