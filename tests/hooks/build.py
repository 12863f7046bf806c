"""Build tests/hooks/libbnn_test_hooks.so (test infrastructure; needs libbnn.so built first)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
PKG = os.path.join(ROOT, "paper_2301_05126_amd")
LIB = os.path.join(HERE, "libbnn_test_hooks.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build() -> str:
    cmd = [HIPCC, "--offload-arch=gfx950", "-O2", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(PKG, "csrc"),
           os.path.join(HERE, "conv_tiles_hook.hip"), "-o", LIB,
           "-L" + PKG, "-lbnn", "-Wl,-rpath,$ORIGIN/../../paper_2301_05126_amd"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("test hook build failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build())
