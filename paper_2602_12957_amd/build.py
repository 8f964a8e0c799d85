"""Builds libhsd.so (HIP, gfx950) in-tree with hipcc."""
import os
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libhsd.so")

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
    # hipcc -O3 must not form packed-fp32 instructions on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_library(verbose: bool = False, defines=(), out_path: str = LIB_PATH) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *[f"-D{d}" for d in defines], os.path.join(CSRC, "hsd_api.hip"), "-o", out_path + ".tmp"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    os.replace(out_path + ".tmp", out_path)
    if verbose:
        print("built", out_path)
    return out_path


if __name__ == "__main__":
    build_library(verbose=True)
