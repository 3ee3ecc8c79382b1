"""Build the C-ABI library libqoq_w4a8.so from csrc/*.hip with hipcc for gfx950.

Usage: python -m paper_2405_04532_amd.build   (cross-compiles; no GPU needed)
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libqoq_w4a8.so")
SOURCES = ["qoq_api.hip", "qoq_pack.hip", "qoq_act.hip", "qoq_gemm.hip", "qoq_kv4.hip", "qoq_transforms.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed FP32 instructions off (they have produced wrong results on these machines)
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src, extra):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = ["hipcc", "-c", os.path.join(CSRC, src), "-o", obj, "-save-temps=obj"] + FLAGS + extra
    subprocess.check_call(cmd)
    _check_device_asm(os.path.join(OBJ, src.replace(".hip", "-hip-amdgcn-amd-amdhsa-gfx950.s")))
    return obj


def _check_device_asm(path):
    """Refuse kernels that read the dispatch packet.  The compiler does that when it moves an indexed per-thread
    array into LDS (it then needs the workgroup size and all three thread ids); the packet lives in host-visible
    queue memory, and the scalar load from it was measured to cost every workgroup several microseconds."""
    if not os.path.exists(path):
        return
    kernel = None
    for line in open(path):
        t = line.strip()
        if t.startswith(".amdhsa_kernel "):
            kernel = t.split()[1]
        elif t == ".amdhsa_user_sgpr_dispatch_ptr 1":
            raise RuntimeError(f"{kernel} reads the dispatch packet: an indexed private array was moved to LDS")


def build(extra_flags=(), verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    extra = list(extra_flags)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra), SOURCES))
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(sys.argv[1:], verbose=True)
