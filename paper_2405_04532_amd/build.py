"""Build the C-ABI library libqoq_w4a8.so (and the benchmark's read probe libqoq_probe.so) from csrc/*.hip with hipcc for gfx950.

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
PROBE_LIB = os.path.join(HERE, "libqoq_probe.so")     # measurement probes of the benchmark (plain streaming read, matrix-core ceiling)
SOURCES = ["qoq_api.hip", "qoq_pack.hip", "qoq_act.hip", "qoq_gemm.hip", "qoq_gemm_astat.hip", "qoq_kv4.hip", "qoq_transforms.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed FP32 instructions off (they have produced wrong results on these machines)
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src, extra):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = ["hipcc", "-c", os.path.join(CSRC, src), "-o", obj, "-save-temps=obj"] + FLAGS + extra
    subprocess.check_call(cmd)
    _check_device_asm(os.path.join(OBJ, src.replace(".hip", "-hip-amdgcn-amd-amdhsa-gfx950.s")))
    if src == "qoq_gemm_astat.hip":
        _check_astat_prologue(os.path.join(OBJ, src.replace(".hip", "-hip-amdgcn-amd-amdhsa-gfx950.s")))
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


def _check_astat_prologue(path):
    """The activation-stationary kernels wait for their global->LDS copies with hand-written counts that include the
    weight loads the compiler emits between two markers; refuse a build in which that number is not the one the
    kernel's source assumes (R * J units, two loads each in group mode, one in per-channel mode)."""
    import re
    if not os.path.exists(path):
        return
    kernel, counting, count, seen = None, False, 0, 0
    for line in open(path):
        t = line.strip()
        m = re.match(r"(_ZN3qoq\S*astat_kernelILi(\d+)ELi(\d+)ELi(\d+)ELb([01])ELi(\d+)E\S*):", t)
        if m:
            kernel = (m.group(1), int(m.group(3)) * int(m.group(4)) * (2 if m.group(5) == "1" else 1))
        elif "astat weight prologue begin" in t:
            counting, count = True, 0
        elif "astat weight prologue end" in t:
            counting = False
            seen += 1
            if kernel is None or count != kernel[1]:
                raise RuntimeError(f"{kernel}: {count} loads in the weight prologue, the wait counts assume {kernel and kernel[1]}")
        elif counting and (t.startswith("global_load") or t.startswith("flat_load") or t.startswith("buffer_load") or
                           t.startswith("global_store") or t.startswith("flat_store")):
            count += 1
    if seen == 0:
        raise RuntimeError("no activation-stationary kernel found in " + path)


def build(extra_flags=(), verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    extra = list(extra_flags)
    with ThreadPoolExecutor(max_workers=7) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra), SOURCES))
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    subprocess.check_call(["hipcc", "-shared", os.path.join(CSRC, "probe_read.hip"), os.path.join(CSRC, "probe_mfma.hip"),
                           "-o", PROBE_LIB] + FLAGS + extra)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(sys.argv[1:], verbose=True)
