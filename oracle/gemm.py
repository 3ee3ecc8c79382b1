"""Loader for the plain-C int64 GEMM of the CPU oracle (TEST INFRASTRUCTURE ONLY).

`build()` compiles oracle/gemm_i64.c with gcc; `gemm_i64` calls it through ctypes.
The forward helpers below chain the oracle's own quantizers, this GEMM and the FP64
epilogue in the order the paper states them (Sections 4.1, 5.1, 5.2.2).
"""
import ctypes
import os
import subprocess

import numpy as np

from . import qoq_quant as qq

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_i64.c")
_LIB = os.path.join(_HERE, "libqoq_oracle.so")
_lib = None


def build(force=True):
    """Compile the C part of the oracle (gcc -O2 -fopenmp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", _LIB])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_gemm_i8_i64.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
        _lib.oracle_gemm_i8_i64.restype = None
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def gemm_i64(qx, w_hat):
    """acc[m, n] = sum_k qx[m, k] * w_hat[n, k]; operands must fit INT8, sums are int64."""
    qx = np.asarray(qx)
    w_hat = np.asarray(w_hat)
    assert qx.min(initial=0) >= -128 and qx.max(initial=0) <= 127
    assert w_hat.min(initial=0) >= -128 and w_hat.max(initial=0) <= 127
    a = np.ascontiguousarray(qx, dtype=np.int8)
    b = np.ascontiguousarray(w_hat, dtype=np.int8)
    m, k = a.shape
    n, k2 = b.shape
    assert k == k2
    acc = np.empty((m, n), dtype=np.int64)
    if m and n:
        _load().oracle_gemm_i8_i64(a.ctypes.data, b.ctypes.data, acc.ctypes.data, m, n, k)
    return acc


def forward_group(w_fp16, x_fp16, group=qq.GROUP):
    """Whole per-group W4A8 path on FP16 inputs: progressive weight quantization,
    per-token activation quantization, INT8 GEMM, FP16 epilogue."""
    wq = qq.progressive_quant(w_fp16, group)
    qx, sx, rowsum, tx = qq.act_quant(x_fp16)
    acc = gemm_i64(qx, wq["w_hat"])
    assert np.abs(acc).max(initial=0) < 2 ** 31
    return dict(wq=wq, qx=qx, sx=sx, rowsum=rowsum, tx=tx, acc=acc,
                out64=qq.output_fp64(acc, sx, wq["s0"]), out=qq.output_fp16(acc, sx, wq["s0"]))


def forward_per_channel(w_fp16, x_fp16):
    """Whole per-channel W4A8 path (Section 5.2.2) with the exact integer zero fold."""
    code, z, sw = qq.per_channel_quant(w_fp16)
    qx, sx, rowsum, tx = qq.act_quant(x_fp16)
    raw = gemm_i64(qx, code)
    acc = qq.per_channel_acc(raw, z, rowsum)
    assert np.abs(acc).max(initial=0) < 2 ** 31
    return dict(Q=code, z=z, sw=sw, qx=qx, sx=sx, rowsum=rowsum, tx=tx, raw=raw, acc=acc,
                out64=qq.output_fp64(acc, sx, sw), out=qq.output_fp16(acc, sx, sw))
