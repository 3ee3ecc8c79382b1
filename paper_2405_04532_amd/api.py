"""Thin ctypes binding of libqoq_w4a8.so (same names as include/qoq_w4a8.h).

Argument marshalling only: torch owns device memory and streams, every step of the path
runs in the library's HIP kernels.  There is no fallback: if the library is not built or
a call fails, an exception is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqoq_w4a8.so")

QOQ_GROUP128 = 0
QOQ_PER_CHANNEL = 1
# qoq_status
QOQ_OK, QOQ_ERR_NULL, QOQ_ERR_SHAPE, QOQ_ERR_ALIGN, QOQ_ERR_BLOB, QOQ_ERR_WORKSPACE, QOQ_ERR_ARCH, QOQ_ERR_HIP = range(8)
GROUP = 128

_lib = None

_SIGNATURES = {
    "qoq_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "qoq_packed_bytes": (ctypes.c_size_t, [ctypes.c_int64, ctypes.c_int64, ctypes.c_int]),
    "qoq_gemm_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]),
    "qoq_gemm_workspace_prepare": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "qoq_pack_weights": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                        ctypes.c_void_p, ctypes.c_void_p]),
    "qoq_pack_quantized": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p,
                                          ctypes.c_void_p]),
    "qoq_unpack_weights": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p]),
    "qoq_quant_act_per_token": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "qoq_w4a8_gemm": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                     ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "qoq_w4a8_gemm_noalloc": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                             ctypes.c_void_p, ctypes.c_void_p]),
    "qoq_w4a8_gemm_i32": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "qoq_rmsnorm_quant": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double, ctypes.c_int64, ctypes.c_int64,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p]),
    "qoq_silu_mul_quant": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "qoq_w4a8_gemm_token_sum": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                               ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "qoq_w4a8_linear": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                       ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "qoq_set_gemm_config": (ctypes.c_int, [ctypes.c_int, ctypes.c_int]),
    "qoq_query_gemm_config": (ctypes.c_int, [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                             ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]),
    "qoq_channel_absmax": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]),
    "qoq_channel_order_host": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]),
    "qoq_gather_channels": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                           ctypes.c_void_p]),
    "qoq_quant_act_per_token_reordered": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                                         ctypes.c_void_p]),
    "qoq_hadamard_rotate": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                           ctypes.c_void_p]),
    "qoq_kv4_cache_bytes": (ctypes.c_size_t, [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]),
    "qoq_kv4_append": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                      ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]),
    "qoq_kv4_attention_decode": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                                ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                                ctypes.c_void_p, ctypes.c_void_p]),
    "qoq_kv4_attention_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                                            ctypes.c_int64]),
    "qoq_kv4_attention_decode_split": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                                      ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "qoq_kv4_unpack": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.c_void_p]),
}

EXPORTS = tuple(_SIGNATURES)


class QoqError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(message)
        self.status = status


def lib():
    """Load the built library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2405_04532_amd.build` first")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def status_string(status):
    return lib().qoq_status_string(int(status)).decode()


def _check(status):
    if status != 0:
        raise QoqError(status, status_string(status))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(device):
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def _dev(t, dtype, name):
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous {dtype} tensor on the GPU")
    return t


def packed_bytes(N, K, mode=QOQ_GROUP128):
    return int(lib().qoq_packed_bytes(N, K, mode))


def gemm_workspace_bytes(M, N, K, mode=QOQ_GROUP128):
    return int(lib().qoq_gemm_workspace_bytes(M, N, K, mode))


def set_gemm_config(tile_m=0, split_k=0):
    _check(lib().qoq_set_gemm_config(tile_m, split_k))


def query_gemm_config(M, N, K, mode=QOQ_GROUP128):
    """(tile_m, split_k) a GEMM call of this shape would run with (host only)."""
    t, k = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().qoq_query_gemm_config(M, N, K, mode, ctypes.byref(t), ctypes.byref(k)))
    return t.value, k.value


def pack_weights(w, mode=QOQ_GROUP128, out=None):
    """FP16 weights [N, K] on the GPU -> packed blob (uint8 tensor)."""
    _dev(w, torch.float16, "w")
    N, K = w.shape
    size = packed_bytes(N, K, mode)
    if size == 0:
        _check(2)
    blob = out if out is not None else torch.empty(size, dtype=torch.uint8, device=w.device)
    _check(lib().qoq_pack_weights(_ptr(w), N, K, mode, _ptr(blob), _stream(w.device)))
    return blob


def pack_quantized(q, s1, z, s, mode=QOQ_GROUP128):
    """Already-quantized tensors (uint8 codes [N,K], uint8 s1/z, FP16 scales) -> packed blob."""
    _dev(q, torch.uint8, "q")
    N, K = q.shape
    size = packed_bytes(N, K, mode)
    if size == 0:
        _check(2)
    blob = torch.zeros(size, dtype=torch.uint8, device=q.device)
    _check(lib().qoq_pack_quantized(_ptr(q), _ptr(s1), _ptr(z), _ptr(s), N, K, mode, _ptr(blob), _stream(q.device)))
    return blob


def unpack_weights(blob, N, K, mode=QOQ_GROUP128):
    """Packed blob -> (codes uint8 [N,K], s1 uint8 [N,K/128] or None, z uint8, scales FP16 [N])."""
    dev = blob.device
    q = torch.empty((N, K), dtype=torch.uint8, device=dev)
    s = torch.empty(N, dtype=torch.float16, device=dev)
    if mode == QOQ_GROUP128:
        s1 = torch.empty((N, K // GROUP), dtype=torch.uint8, device=dev)
        z = torch.empty((N, K // GROUP), dtype=torch.uint8, device=dev)
    else:
        s1 = None
        z = torch.empty(N, dtype=torch.uint8, device=dev)
    _check(lib().qoq_unpack_weights(_ptr(blob), N, K, mode, _ptr(q), _ptr(s1), _ptr(z), _ptr(s), _stream(dev)))
    return q, s1, z, s


def quant_act_per_token(x, want_rowsum=True, want_tx=False):
    """FP16 activations [M, K] -> (qx int8 [M,K], sx FP16 [M], rowsum int32 [M] | None, tx FP32 [M] | None)."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    qx = torch.empty((M, K), dtype=torch.int8, device=x.device)
    sx = torch.empty(M, dtype=torch.float16, device=x.device)
    rowsum = torch.empty(M, dtype=torch.int32, device=x.device) if want_rowsum else None
    tx = torch.empty(M, dtype=torch.float32, device=x.device) if want_tx else None
    _check(lib().qoq_quant_act_per_token(_ptr(x), M, K, _ptr(qx), _ptr(sx), _ptr(rowsum), _ptr(tx), _stream(x.device)))
    return qx, sx, rowsum, tx


def new_workspace(nbytes, device):
    """Allocate a GEMM workspace and zero-fill it with the library's own kernel."""
    nbytes = (int(nbytes) + 15) // 16 * 16
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)
    _check(lib().qoq_gemm_workspace_prepare(_ptr(ws), ws.numel(), _stream(device)))
    return ws


def _workspace(M, N, K, mode, device, workspace):
    need = gemm_workspace_bytes(M, N, K, mode)
    if workspace is None and need:
        workspace = new_workspace(need, device)
    return workspace, (workspace.numel() * workspace.element_size() if workspace is not None else 0)


def w4a8_gemm(qx, sx, packed, N, mode=QOQ_GROUP128, rowsum=None, out=None, workspace=None):
    """out[M, N] FP16 = W4A8 GEMM of INT8 activations with a packed weight blob."""
    _dev(qx, torch.int8, "qx")
    M, K = qx.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=qx.device)
    workspace, ws_bytes = _workspace(M, N, K, mode, qx.device, workspace)
    _check(lib().qoq_w4a8_gemm(_ptr(qx), _ptr(sx), _ptr(rowsum), _ptr(packed), M, N, K, mode, _ptr(out),
                               _ptr(workspace), ws_bytes, _stream(qx.device)))
    return out


def w4a8_gemm_noalloc(qx, sx, packed, N, out, mode=QOQ_GROUP128, rowsum=None):
    """qoq_w4a8_gemm_noalloc: the same GEMM with the library's own per-GPU scratch array; `out` [M, N] FP16 is the
    caller's (nothing is allocated on the way, here or in the library)."""
    _dev(qx, torch.int8, "qx")
    _dev(out, torch.float16, "out")
    M, K = qx.shape
    _check(lib().qoq_w4a8_gemm_noalloc(_ptr(qx), _ptr(sx), _ptr(rowsum), _ptr(packed), M, N, K, mode, _ptr(out),
                                       _stream(qx.device)))
    return out


def w4a8_gemm_i32(qx, packed, N, mode=QOQ_GROUP128, rowsum=None, out=None, workspace=None):
    """Raw INT32 accumulators [M, N] of the same GEMM (debug entry)."""
    _dev(qx, torch.int8, "qx")
    M, K = qx.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=qx.device)
    workspace, ws_bytes = _workspace(M, N, K, mode, qx.device, workspace)
    _check(lib().qoq_w4a8_gemm_i32(_ptr(qx), _ptr(rowsum), _ptr(packed), M, N, K, mode, _ptr(out),
                                   _ptr(workspace), ws_bytes, _stream(qx.device)))
    return out


def w4a8_linear(x, packed, N, mode=QOQ_GROUP128, out=None, qx=None, sx=None, rowsum=None, workspace=None):
    """Activation quantization + GEMM in one call; returns (out FP16 [M,N], qx, sx, rowsum)."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    dev = x.device
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=dev)
    if qx is None:
        qx = torch.empty((M, K), dtype=torch.int8, device=dev)
    if sx is None:
        sx = torch.empty(M, dtype=torch.float16, device=dev)
    if rowsum is None:
        rowsum = torch.empty(M, dtype=torch.int32, device=dev)
    workspace, ws_bytes = _workspace(M, N, K, mode, dev, workspace)
    _check(lib().qoq_w4a8_linear(_ptr(x), _ptr(packed), M, N, K, mode, _ptr(out), _ptr(qx), _ptr(sx), _ptr(rowsum),
                                 _ptr(workspace), ws_bytes, _stream(dev)))
    return out, qx, sx, rowsum


def w4a8_gemm_token_sum(qx, sx, tx, packed, N, out=None, workspace=None):
    """Per-channel GEMM with the token-sum (subtraction after multiplication) epilogue; tx = FP32 [M]."""
    _dev(qx, torch.int8, "qx")
    _dev(tx, torch.float32, "tx")
    M, K = qx.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=qx.device)
    workspace, ws_bytes = _workspace(M, N, K, QOQ_PER_CHANNEL, qx.device, workspace)
    _check(lib().qoq_w4a8_gemm_token_sum(_ptr(qx), _ptr(sx), _ptr(tx), _ptr(packed), M, N, K, _ptr(out),
                                         _ptr(workspace), ws_bytes, _stream(qx.device)))
    return out


def _quant_outputs(M, K, dev, want_y, want_rowsum, want_tx):
    y = torch.empty((M, K), dtype=torch.float16, device=dev) if want_y else None
    qx = torch.empty((M, K), dtype=torch.int8, device=dev)
    sx = torch.empty(M, dtype=torch.float16, device=dev)
    rowsum = torch.empty(M, dtype=torch.int32, device=dev) if want_rowsum else None
    tx = torch.empty(M, dtype=torch.float32, device=dev) if want_tx else None
    return y, qx, sx, rowsum, tx


def rmsnorm_quant(x, gamma, eps, want_y=True, want_rowsum=True, want_tx=False):
    """RMSNorm with the per-token quantization fused in; returns (y FP16 | None, qx, sx, rowsum | None, tx | None)."""
    _dev(x, torch.float16, "x")
    _dev(gamma, torch.float16, "gamma")
    M, K = x.shape
    y, qx, sx, rowsum, tx = _quant_outputs(M, K, x.device, want_y, want_rowsum, want_tx)
    _check(lib().qoq_rmsnorm_quant(_ptr(x), _ptr(gamma), float(eps), M, K, _ptr(y), _ptr(qx), _ptr(sx), _ptr(rowsum),
                                   _ptr(tx), _stream(x.device)))
    return y, qx, sx, rowsum, tx


def silu_mul_quant(gate_up, want_y=True, want_rowsum=True, want_tx=False):
    """SiLU(gate) * up on a fused [M, 2K] tensor with the per-token quantization fused in."""
    _dev(gate_up, torch.float16, "gate_up")
    M, K2 = gate_up.shape
    K = K2 // 2
    y, qx, sx, rowsum, tx = _quant_outputs(M, K, gate_up.device, want_y, want_rowsum, want_tx)
    _check(lib().qoq_silu_mul_quant(_ptr(gate_up), M, K, _ptr(y), _ptr(qx), _ptr(sx), _ptr(rowsum), _ptr(tx),
                                    _stream(gate_up.device)))
    return y, qx, sx, rowsum, tx


# ---------------------------------------------------------------------------------------
# KV4 cache and decode attention
# ---------------------------------------------------------------------------------------
def kv4_cache_bytes(B, Hkv, S_max, D=128):
    return int(lib().qoq_kv4_cache_bytes(B, Hkv, S_max, D))


def kv4_new_cache(B, Hkv, S_max, device, D=128):
    """An empty (zero-filled) cache buffer for B sequences of up to S_max tokens."""
    n = kv4_cache_bytes(B, Hkv, S_max, D)
    if n == 0 and B > 0:
        raise QoqError(2, "unsupported KV4 cache shape")
    return torch.zeros(max(n, 16), dtype=torch.uint8, device=device)


def kv4_append(cache, k, v, positions, S_max):
    """Quantize k, v [B, T, Hkv, D] FP16 and write them at token positions positions[b] .. + T - 1."""
    _dev(k, torch.float16, "k")
    _dev(v, torch.float16, "v")
    _dev(positions, torch.int32, "positions")
    B, T, Hkv, D = k.shape
    _check(lib().qoq_kv4_append(_ptr(k), _ptr(v), _ptr(positions), B, T, Hkv, D, S_max, _ptr(cache), _stream(k.device)))


def kv4_attention_workspace_bytes(B, H, Hkv, S_max, D=128):
    return int(lib().qoq_kv4_attention_workspace_bytes(B, H, Hkv, D, S_max))


def kv4_attention_decode(q, cache, seq_lens, Hkv, S_max, out=None, workspace=None):
    """out[b, h] = softmax(q[b, h] . K^ / sqrt(D)) V^ over the first seq_lens[b] tokens of the cache.
    With a `workspace` (uint8 tensor of kv4_attention_workspace_bytes) the library may split long sequences
    over several workgroups."""
    _dev(q, torch.float16, "q")
    _dev(seq_lens, torch.int32, "seq_lens")
    B, H, D = q.shape
    if out is None:
        out = torch.empty((B, H, D), dtype=torch.float16, device=q.device)
    if workspace is None:
        _check(lib().qoq_kv4_attention_decode(_ptr(q), _ptr(cache), _ptr(seq_lens), B, H, Hkv, D, S_max, _ptr(out),
                                              _stream(q.device)))
    else:
        _check(lib().qoq_kv4_attention_decode_split(_ptr(q), _ptr(cache), _ptr(seq_lens), B, H, Hkv, D, S_max, _ptr(out),
                                                    _ptr(workspace), workspace.numel(), _stream(q.device)))
    return out


def kv4_unpack(cache, B, Hkv, S_max, D=128):
    """(k_codes, k_s, k_z, v_codes, v_s, v_z): one byte per code, FP16 scales and zeros (tests)."""
    dev = cache.device
    kc = torch.empty((B, Hkv, S_max, D), dtype=torch.uint8, device=dev)
    vc = torch.empty_like(kc)
    ks = torch.empty((B, Hkv, S_max), dtype=torch.float16, device=dev)
    kz, vs, vz = torch.empty_like(ks), torch.empty_like(ks), torch.empty_like(ks)
    _check(lib().qoq_kv4_unpack(_ptr(cache), B, Hkv, S_max, D, _ptr(kc), _ptr(ks), _ptr(kz), _ptr(vc), _ptr(vs), _ptr(vz),
                                _stream(dev)))
    return kc, ks, kz, vc, vs, vz


# ---------------------------------------------------------------------------------------
# Data-free offline transforms: channel reordering, Hadamard rotation
# ---------------------------------------------------------------------------------------
def channel_absmax(x):
    """max over tokens of |x| per input channel: FP16 [M, K] -> FP32 [K]."""
    _dev(x, torch.float16, "x")
    M, K = x.shape
    out = torch.empty(K, dtype=torch.float32, device=x.device)
    _check(lib().qoq_channel_absmax(_ptr(x), M, K, _ptr(out), _stream(x.device)))
    return out


def channel_order(salience):
    """Permutation (INT32, on the device of `salience`): most salient channel first; sorted on the host."""
    host = salience.detach().to("cpu", torch.float32).contiguous()
    perm = torch.empty(host.numel(), dtype=torch.int32)
    _check(lib().qoq_channel_order_host(host.data_ptr(), host.numel(), perm.data_ptr()))
    return perm.to(salience.device)


def gather_channels(src, perm):
    _dev(src, torch.float16, "src")
    _dev(perm, torch.int32, "perm")
    rows, K = src.shape
    dst = torch.empty_like(src)
    _check(lib().qoq_gather_channels(_ptr(src), _ptr(perm), rows, K, _ptr(dst), _stream(src.device)))
    return dst


def quant_act_per_token_reordered(x, perm, want_rowsum=True, want_tx=False):
    """quant_act_per_token of x[:, perm] in one pass."""
    _dev(x, torch.float16, "x")
    _dev(perm, torch.int32, "perm")
    M, K = x.shape
    _, qx, sx, rowsum, tx = _quant_outputs(M, K, x.device, False, want_rowsum, want_tx)
    _check(lib().qoq_quant_act_per_token_reordered(_ptr(x), _ptr(perm), M, K, _ptr(qx), _ptr(sx), _ptr(rowsum), _ptr(tx),
                                                   _stream(x.device)))
    return qx, sx, rowsum, tx


def hadamard_rotate(src, block=None, out=None):
    """src (I (x) H_block) / sqrt(block), rounded once to FP16; block defaults to the largest power of two dividing K."""
    _dev(src, torch.float16, "src")
    rows, K = src.shape
    if block is None:
        block = min(K & -K, 8192)
    if out is None:
        out = torch.empty_like(src)
    _check(lib().qoq_hadamard_rotate(_ptr(src), rows, K, block, _ptr(out), _stream(src.device)))
    return out
