"""Thin ctypes binding of libtsa.so: same names as the C ABI (include/tsa.h), argument
marshalling only.  Tensors are torch CUDA tensors used purely as device memory; every step
runs in the library's HIP kernels.  There is no fallback: if the library is missing or a
call fails, an exception is raised."""
from __future__ import annotations

import ctypes
import math
import os

import torch

from . import build as _build

TSA_OK, TSA_ERR_ARG, TSA_ERR_UNSUPPORTED, TSA_ERR_WORKSPACE, TSA_ERR_HIP = 0, 1, 2, 3, 4

EXPORTS = ("tsa_version", "tsa_last_error", "tsa_keep_count", "tsa_workspace_bytes", "tsa_score", "tsa_coverage_budget",
           "tsa_score_queries_workspace_bytes", "tsa_score_queries", "tsa_gather_queries", "tsa_pool_queries_workspace_bytes", "tsa_pool_queries",
           "tsa_select", "tsa_compress", "tsa_attend_workspace_bytes", "tsa_attend", "tsa_decompress", "tsa_compress_v_tiles", "tsa_attend_fused", "tsa_forward",
           "tsa_forward_dynamic_workspace_bytes", "tsa_forward_dynamic",
           "tsa_layer_drift_workspace_bytes", "tsa_layer_drift", "tsa_sparse_layers", "tsa_mfma_probe", "tsa_mix_probe", "tsa_read_probe", "tsa_copy_probe", "tsa_bench_set_attend_form",
           "tsa_select_static", "tsa_select_static_capacity")


class TsaError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libtsa error %d: %s" % (code, msg))
        self.code = code


class tsa_desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("L", ctypes.c_int32),
                ("d", ctypes.c_int32), ("last_q", ctypes.c_int32), ("pool_w", ctypes.c_int32),
                ("group_mode", ctypes.c_int32), ("force_first", ctypes.c_int32), ("force_last", ctypes.c_int32),
                ("scale", ctypes.c_float), ("block_list_per_head", ctypes.c_int32), ("q_stride_b", ctypes.c_int64), ("q_stride_h", ctypes.c_int64), ("q_stride_l", ctypes.c_int64),
                ("kv_stride_b", ctypes.c_int64), ("kv_stride_h", ctypes.c_int64), ("kv_stride_l", ctypes.c_int64),
                ("o_stride_b", ctypes.c_int64), ("o_stride_h", ctypes.c_int64), ("o_stride_l", ctypes.c_int64)]


def make_desc(B, Hq, Hkv, L, d, last_q=64, pool_w=1, group_mode=0, force_first=0, force_last=0, scale=0.0,
              block_list_per_head=0, q_strides=(0, 0, 0), kv_strides=(0, 0, 0), o_strides=(0, 0, 0)):
    """*_strides = (stride_b, stride_h, stride_l) in elements of Q, of K and V, of O; zeros = contiguous [B,H,L,d]."""
    return tsa_desc(B, Hq, Hkv, L, d, last_q, pool_w, group_mode, force_first, force_last, scale, block_list_per_head,
                    *q_strides, *kv_strides, *o_strides)


def blhd_strides(H, L, d):
    """Strides of a [B,L,H,d] tensor addressed as (b, h, t)."""
    return (L * H * d, d, H * d)


_lib = None


def load_library(build_if_missing: bool = True) -> ctypes.CDLL:
    """Loads the in-tree libtsa.so; builds it first only if it does not exist."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB_PATH
    if not os.path.exists(path):
        if not build_if_missing:
            raise ImportError("libtsa.so is not built (%s)" % path)
        _build.build_library()
    lib = ctypes.CDLL(path)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    dp = ctypes.POINTER(tsa_desc)
    lib.tsa_version.restype = ctypes.c_int
    lib.tsa_version.argtypes = []
    lib.tsa_last_error.restype = ctypes.c_char_p
    lib.tsa_last_error.argtypes = []
    lib.tsa_keep_count.restype = i32
    lib.tsa_keep_count.argtypes = [i32, ctypes.c_double]
    lib.tsa_workspace_bytes.restype = sz
    lib.tsa_workspace_bytes.argtypes = [dp, i32]
    lib.tsa_score.restype = ctypes.c_int
    lib.tsa_score.argtypes = [dp, vp, vp, vp, vp, sz, vp]
    ip = ctypes.POINTER(i32)
    lib.tsa_score_queries.restype = ctypes.c_int
    lib.tsa_score_queries.argtypes = [dp, vp, ip, i32, vp, vp, vp, sz, vp]
    lib.tsa_score_queries_workspace_bytes.restype = sz
    lib.tsa_score_queries_workspace_bytes.argtypes = [dp, i32]
    lib.tsa_bench_set_attend_form.restype = ctypes.c_int
    lib.tsa_bench_set_attend_form.argtypes = [i32]
    lib.tsa_copy_probe.restype = ctypes.c_int
    lib.tsa_copy_probe.argtypes = [vp, vp, sz, vp]
    lib.tsa_read_probe.restype = ctypes.c_int
    lib.tsa_read_probe.argtypes = [vp, sz, vp, vp]
    lib.tsa_mix_probe.restype = ctypes.c_int
    lib.tsa_mix_probe.argtypes = [i32, vp, i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.tsa_gather_queries.restype = ctypes.c_int
    lib.tsa_gather_queries.argtypes = [dp, vp, ip, i32, vp, vp]
    lib.tsa_pool_queries_workspace_bytes.restype = sz
    lib.tsa_pool_queries_workspace_bytes.argtypes = [dp, i32]
    lib.tsa_pool_queries.restype = ctypes.c_int
    lib.tsa_pool_queries.argtypes = [dp, vp, i32, vp, ip, vp, sz, vp]
    lib.tsa_coverage_budget.restype = ctypes.c_int
    lib.tsa_coverage_budget.argtypes = [dp, vp, ctypes.c_double, vp, vp, sz, vp]
    lib.tsa_select.restype = ctypes.c_int
    lib.tsa_select.argtypes = [dp, vp, i32, vp, vp, vp, sz, vp]
    lib.tsa_select_static.restype = ctypes.c_int
    lib.tsa_select_static.argtypes = [dp, vp, i32, vp, vp, vp]
    lib.tsa_select_static_capacity.restype = sz
    lib.tsa_select_static_capacity.argtypes = []
    lib.tsa_compress.restype = ctypes.c_int
    lib.tsa_compress.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp, vp, vp]
    lib.tsa_attend.restype = ctypes.c_int
    lib.tsa_attend.argtypes = [dp, vp, vp, vp, i32, i32, vp, i32, i32, vp, vp, vp, sz, vp]
    lib.tsa_compress_v_tiles.restype = ctypes.c_int
    lib.tsa_compress_v_tiles.argtypes = [dp, vp, vp, i32, vp, sz, vp]
    lib.tsa_attend_fused.restype = ctypes.c_int
    lib.tsa_attend_fused.argtypes = [dp, vp, vp, vp, vp, vp, i32, vp, i32, i32, vp, vp, vp, vp]
    lib.tsa_mfma_probe.restype = ctypes.c_int
    lib.tsa_mfma_probe.argtypes = [vp, i32, i32, vp, vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32), vp]
    lib.tsa_attend_workspace_bytes.restype = sz
    lib.tsa_attend_workspace_bytes.argtypes = [dp, i32, i32]
    lib.tsa_decompress.restype = ctypes.c_int
    lib.tsa_decompress.argtypes = [dp, vp, vp, vp, i32, vp, vp, vp]
    lib.tsa_forward_dynamic_workspace_bytes.restype = sz
    lib.tsa_forward_dynamic_workspace_bytes.argtypes = [dp, i32]
    lib.tsa_forward_dynamic.restype = ctypes.c_int
    lib.tsa_forward_dynamic.argtypes = [dp, vp, vp, vp, ctypes.c_double, i32, vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.tsa_forward.restype = ctypes.c_int
    lib.tsa_forward.argtypes = [dp, vp, vp, vp, i32, vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.tsa_layer_drift_workspace_bytes.restype = sz
    lib.tsa_layer_drift_workspace_bytes.argtypes = [ctypes.c_int64]
    lib.tsa_layer_drift.restype = ctypes.c_int
    lib.tsa_layer_drift.argtypes = [vp, vp, ctypes.c_int64, i32, ctypes.c_float, vp, vp, sz, vp]
    lib.tsa_sparse_layers.restype = ctypes.c_int
    lib.tsa_sparse_layers.argtypes = [ctypes.POINTER(ctypes.c_float), i32, ctypes.c_double, ctypes.POINTER(i32)]
    _lib = lib
    return lib


def _check(rc):
    if rc != TSA_OK:
        raise TsaError(rc, load_library().tsa_last_error().decode())


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise TsaError(TSA_ERR_ARG, "tensor is not on the GPU")
    if not t.is_contiguous():
        raise TsaError(TSA_ERR_ARG, "tensor is not contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(ws):
    if ws is None:
        return None, 0
    return _ptr(ws), ws.numel() * ws.element_size()


def tsa_version() -> int:
    return load_library().tsa_version()


def tsa_last_error() -> str:
    return load_library().tsa_last_error().decode()


def tsa_keep_count(L: int, tau: float) -> int:
    return load_library().tsa_keep_count(L, tau)


def tsa_workspace_bytes(desc: tsa_desc, k_keep: int) -> int:
    return load_library().tsa_workspace_bytes(ctypes.byref(desc), k_keep)


def tsa_score(desc, Q, K, scores, ws):
    p, n = _ws(ws)
    _check(load_library().tsa_score(ctypes.byref(desc), _ptr(Q), _ptr(K), _ptr(scores), p, n, _stream()))


def _host_ints(values):
    return (ctypes.c_int32 * len(values))(*[int(v) for v in values])


def tsa_score_queries_workspace_bytes(desc, n) -> int:
    return int(load_library().tsa_score_queries_workspace_bytes(ctypes.byref(desc), n))


def tsa_score_queries(desc, Qsel, qpos, K, scores, ws=None):
    """qpos: sequence of host ints (ascending positions of the rows of Qsel)."""
    if ws is None:
        ws = torch.empty(max(256, tsa_score_queries_workspace_bytes(desc, len(qpos))), dtype=torch.uint8, device=K.device)
    p, n = _ws(ws)
    _check(load_library().tsa_score_queries(ctypes.byref(desc), _ptr(Qsel), _host_ints(qpos), len(qpos), _ptr(K),
                                            _ptr(scores), p, n, _stream()))


def tsa_gather_queries(desc, Q, qpos, Qsel):
    _check(load_library().tsa_gather_queries(ctypes.byref(desc), _ptr(Q), _host_ints(qpos), len(qpos), _ptr(Qsel), _stream()))


def tsa_pool_queries(desc, Q, n_pool, Qsel, ws=None):
    """Returns the positions (host list) of the pooled queries."""
    if ws is None:
        ws = torch.empty(max(256, load_library().tsa_pool_queries_workspace_bytes(ctypes.byref(desc), n_pool)),
                         dtype=torch.uint8, device=Q.device)
    p, n = _ws(ws)
    qpos = (ctypes.c_int32 * n_pool)()
    _check(load_library().tsa_pool_queries(ctypes.byref(desc), _ptr(Q), n_pool, _ptr(Qsel), qpos, p, n, _stream()))
    return list(qpos)


def tsa_coverage_budget(desc, scores, tau_cov, k_keep, ws):
    p, n = _ws(ws)
    _check(load_library().tsa_coverage_budget(ctypes.byref(desc), _ptr(scores), float(tau_cov), _ptr(k_keep), p, n, _stream()))


def tsa_select(desc, scores, k_keep, idx, inv, ws=None):
    p, n = _ws(ws)
    _check(load_library().tsa_select(ctypes.byref(desc), _ptr(scores), k_keep, _ptr(idx), _ptr(inv), p, n, _stream()))


def tsa_select_static(desc, scores, k_keep, idx, inv):
    _check(load_library().tsa_select_static(ctypes.byref(desc), _ptr(scores), k_keep, _ptr(idx), _ptr(inv), _stream()))


def tsa_compress(desc, Q, K, V, idx, k_keep, Qc, Kc, Vc):
    _check(load_library().tsa_compress(ctypes.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(idx), k_keep,
                                       _ptr(Qc), _ptr(Kc), _ptr(Vc), _stream()))


def tsa_attend_workspace_bytes(desc, Lc, kv_heads):
    return int(load_library().tsa_attend_workspace_bytes(ctypes.byref(desc), Lc, kv_heads))


def tsa_attend(desc, Qc, Kc, Vc, Lc, kv_heads, Oc, ws, lse=None, block_list=None, block_size=0, max_blocks_per_row=0):
    p, n = _ws(ws)
    _check(load_library().tsa_attend(ctypes.byref(desc), _ptr(Qc), _ptr(Kc), _ptr(Vc), Lc, kv_heads,
                                     _ptr(block_list), block_size, max_blocks_per_row, _ptr(Oc), _ptr(lse),
                                     p, n, _stream()))


def tsa_decompress(desc, Oc, idx, inv, k_keep, O=None, residual=None):
    _check(load_library().tsa_decompress(ctypes.byref(desc), _ptr(Oc), _ptr(idx), _ptr(inv), k_keep,
                                         _ptr(O), _ptr(residual), _stream()))


def tsa_compress_v_tiles(desc, V, idx, k_keep, Vt):
    p, n = _ws(Vt)
    _check(load_library().tsa_compress_v_tiles(ctypes.byref(desc), _ptr(V), _ptr(idx), k_keep, p, n, _stream()))


def tsa_attend_fused(desc, Q, K, Vt, idx, inv, k_keep, O=None, Oc=None, residual=None,
                     block_list=None, block_size=0, max_blocks_per_row=0):
    _check(load_library().tsa_attend_fused(ctypes.byref(desc), _ptr(Q), _ptr(K), _ptr(Vt), _ptr(idx), _ptr(inv), k_keep,
                                           _ptr(block_list), block_size, max_blocks_per_row, _ptr(O), _ptr(Oc),
                                           _ptr(residual), _stream()))


def alloc_forward_dynamic_workspace(desc, k_max, device="cuda"):
    """Device buffer of tsa_forward_dynamic_workspace_bytes() bytes."""
    n = load_library().tsa_forward_dynamic_workspace_bytes(ctypes.byref(desc), k_max)
    if n == 0:
        raise TsaError(TSA_ERR_ARG, tsa_last_error())
    return torch.empty(n, dtype=torch.uint8, device=device)


def tsa_forward_dynamic(desc, Q, K, V, tau_cov, k_max, O, ws, residual=None, k_keep_out=None, idx_out=None,
                        block_list=None, block_size=0, max_blocks_per_row=0):
    p, n = _ws(ws)
    _check(load_library().tsa_forward_dynamic(ctypes.byref(desc), _ptr(Q), _ptr(K), _ptr(V), float(tau_cov), k_max,
                                              _ptr(block_list), block_size, max_blocks_per_row,
                                              _ptr(O), _ptr(residual), _ptr(k_keep_out), _ptr(idx_out), p, n, _stream()))


def tsa_forward(desc, Q, K, V, k_keep, O, ws, residual=None, idx_out=None,
                block_list=None, block_size=0, max_blocks_per_row=0):
    p, n = _ws(ws)
    _check(load_library().tsa_forward(ctypes.byref(desc), _ptr(Q), _ptr(K), _ptr(V), k_keep,
                                      _ptr(block_list), block_size, max_blocks_per_row,
                                      _ptr(O), _ptr(residual), _ptr(idx_out), p, n, _stream()))


def tsa_layer_drift(h_in, h_out, eps, drift_out, ws=None):
    """h_in, h_out [n_tokens, width] bf16 CUDA tensors; drift_out: 1-element fp32 CUDA tensor."""
    n_tokens, width = h_in.shape
    if ws is None:
        ws = torch.empty(load_library().tsa_layer_drift_workspace_bytes(n_tokens), dtype=torch.uint8, device=h_in.device)
    p, n = _ws(ws)
    _check(load_library().tsa_layer_drift(_ptr(h_in), _ptr(h_out), n_tokens, width, eps, _ptr(drift_out), p, n, _stream()))


def tsa_sparse_layers(drift, delta=0.5):
    """Eq. 2 on the host: list of 0/1 flags, 1 = layer is eligible for Token Sparse Attention."""
    n = len(drift)
    arr = (ctypes.c_float * n)(*[float(v) for v in drift])
    out = (ctypes.c_int32 * n)()
    _check(load_library().tsa_sparse_layers(arr, n, float(delta), out))
    return list(out)


def tsa_mfma_probe(operands, iters, blocks, sink, clocks):
    """Queues the bare MFMA loop; returns (flops of the launch, wall clock rate in kHz)."""
    flops, khz = ctypes.c_double(0.0), ctypes.c_int32(0)
    _check(load_library().tsa_mfma_probe(_ptr(operands), iters, blocks, _ptr(sink), _ptr(clocks),
                                         ctypes.byref(flops), ctypes.byref(khz), _stream()))
    return flops.value, khz.value


def tsa_mix_probe(mix, operands, iters, blocks, sink):
    """Queues the instruction-mix loop `mix` (0..3); returns the flops of the launch's MFMAs."""
    flops = ctypes.c_double(0.0)
    _check(load_library().tsa_mix_probe(mix, _ptr(operands), iters, blocks, _ptr(sink), ctypes.byref(flops), _stream()))
    return flops.value


def tsa_read_probe(src, sink):
    """Queues the streaming read of src (byte size a multiple of 16); sink: a device tensor of at least 4 bytes."""
    _check(load_library().tsa_read_probe(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream()))


def tsa_bench_set_attend_form(form: int):
    _check(load_library().tsa_bench_set_attend_form(form))


def tsa_copy_probe(src, dst):
    """Queues the streaming copy dst = src (same byte size, a multiple of 16)."""
    nbytes = src.numel() * src.element_size()
    if nbytes != dst.numel() * dst.element_size():
        raise TsaError(TSA_ERR_ARG, "src and dst differ in size")
    _check(load_library().tsa_copy_probe(_ptr(src), _ptr(dst), nbytes, _stream()))


def alloc_attend_workspace(desc, Lc, kv_heads, device="cuda"):
    n = tsa_attend_workspace_bytes(desc, Lc, kv_heads)
    if n == 0:
        raise TsaError(TSA_ERR_ARG, tsa_last_error())
    return torch.empty(n, dtype=torch.uint8, device=device)


def alloc_workspace(desc, k_keep, device="cuda"):
    """Device buffer of tsa_workspace_bytes() bytes (torch allocations are 256-byte aligned)."""
    n = tsa_workspace_bytes(desc, k_keep)
    if n == 0:
        raise TsaError(TSA_ERR_ARG, tsa_last_error())
    return torch.empty(n, dtype=torch.uint8, device=device)
