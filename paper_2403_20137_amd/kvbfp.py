"""Thin ctypes binding of libkvbfp.so: same names as the C ABI (include/kvbfp.h), argument
marshalling only.  Every step of the path runs inside the library's HIP kernels; PyTorch is used
for device memory and streams.  There is no fallback: if the library is missing, importing the
functions raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libkvbfp.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, -1, -2, -3, -4
F32, F16, BF16 = 0, 1, 2
STAT_MAXABS, STAT_L2 = 0, 1
ROPE_PAIRS_ADJACENT, ROPE_PAIRS_HALF_SPLIT = 0, 1

_TORCH_DT = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}
_NP_DT = {np.dtype(np.float32): F32, np.dtype(np.float16): F16}

EXPORTS = ["kvbfp_cache_bytes", "kvbfp_calibrate_perm", "kvbfp_permute_weights", "kvbfp_permute_weight_columns",
           "kvbfp_quantize_append", "kvbfp_dequantize", "kvbfp_decode_workspace_bytes",
           "kvbfp_decode_attention", "kvbfp_decode_attention_qbfp", "kvbfp_append_decode_attention", "kvbfp_decode_attention_multi", "kvbfp_decode_attention_profile",
           "kvbfp_permute_rope", "kvbfp_decode_attention_rope",
           "kvbfp_quantize_append_paged", "kvbfp_dequantize_paged", "kvbfp_decode_workspace_bytes_paged",
           "kvbfp_decode_attention_paged", "kvbfp_append_decode_attention_paged", "kvbfp_decode_attention_multi_paged",
           "kvbfp_decode_attention_noalloc", "kvbfp_measure_stream_read", "kvbfp_decode_attention_profile_ring",
           "kvbfp_last_error", "kvbfp_version"]


class KvbfpError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("kvbfp status %d: %s" % (status, message))
        self.status = status


class Layout(C.Structure):
    _fields_ = [("struct_bytes", C.c_uint32), ("head_dim", C.c_int32), ("block", C.c_int32),
                ("mant_bits", C.c_int32), ("n_kv_heads", C.c_int32), ("batch", C.c_int32),
                ("max_seq", C.c_int64)]


class CachePtrs(C.Structure):
    _fields_ = [("k_mant", C.c_void_p), ("k_exp", C.c_void_p), ("v_mant", C.c_void_p),
                ("v_exp", C.c_void_p)]


_lib = None


def lib():
    """Loads libkvbfp.so; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libkvbfp.so not found at %s -- build it with "
                               "`python -m paper_2403_20137_amd.build` (needs hipcc)" % LIB_PATH)
        l = C.CDLL(LIB_PATH)
        l.kvbfp_last_error.restype = C.c_char_p
        l.kvbfp_version.restype = C.c_char_p
        l.kvbfp_decode_workspace_bytes.restype = C.c_size_t
        l.kvbfp_decode_workspace_bytes.argtypes = [C.POINTER(Layout), C.c_int32, C.c_int64]
        l.kvbfp_cache_bytes.argtypes = [C.POINTER(Layout), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        l.kvbfp_calibrate_perm.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int32, C.c_int32,
                                           C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_int32, C.c_void_p]
        l.kvbfp_permute_weights.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int32,
                                            C.c_int64, C.c_int32, C.c_void_p]
        l.kvbfp_permute_weight_columns.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int32, C.c_int32,
                                                   C.c_int32, C.c_void_p]
        l.kvbfp_permute_rope.argtypes = [C.c_void_p, C.c_int, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p]
        l.kvbfp_decode_attention_rope.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_int32, C.c_void_p,
                                                  C.c_int, C.c_void_p, C.c_int64, C.c_float, C.c_void_p,
                                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                  C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        l.kvbfp_quantize_append_paged.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_void_p, C.c_int64,
                                                  C.c_int32, C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int64,
                                                  C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                                  C.c_void_p, C.c_void_p]
        l.kvbfp_dequantize_paged.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_void_p, C.c_int64, C.c_int32,
                                             C.c_int32, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_int,
                                             C.c_void_p]
        l.kvbfp_decode_workspace_bytes_paged.restype = C.c_size_t
        l.kvbfp_decode_workspace_bytes_paged.argtypes = [C.POINTER(Layout), C.c_int64, C.c_int32, C.c_int32, C.c_int64]
        l.kvbfp_decode_attention_paged.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_void_p, C.c_int64,
                                                   C.c_int32, C.c_int32, C.c_void_p, C.c_int, C.c_void_p, C.c_int64,
                                                   C.c_float, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                                   C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        _paged = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_void_p, C.c_int64, C.c_int32]
        l.kvbfp_append_decode_attention_paged.argtypes = _paged + [
            C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int, C.c_void_p, C.c_int64,
            C.c_float, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        l.kvbfp_decode_attention_multi_paged.argtypes = _paged + [
            C.c_int32, C.c_int32, C.c_void_p, C.c_int, C.c_void_p, C.c_int64, C.c_float, C.c_void_p, C.c_void_p,
            C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        l.kvbfp_quantize_append.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_void_p, C.c_void_p,
                                            C.c_int, C.c_int32, C.c_int64, C.c_int64, C.c_int64, C.c_int64,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        l.kvbfp_dequantize.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_int32, C.c_int64,
                                       C.c_int64, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        l.kvbfp_decode_attention.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_int32, C.c_void_p,
                                             C.c_int, C.c_void_p, C.c_int64, C.c_float, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        l.kvbfp_decode_attention_qbfp.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_int32, C.c_void_p,
                                                  C.c_int, C.c_void_p, C.c_int64, C.c_float, C.c_void_p,
                                                  C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t,
                                                  C.c_void_p]
        l.kvbfp_append_decode_attention.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_int32, C.c_void_p,
                                                    C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int,
                                                    C.c_void_p, C.c_int64, C.c_float, C.c_void_p, C.c_void_p,
                                                    C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        l.kvbfp_decode_attention_multi.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_int32, C.c_int32,
                                                   C.c_void_p, C.c_int, C.c_void_p, C.c_int64, C.c_float,
                                                   C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                                   C.c_size_t, C.c_void_p]
        l.kvbfp_decode_attention_profile.argtypes = l.kvbfp_decode_attention_qbfp.argtypes + [C.POINTER(C.c_float)]
        l.kvbfp_decode_attention_profile_ring.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_int32, C.c_int32,
                                                          C.c_int32, C.c_void_p, C.c_int, C.c_void_p, C.c_int64,
                                                          C.c_float, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                                          C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_float)]
        l.kvbfp_measure_stream_read.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_int64, C.c_int32,
                                                C.c_void_p, C.c_void_p, C.POINTER(C.c_float)]
        l.kvbfp_decode_attention_noalloc.argtypes = [C.POINTER(Layout), C.POINTER(CachePtrs), C.c_int32, C.c_void_p,
                                                     C.c_int, C.c_void_p, C.c_int64, C.c_float, C.c_void_p,
                                                     C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        _lib = l
    return _lib


def _check(status):
    if status != OK:
        raise KvbfpError(status, lib().kvbfp_last_error().decode())


def last_error() -> str:
    return lib().kvbfp_last_error().decode()


def version() -> str:
    return lib().kvbfp_version().decode()


def make_layout(head_dim, block, mant_bits, n_kv_heads, batch, max_seq) -> Layout:
    return Layout(C.sizeof(Layout), head_dim, block, mant_bits, n_kv_heads, batch, max_seq)


def cache_bytes(layout: Layout):
    m, e = C.c_size_t(0), C.c_size_t(0)
    _check(lib().kvbfp_cache_bytes(C.byref(layout), C.byref(m), C.byref(e)))
    return m.value, e.value


class Cache:
    """The four packed planes of one layer as uint8 device tensors (caller-owned memory)."""

    def __init__(self, layout: Layout, k_mant, k_exp, v_mant, v_exp):
        self.layout = layout
        self.k_mant, self.k_exp, self.v_mant, self.v_exp = k_mant, k_exp, v_mant, v_exp

    @property
    def ptrs(self) -> CachePtrs:
        return CachePtrs(*[t.data_ptr() if t is not None else None
                           for t in (self.k_mant, self.k_exp, self.v_mant, self.v_exp)])

    def planes(self):
        return self.k_mant, self.k_exp, self.v_mant, self.v_exp

    def nbytes(self):
        return sum(t.numel() for t in self.planes())


def alloc_cache(layout: Layout, device="cuda", fill=None) -> Cache:
    mb, eb = cache_bytes(layout)
    ms = (layout.batch, layout.n_kv_heads, layout.max_seq, layout.head_dim * layout.mant_bits // 8)
    es = (layout.batch, layout.n_kv_heads, layout.max_seq, layout.head_dim // layout.block)
    planes = []
    for shape in (ms, es, ms, es):
        t = torch.empty(shape, dtype=torch.uint8, device=device)
        if fill is not None:
            t.fill_(fill)
        planes.append(t)
    assert planes[0].numel() == mb and planes[1].numel() == eb
    return Cache(layout, *planes)


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev_ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("expected a device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected dtype %s, got %s" % (dtype, t.dtype))
    return C.c_void_p(t.data_ptr())


def _host_array(x):
    """numpy view + dtype code of a host tensor/array (bf16 is passed as its 16-bit pattern)."""
    if isinstance(x, torch.Tensor):
        if x.is_cuda:
            raise ValueError("host function needs host memory")
        if x.dtype == torch.bfloat16:
            return x.contiguous().view(torch.int16).numpy(), BF16
        x = x.contiguous().numpy()
    x = np.ascontiguousarray(x)
    if x.dtype not in _NP_DT:
        raise ValueError("unsupported dtype %s" % x.dtype)
    return x, _NP_DT[x.dtype]


def calibrate_perm(x, stat=STAT_MAXABS, descending=False) -> np.ndarray:
    """HOST.  x: [n_samples][n_heads][head_dim] (calibration rows) -> int32 [n_heads][head_dim]."""
    arr, dt = _host_array(x)
    S, H, D = arr.shape
    perm = np.empty((H, D), dtype=np.int32)
    _check(lib().kvbfp_calibrate_perm(arr.ctypes.data, dt, S, H, D, H * D, D, 1, int(stat),
                                      1 if descending else 0, perm.ctypes.data))
    return perm


def calibrate_perm_from_weights(w, n_heads, head_dim, descending=False) -> np.ndarray:
    """HOST.  Alg. 1 proper: w = W_k as [n_heads*head_dim][row_len]; ranks rows by Euclidean norm."""
    arr, dt = _host_array(w)
    rows, row_len = arr.shape
    if rows != n_heads * head_dim:
        raise ValueError("w must have n_heads*head_dim rows")
    perm = np.empty((n_heads, head_dim), dtype=np.int32)
    _check(lib().kvbfp_calibrate_perm(arr.ctypes.data, dt, row_len, n_heads, head_dim, 1,
                                      head_dim * row_len, row_len, STAT_L2, 1 if descending else 0,
                                      perm.ctypes.data))
    return perm


def permute_weights(w, n_heads, head_dim, perm, heads_per_perm=1):
    """HOST, out of place.  Returns the reordered copy in the input's type (torch or numpy)."""
    arr, dt = _host_array(w)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    out = np.empty_like(arr)
    _check(lib().kvbfp_permute_weights(arr.ctypes.data, out.ctypes.data, dt, n_heads, head_dim,
                                       arr.shape[1], heads_per_perm, perm.ctypes.data))
    if isinstance(w, torch.Tensor):
        t = torch.from_numpy(out)
        return t.view(torch.bfloat16) if w.dtype == torch.bfloat16 else t
    return out


def permute_weight_columns(w, n_heads, head_dim, perm, heads_per_perm=1):
    """HOST, out of place.  w: [n_rows][n_heads*head_dim]; returns the copy with reordered columns."""
    arr, dt = _host_array(w)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    if arr.ndim != 2 or arr.shape[1] != n_heads * head_dim:
        raise ValueError("w must be [n_rows][n_heads*head_dim]")
    out = np.empty_like(arr)
    _check(lib().kvbfp_permute_weight_columns(arr.ctypes.data, out.ctypes.data, dt, arr.shape[0], n_heads, head_dim,
                                              heads_per_perm, perm.ctypes.data))
    if isinstance(w, torch.Tensor):
        t = torch.from_numpy(out)
        return t.view(torch.bfloat16) if w.dtype == torch.bfloat16 else t
    return out


def permute_rope(theta, perm, pairs=ROPE_PAIRS_ADJACENT):
    """HOST.  theta: float32 [head_dim/2]; perm: int32 [n_heads][head_dim].
    Returns (theta', partner', sign') as numpy arrays [n_heads][head_dim] (float32, int32, float32)."""
    theta = np.ascontiguousarray(theta, dtype=np.float32)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    if perm.ndim != 2 or theta.shape != (perm.shape[1] // 2,):
        raise ValueError("theta must be [head_dim/2] and perm [n_heads][head_dim]")
    th = np.empty(perm.shape, dtype=np.float32)
    pa = np.empty(perm.shape, dtype=np.int32)
    sg = np.empty(perm.shape, dtype=np.float32)
    _check(lib().kvbfp_permute_rope(theta.ctypes.data, int(pairs), perm.shape[0], perm.shape[1], perm.ctypes.data,
                                    th.ctypes.data, pa.ctypes.data, sg.ctypes.data))
    return th, pa, sg


def quantize_append(cache: Cache, k_new, v_new, pos0=0, pos_dev=None, perm_k=None, perm_v=None,
                    stream=None):
    """DEVICE, async.  k_new / v_new: [batch][n_new][n_kv_heads][head_dim] device tensors (strided in
    the first three dims, channel stride 1) or None."""
    ref = k_new if k_new is not None else v_new
    if ref is None:
        return
    for t in (k_new, v_new):
        if t is not None:
            if t.dim() != 4 or t.stride(3) != 1 or t.shape != ref.shape or t.stride() != ref.stride() \
                    or t.dtype != ref.dtype:
                raise ValueError("k_new/v_new must be 4-D, channel-contiguous, same shape/strides/dtype")
    L = cache.layout
    if ref.shape[0] != L.batch or ref.shape[2] != L.n_kv_heads or ref.shape[3] != L.head_dim:
        raise ValueError("k_new/v_new shape does not match the layout")
    ptrs = cache.ptrs
    _check(lib().kvbfp_quantize_append(C.byref(L), C.byref(ptrs), _dev_ptr(k_new), _dev_ptr(v_new),
                                       _TORCH_DT[ref.dtype], ref.shape[1], ref.stride(0), ref.stride(1),
                                       ref.stride(2), int(pos0), _dev_ptr(pos_dev, torch.int32),
                                       _dev_ptr(perm_k, torch.int32), _dev_ptr(perm_v, torch.int32),
                                       _stream_ptr(stream)))


def dequantize(cache: Cache, which, t0, n_tok, dtype=torch.float32, perm=None, out=None, stream=None):
    """DEVICE, async.  Returns [batch][n_tok][n_kv_heads][head_dim] of `dtype`."""
    L = cache.layout
    if out is None:
        out = torch.empty((L.batch, n_tok, L.n_kv_heads, L.head_dim), dtype=dtype,
                          device=cache.k_mant.device if cache.k_mant is not None else cache.v_mant.device)
    ptrs = cache.ptrs
    _check(lib().kvbfp_dequantize(C.byref(L), C.byref(ptrs), int(which), int(t0), int(n_tok),
                                  _dev_ptr(perm, torch.int32), _dev_ptr(out), _TORCH_DT[out.dtype],
                                  _stream_ptr(stream)))
    return out


def decode_workspace_bytes(layout: Layout, n_q_heads, max_len) -> int:
    return int(lib().kvbfp_decode_workspace_bytes(C.byref(layout), int(n_q_heads), int(max_len)))


def _decode_common(cache, q, max_len, out, workspace):
    L = cache.layout
    if q.dim() != 3 or not q.is_contiguous():
        raise ValueError("q must be a contiguous [batch][n_q_heads][head_dim] tensor")
    n_q_heads = q.shape[1]
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need = decode_workspace_bytes(L, n_q_heads, max_len)
        if need == 0:
            _check(ERR_INVALID_ARG)
        workspace = torch.empty((need,), dtype=torch.uint8, device=q.device)
    return L, n_q_heads, out, workspace


def decode_attention(cache: Cache, q, max_len, softmax_scale, seq_len_dev=None, perm_k=None,
                     perm_v=None, out=None, workspace=None, stream=None):
    """DEVICE, async.  q: [batch][n_q_heads][head_dim] contiguous device tensor; returns `out`."""
    L, n_q_heads, out, workspace = _decode_common(cache, q, max_len, out, workspace)
    ptrs = cache.ptrs
    _check(lib().kvbfp_decode_attention(C.byref(L), C.byref(ptrs), n_q_heads, _dev_ptr(q),
                                        _TORCH_DT[q.dtype], _dev_ptr(seq_len_dev, torch.int32),
                                        int(max_len), float(softmax_scale),
                                        _dev_ptr(perm_k, torch.int32), _dev_ptr(perm_v, torch.int32),
                                        _dev_ptr(out), _dev_ptr(workspace), workspace.numel(),
                                        _stream_ptr(stream)))
    return out


def decode_attention_qbfp(cache: Cache, q, max_len, softmax_scale, q_mant_bits, seq_len_dev=None, perm_k=None,
                          perm_v=None, out=None, workspace=None, stream=None):
    """DEVICE, async.  decode_attention with the permuted query cast to BFP (q_mant_bits 4 or 8) first."""
    L, n_q_heads, out, workspace = _decode_common(cache, q, max_len, out, workspace)
    ptrs = cache.ptrs
    _check(lib().kvbfp_decode_attention_qbfp(C.byref(L), C.byref(ptrs), n_q_heads, _dev_ptr(q),
                                             _TORCH_DT[q.dtype], _dev_ptr(seq_len_dev, torch.int32),
                                             int(max_len), float(softmax_scale),
                                             _dev_ptr(perm_k, torch.int32), _dev_ptr(perm_v, torch.int32),
                                             int(q_mant_bits), _dev_ptr(out), _dev_ptr(workspace),
                                             workspace.numel(), _stream_ptr(stream)))
    return out


def decode_attention_rope(cache: Cache, q, max_len, softmax_scale, rope_theta, rope_partner, rope_sign,
                          seq_len_dev=None, perm_k=None, perm_v=None, out=None, workspace=None, stream=None,
                          profile=False):
    """DEVICE, async (synchronous with profile=True).  Keys cached before the rotary embedding, rotated at
    read; rope_theta / rope_partner / rope_sign: device tensors [n_kv_heads][head_dim] (float32, int32,
    float32) as permute_rope returns them.  Returns `out`, or (out, split_ms, combine_ms) with profile."""
    L, n_q_heads, out, workspace = _decode_common(cache, q, max_len, out, workspace)
    for t in (rope_theta, rope_partner, rope_sign):
        if t is None or tuple(t.shape) != (L.n_kv_heads, L.head_dim) or not t.is_contiguous():
            raise ValueError("rope_theta/rope_partner/rope_sign must be contiguous [n_kv_heads][head_dim] device tensors")
    ptrs = cache.ptrs
    ms = (C.c_float * 2)() if profile else None
    _check(lib().kvbfp_decode_attention_rope(C.byref(L), C.byref(ptrs), n_q_heads, _dev_ptr(q),
                                             _TORCH_DT[q.dtype], _dev_ptr(seq_len_dev, torch.int32),
                                             int(max_len), float(softmax_scale),
                                             _dev_ptr(perm_k, torch.int32), _dev_ptr(perm_v, torch.int32),
                                             _dev_ptr(rope_theta, torch.float32), _dev_ptr(rope_partner, torch.int32),
                                             _dev_ptr(rope_sign, torch.float32), _dev_ptr(out), _dev_ptr(workspace),
                                             workspace.numel(), _stream_ptr(stream), ms))
    return (out, float(ms[0]), float(ms[1])) if profile else out


def _check_table(block_table, batch):
    if block_table is None or block_table.dim() != 2 or block_table.dtype != torch.int32 or \
            not block_table.is_contiguous() or block_table.shape[0] != batch:
        raise ValueError("block_table must be a contiguous int32 device tensor [batch][pages per sequence]")


def quantize_append_paged(pool: Cache, block_table, k_new, v_new, pos0=0, pos_dev=None, perm_k=None, perm_v=None,
                          stream=None):
    """DEVICE, async.  quantize_append into a pool of pages (pool.layout: batch = pages, max_seq = tokens
    per page); block_table: int32 [batch][pages per sequence]."""
    ref = k_new if k_new is not None else v_new
    if ref is None:
        return
    for t in (k_new, v_new):
        if t is not None:
            if t.dim() != 4 or t.stride(3) != 1 or t.shape != ref.shape or t.stride() != ref.stride() \
                    or t.dtype != ref.dtype:
                raise ValueError("k_new/v_new must be 4-D, channel-contiguous, same shape/strides/dtype")
    _check_table(block_table, ref.shape[0])
    L = pool.layout
    if ref.shape[2] != L.n_kv_heads or ref.shape[3] != L.head_dim:
        raise ValueError("k_new/v_new shape does not match the layout")
    ptrs = pool.ptrs
    _check(lib().kvbfp_quantize_append_paged(C.byref(L), C.byref(ptrs), _dev_ptr(block_table, torch.int32),
                                             block_table.shape[1], ref.shape[0], _dev_ptr(k_new), _dev_ptr(v_new),
                                             _TORCH_DT[ref.dtype], ref.shape[1], ref.stride(0), ref.stride(1),
                                             ref.stride(2), int(pos0), _dev_ptr(pos_dev, torch.int32),
                                             _dev_ptr(perm_k, torch.int32), _dev_ptr(perm_v, torch.int32),
                                             _stream_ptr(stream)))


def dequantize_paged(pool: Cache, block_table, which, t0, n_tok, dtype=torch.float32, perm=None, out=None, stream=None):
    """DEVICE, async.  dequantize from a pool of pages; returns [batch][n_tok][n_kv_heads][head_dim]."""
    L = pool.layout
    if block_table is None or block_table.dim() != 2 or block_table.dtype != torch.int32 or not block_table.is_contiguous():
        raise ValueError("block_table must be a contiguous int32 device tensor [batch][pages per sequence]")
    batch = block_table.shape[0]
    if out is None:
        out = torch.empty((batch, n_tok, L.n_kv_heads, L.head_dim), dtype=dtype, device=block_table.device)
    ptrs = pool.ptrs
    _check(lib().kvbfp_dequantize_paged(C.byref(L), C.byref(ptrs), _dev_ptr(block_table, torch.int32), block_table.shape[1],
                                        batch, int(which), int(t0), int(n_tok), _dev_ptr(perm, torch.int32), _dev_ptr(out),
                                        _TORCH_DT[out.dtype], _stream_ptr(stream)))
    return out


def decode_workspace_bytes_paged(pool_layout: Layout, pages_per_seq, batch, n_q_heads, max_len):
    return int(lib().kvbfp_decode_workspace_bytes_paged(C.byref(pool_layout), int(pages_per_seq), int(batch),
                                                        int(n_q_heads), int(max_len)))


def decode_attention_paged(pool: Cache, block_table, q, max_len, softmax_scale, q_mant_bits=0, seq_len_dev=None,
                           perm_k=None, perm_v=None, out=None, workspace=None, stream=None, profile=False):
    """DEVICE, async (synchronous with profile=True).  decode_attention over a pool of pages.
    Returns `out`, or (out, split_ms, combine_ms) with profile."""
    L = pool.layout
    if q.dim() != 3 or not q.is_contiguous():
        raise ValueError("q must be a contiguous [batch][n_q_heads][head_dim] tensor")
    _check_table(block_table, q.shape[0])
    n_q_heads = q.shape[1]
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need = decode_workspace_bytes_paged(L, block_table.shape[1], q.shape[0], n_q_heads, max_len)
        if need == 0:
            _check(ERR_INVALID_ARG)
        workspace = torch.empty((need,), dtype=torch.uint8, device=q.device)
    ptrs = pool.ptrs
    ms = (C.c_float * 2)() if profile else None
    _check(lib().kvbfp_decode_attention_paged(C.byref(L), C.byref(ptrs), _dev_ptr(block_table, torch.int32),
                                              block_table.shape[1], q.shape[0], n_q_heads, _dev_ptr(q),
                                              _TORCH_DT[q.dtype], _dev_ptr(seq_len_dev, torch.int32), int(max_len),
                                              float(softmax_scale), _dev_ptr(perm_k, torch.int32),
                                              _dev_ptr(perm_v, torch.int32), int(q_mant_bits), _dev_ptr(out),
                                              _dev_ptr(workspace), workspace.numel(), _stream_ptr(stream), ms))
    return (out, float(ms[0]), float(ms[1])) if profile else out


def append_decode_attention_paged(pool: Cache, block_table, k_new, v_new, q, max_len, softmax_scale, seq_len_dev=None,
                                  perm_k=None, perm_v=None, q_mant_bits=0, out=None, workspace=None, stream=None):
    """DEVICE, async.  append_decode_attention over a pool of pages."""
    L = pool.layout
    if q.dim() != 3 or not q.is_contiguous():
        raise ValueError("q must be a contiguous [batch][n_q_heads][head_dim] tensor")
    _check_table(block_table, q.shape[0])
    if k_new.dim() == 4:
        k_new, v_new = k_new[:, 0], v_new[:, 0]
    if k_new.dim() != 3 or k_new.stride(2) != 1 or k_new.shape != v_new.shape or k_new.stride() != v_new.stride() \
            or k_new.dtype != q.dtype or v_new.dtype != q.dtype:
        raise ValueError("k_new/v_new must be [batch][n_kv_heads][head_dim], channel-contiguous, same strides, q's dtype")
    if k_new.shape != (q.shape[0], L.n_kv_heads, L.head_dim):
        raise ValueError("k_new/v_new shape does not match the layout")
    n_q_heads = q.shape[1]
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need = decode_workspace_bytes_paged(L, block_table.shape[1], q.shape[0], n_q_heads, max_len)
        if need == 0:
            _check(ERR_INVALID_ARG)
        workspace = torch.empty((need,), dtype=torch.uint8, device=q.device)
    ptrs = pool.ptrs
    _check(lib().kvbfp_append_decode_attention_paged(
        C.byref(L), C.byref(ptrs), _dev_ptr(block_table, torch.int32), block_table.shape[1], q.shape[0], n_q_heads,
        _dev_ptr(k_new), _dev_ptr(v_new), k_new.stride(0), k_new.stride(1), _dev_ptr(q), _TORCH_DT[q.dtype],
        _dev_ptr(seq_len_dev, torch.int32), int(max_len), float(softmax_scale), _dev_ptr(perm_k, torch.int32),
        _dev_ptr(perm_v, torch.int32), int(q_mant_bits), _dev_ptr(out), _dev_ptr(workspace), workspace.numel(),
        _stream_ptr(stream)))
    return out


def decode_attention_multi_paged(pool: Cache, block_table, q, max_len, softmax_scale, seq_len_dev=None, perm_k=None,
                                 perm_v=None, q_mant_bits=0, out=None, workspace=None, stream=None):
    """DEVICE, async.  decode_attention_multi over a pool of pages; q: [batch][n_q_tokens][n_q_heads][head_dim]."""
    L = pool.layout
    if q.dim() != 4 or not q.is_contiguous():
        raise ValueError("q must be a contiguous [batch][n_q_tokens][n_q_heads][head_dim] tensor")
    _check_table(block_table, q.shape[0])
    n_tok, n_q_heads = q.shape[1], q.shape[2]
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need = decode_workspace_bytes_paged(L, block_table.shape[1], q.shape[0], n_q_heads * n_tok, max_len)
        if need == 0:
            _check(ERR_INVALID_ARG)
        workspace = torch.empty((need,), dtype=torch.uint8, device=q.device)
    ptrs = pool.ptrs
    _check(lib().kvbfp_decode_attention_multi_paged(
        C.byref(L), C.byref(ptrs), _dev_ptr(block_table, torch.int32), block_table.shape[1], q.shape[0], n_q_heads,
        n_tok, _dev_ptr(q), _TORCH_DT[q.dtype], _dev_ptr(seq_len_dev, torch.int32), int(max_len),
        float(softmax_scale), _dev_ptr(perm_k, torch.int32), _dev_ptr(perm_v, torch.int32), int(q_mant_bits),
        _dev_ptr(out), _dev_ptr(workspace), workspace.numel(), _stream_ptr(stream)))
    return out


def decode_attention_profile(cache: Cache, q, max_len, softmax_scale, q_mant_bits=0, seq_len_dev=None, perm_k=None,
                             perm_v=None, out=None, workspace=None, stream=None):
    """DEVICE, synchronous.  Same launches as decode_attention_qbfp; returns (out, split_ms, combine_ms)."""
    L, n_q_heads, out, workspace = _decode_common(cache, q, max_len, out, workspace)
    ptrs = cache.ptrs
    ms = (C.c_float * 2)()
    _check(lib().kvbfp_decode_attention_profile(C.byref(L), C.byref(ptrs), n_q_heads, _dev_ptr(q),
                                                _TORCH_DT[q.dtype], _dev_ptr(seq_len_dev, torch.int32),
                                                int(max_len), float(softmax_scale),
                                                _dev_ptr(perm_k, torch.int32), _dev_ptr(perm_v, torch.int32),
                                                int(q_mant_bits), _dev_ptr(out), _dev_ptr(workspace),
                                                workspace.numel(), _stream_ptr(stream), ms))
    return out, float(ms[0]), float(ms[1])


def append_decode_attention(cache: Cache, k_new, v_new, q, max_len, softmax_scale, seq_len_dev=None, perm_k=None,
                            perm_v=None, q_mant_bits=0, out=None, workspace=None, stream=None):
    """DEVICE, async.  k_new / v_new: [batch][1][n_kv_heads][head_dim] (or [batch][n_kv_heads][head_dim]), the
    current token; stored at position seq_len - 1 (max_len - 1 without seq_len_dev), then attention."""
    L, n_q_heads, out, workspace = _decode_common(cache, q, max_len, out, workspace)
    if k_new.dim() == 4:
        k_new, v_new = k_new[:, 0], v_new[:, 0]
    if k_new.dim() != 3 or k_new.stride(2) != 1 or k_new.shape != v_new.shape or k_new.stride() != v_new.stride() \
            or k_new.dtype != q.dtype or v_new.dtype != q.dtype:
        raise ValueError("k_new/v_new must be [batch][n_kv_heads][head_dim], channel-contiguous, same strides, q's dtype")
    if k_new.shape != (L.batch, L.n_kv_heads, L.head_dim):
        raise ValueError("k_new/v_new shape does not match the layout")
    ptrs = cache.ptrs
    _check(lib().kvbfp_append_decode_attention(C.byref(L), C.byref(ptrs), n_q_heads, _dev_ptr(k_new), _dev_ptr(v_new),
                                               k_new.stride(0), k_new.stride(1), _dev_ptr(q), _TORCH_DT[q.dtype],
                                               _dev_ptr(seq_len_dev, torch.int32), int(max_len), float(softmax_scale),
                                               _dev_ptr(perm_k, torch.int32), _dev_ptr(perm_v, torch.int32),
                                               int(q_mant_bits), _dev_ptr(out), _dev_ptr(workspace), workspace.numel(),
                                               _stream_ptr(stream)))
    return out


def decode_attention_multi(cache: Cache, q, max_len, softmax_scale, seq_len_dev=None, perm_k=None, perm_v=None,
                           q_mant_bits=0, out=None, workspace=None, stream=None):
    """DEVICE, async.  q: [batch][n_q_tokens][n_q_heads][head_dim] contiguous: the last n_q_tokens tokens of every
    sequence (already cached), causal among themselves.  Returns out of the same shape."""
    L = cache.layout
    if q.dim() != 4 or not q.is_contiguous():
        raise ValueError("q must be a contiguous [batch][n_q_tokens][n_q_heads][head_dim] tensor")
    n_tok, n_q_heads = q.shape[1], q.shape[2]
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need = decode_workspace_bytes(L, n_q_heads * n_tok, max_len)
        if need == 0:
            _check(ERR_INVALID_ARG)
        workspace = torch.empty((need,), dtype=torch.uint8, device=q.device)
    ptrs = cache.ptrs
    _check(lib().kvbfp_decode_attention_multi(C.byref(L), C.byref(ptrs), n_q_heads, n_tok, _dev_ptr(q), _TORCH_DT[q.dtype],
                                              _dev_ptr(seq_len_dev, torch.int32), int(max_len), float(softmax_scale),
                                              _dev_ptr(perm_k, torch.int32), _dev_ptr(perm_v, torch.int32),
                                              int(q_mant_bits), _dev_ptr(out), _dev_ptr(workspace), workspace.numel(),
                                              _stream_ptr(stream)))
    return out


NOALLOC_SCRATCH_BYTES = 4 << 20


def decode_attention_noalloc(cache: Cache, q, max_len, softmax_scale, out, q_mant_bits=0, seq_len_dev=None,
                             perm_k=None, perm_v=None, stream=None):
    """DEVICE, async.  decode_attention_qbfp without a workspace: the split partials live in a fixed device
    array inside the library.  `out` is the caller's (nothing is allocated here either)."""
    L = cache.layout
    if q.dim() != 3 or not q.is_contiguous() or out.shape != q.shape or out.dtype != q.dtype or not out.is_contiguous():
        raise ValueError("q and out must be contiguous [batch][n_q_heads][head_dim] tensors of one dtype")
    ptrs = cache.ptrs
    _check(lib().kvbfp_decode_attention_noalloc(C.byref(L), C.byref(ptrs), q.shape[1], _dev_ptr(q), _TORCH_DT[q.dtype],
                                                _dev_ptr(seq_len_dev, torch.int32), int(max_len), float(softmax_scale),
                                                _dev_ptr(perm_k, torch.int32), _dev_ptr(perm_v, torch.int32),
                                                int(q_mant_bits), _dev_ptr(out), _stream_ptr(stream)))
    return out


def measure_stream_read(cache: Cache, n_tok, wgs_per_unit=0, sink=None, stream=None) -> float:
    """DEVICE, synchronous.  Plain read of rows [0, n_tok) of the four planes; returns the kernel time in ms."""
    L = cache.layout
    if sink is None:
        sink = torch.zeros((4,), dtype=torch.uint8, device=cache.k_mant.device)
    ptrs = cache.ptrs
    ms = C.c_float(0)
    _check(lib().kvbfp_measure_stream_read(C.byref(L), C.byref(ptrs), int(n_tok), int(wgs_per_unit), _dev_ptr(sink),
                                           _stream_ptr(stream), C.byref(ms)))
    return float(ms.value)


def decode_attention_profile_ring(caches, n_launches, q, max_len, softmax_scale, q_mant_bits=0, seq_len_dev=None,
                                  perm_k=None, perm_v=None, out=None, workspace=None, stream=None):
    """DEVICE, synchronous.  The split pass n_launches times back to back over `caches` (a list of Cache objects of
    one layout, used cyclically), then the combine pass as often; returns (out, split_ms, combine_ms) per launch."""
    L, n_q_heads, out, workspace = _decode_common(caches[0], q, max_len, out, workspace)
    arr = (CachePtrs * len(caches))(*[c.ptrs for c in caches])
    ms = (C.c_float * 2)()
    _check(lib().kvbfp_decode_attention_profile_ring(C.byref(L), arr, len(caches), int(n_launches), n_q_heads, _dev_ptr(q),
                                                     _TORCH_DT[q.dtype], _dev_ptr(seq_len_dev, torch.int32), int(max_len),
                                                     float(softmax_scale), _dev_ptr(perm_k, torch.int32),
                                                     _dev_ptr(perm_v, torch.int32), int(q_mant_bits), _dev_ptr(out),
                                                     _dev_ptr(workspace), workspace.numel(), _stream_ptr(stream), ms))
    return out, float(ms[0]), float(ms[1])
