"""ctypes front end of the CPU oracle (oracle/kvbfp_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of bench.py.  The product package never imports this module.

All arrays are numpy, C-contiguous.  Floating inputs are float32 (widen
fp16/bf16 exactly before calling); results are float64 or uint8/int32.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libkvbfp_oracle.so")
_SRC = os.path.join(_HERE, "kvbfp_oracle.cpp")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (CPU only)."""
    stale = (not os.path.exists(_SO)) or os.path.getmtime(_SO) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["sh", os.path.join(_HERE, "build.sh")])
    return _SO


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
        for name in ("kvo_calibrate_perm", "kvo_permute_weights", "kvo_permute_weight_columns", "kvo_quantize_append",
                     "kvo_dequantize", "kvo_decode_attention", "kvo_scores", "kvo_permute_rope",
                     "kvo_decode_attention_rope"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _p(a, ctype):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(ctype))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def plane_shapes(B, H, D, n, p, S_max):
    return (B, H, S_max, D * p // 8), (B, H, S_max, D // n)


def calibrate_perm(x, stat="maxabs", descending=False):
    """x: float32 [n_samples][n_heads][D] -> int32 [n_heads][D] (Alg. 1 steps 1-2)."""
    x = _f32(x)
    S, H, D = x.shape
    perm = np.empty((H, D), dtype=np.int32)
    rc = lib().kvo_calibrate_perm(_p(x, C.c_float), C.c_int64(S), C.c_int32(H), C.c_int32(D),
                                  C.c_int64(H * D), C.c_int64(D), C.c_int64(1),
                                  C.c_int32({"maxabs": 0, "l2": 1}[stat]),
                                  C.c_int32(1 if descending else 0), _p(perm, C.c_int32))
    if rc != 0:
        raise ValueError("kvo_calibrate_perm rc=%d" % rc)
    return perm


def calibrate_perm_from_weights(w, n_heads, D, descending=False):
    """w: float32 [n_heads*D][row_len] (rows of W_k) -> int32 [n_heads][D] by row norm."""
    w = _f32(w)
    rows, row_len = w.shape
    assert rows == n_heads * D
    perm = np.empty((n_heads, D), dtype=np.int32)
    rc = lib().kvo_calibrate_perm(_p(w, C.c_float), C.c_int64(row_len), C.c_int32(n_heads),
                                  C.c_int32(D), C.c_int64(1), C.c_int64(D * row_len),
                                  C.c_int64(row_len), C.c_int32(1),
                                  C.c_int32(1 if descending else 0), _p(perm, C.c_int32))
    if rc != 0:
        raise ValueError("kvo_calibrate_perm rc=%d" % rc)
    return perm


def permute_weights(w, n_heads, D, perm, heads_per_perm=1):
    w = _f32(w)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    out = np.empty_like(w)
    rc = lib().kvo_permute_weights(_p(w, C.c_float), _p(out, C.c_float), C.c_int32(n_heads),
                                   C.c_int32(D), C.c_int64(w.shape[1]), C.c_int32(heads_per_perm),
                                   _p(perm, C.c_int32))
    if rc != 0:
        raise ValueError("kvo_permute_weights rc=%d" % rc)
    return out


def permute_weight_columns(w, n_heads, D, perm, heads_per_perm=1):
    """w: [n_rows][n_heads*D]; Sec. III, last paragraph."""
    w = _f32(w)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    out = np.empty_like(w)
    rc = lib().kvo_permute_weight_columns(_p(w, C.c_float), _p(out, C.c_float), C.c_int64(w.shape[0]),
                                          C.c_int32(n_heads), C.c_int32(D), C.c_int32(heads_per_perm),
                                          _p(perm, C.c_int32))
    if rc != 0:
        raise ValueError("kvo_permute_weight_columns rc=%d" % rc)
    return out


def quantize_append(x, n, p, S_max, pos, perm=None, mant=None, exp=None):
    """x: float32 [B][n_new][H][D].  Returns (mant, exp) planes (allocated zeroed if None)."""
    x = _f32(x)
    B, n_new, H, D = x.shape
    ms, es = plane_shapes(B, H, D, n, p, S_max)
    if mant is None:
        mant = np.zeros(ms, dtype=np.uint8)
    if exp is None:
        exp = np.zeros(es, dtype=np.uint8)
    assert mant.shape == ms and exp.shape == es and mant.flags.c_contiguous and exp.flags.c_contiguous
    pos = np.ascontiguousarray(np.broadcast_to(np.asarray(pos, dtype=np.int64), (B,)))
    if perm is not None:
        perm = np.ascontiguousarray(perm, dtype=np.int32)
        assert perm.shape == (H, D)
    rc = lib().kvo_quantize_append(C.c_int32(B), C.c_int32(H), C.c_int32(D), C.c_int32(n),
                                   C.c_int32(p), C.c_int64(S_max), _p(x, C.c_float),
                                   C.c_int32(n_new), _p(pos, C.c_int64), _p(perm, C.c_int32),
                                   _p(mant, C.c_uint8), _p(exp, C.c_uint8))
    if rc != 0:
        raise ValueError("kvo_quantize_append rc=%d" % rc)
    return mant, exp


def dequantize(mant, exp, D, n, p, t0, n_tok, perm=None):
    """Returns float64 [B][n_tok][H][D] (Eq. 1)."""
    B, H, S_max, _ = mant.shape
    assert mant.shape == plane_shapes(B, H, D, n, p, S_max)[0]
    out = np.empty((B, n_tok, H, D), dtype=np.float64)
    if perm is not None:
        perm = np.ascontiguousarray(perm, dtype=np.int32)
    rc = lib().kvo_dequantize(C.c_int32(B), C.c_int32(H), C.c_int32(D), C.c_int32(n), C.c_int32(p),
                              C.c_int64(S_max), _p(mant, C.c_uint8), _p(exp, C.c_uint8),
                              C.c_int64(t0), C.c_int64(n_tok), _p(perm, C.c_int32),
                              _p(out, C.c_double))
    if rc != 0:
        raise ValueError("kvo_dequantize rc=%d" % rc)
    return out


def decode_attention(k_mant, k_exp, v_mant, v_exp, D, n, p, q, seq_len, softmax_scale,
                     perm_k=None, perm_v=None, q_mant_bits=0):
    """q: float32 [B][Hq][D] -> float64 [B][Hq][D]."""
    q = _f32(q)
    B, Hq, Dq = q.shape
    Bc, Hkv, S_max, _ = k_mant.shape
    assert Bc == B and Dq == D
    for a in (k_mant, k_exp, v_mant, v_exp):
        assert a.flags.c_contiguous and a.dtype == np.uint8
    seq_len = np.ascontiguousarray(np.broadcast_to(np.asarray(seq_len, dtype=np.int64), (B,)))
    if perm_k is not None:
        perm_k = np.ascontiguousarray(perm_k, dtype=np.int32)
    if perm_v is not None:
        perm_v = np.ascontiguousarray(perm_v, dtype=np.int32)
    out = np.empty((B, Hq, D), dtype=np.float64)
    rc = lib().kvo_decode_attention(C.c_int32(B), C.c_int32(Hkv), C.c_int32(Hq), C.c_int32(D),
                                    C.c_int32(n), C.c_int32(p), C.c_int64(S_max),
                                    _p(k_mant, C.c_uint8), _p(k_exp, C.c_uint8),
                                    _p(v_mant, C.c_uint8), _p(v_exp, C.c_uint8),
                                    _p(q, C.c_float), _p(seq_len, C.c_int64),
                                    C.c_double(float(softmax_scale)),
                                    _p(perm_k, C.c_int32), _p(perm_v, C.c_int32),
                                    C.c_int32(q_mant_bits), _p(out, C.c_double))
    if rc != 0:
        raise ValueError("kvo_decode_attention rc=%d" % rc)
    return out


def permute_rope(theta, perm, pair_layout=0):
    """Alg. 1 step 5.  theta: float32 [D/2]; perm: int32 [n_heads][D]; pair_layout 0 = consecutive
    pairs (Eq. (RoFreq)), 1 = half-split (footnote of Sec. III).
    -> (theta' float32 [n_heads][D], partner' int32 [n_heads][D], sign' float32 [n_heads][D])."""
    theta = _f32(theta)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    n_heads, D = perm.shape
    assert theta.shape == (D // 2,)
    th = np.empty((n_heads, D), dtype=np.float32)
    pa = np.empty((n_heads, D), dtype=np.int32)
    sg = np.empty((n_heads, D), dtype=np.float32)
    rc = lib().kvo_permute_rope(C.c_int32(D), C.c_int32(n_heads), C.c_int32(pair_layout), _p(theta, C.c_float),
                                _p(perm, C.c_int32), _p(th, C.c_float), _p(pa, C.c_int32), _p(sg, C.c_float))
    if rc != 0:
        raise ValueError("kvo_permute_rope rc=%d" % rc)
    return th, pa, sg


def decode_attention_rope(k_mant, k_exp, v_mant, v_exp, D, n, p, q, seq_len, softmax_scale,
                          rope_theta, rope_partner, rope_sign, perm_k=None, perm_v=None):
    """Keys cached before the rotary embedding, rotated at read with the reordered parameters of
    permute_rope.  q: float32 [B][Hq][D] (already rotated) -> float64 [B][Hq][D]."""
    q = _f32(q)
    B, Hq, Dq = q.shape
    Bc, Hkv, S_max, _ = k_mant.shape
    assert Bc == B and Dq == D
    for a in (k_mant, k_exp, v_mant, v_exp):
        assert a.flags.c_contiguous and a.dtype == np.uint8
    seq_len = np.ascontiguousarray(np.broadcast_to(np.asarray(seq_len, dtype=np.int64), (B,)))
    if perm_k is not None:
        perm_k = np.ascontiguousarray(perm_k, dtype=np.int32)
    if perm_v is not None:
        perm_v = np.ascontiguousarray(perm_v, dtype=np.int32)
    rope_theta = _f32(rope_theta)
    rope_sign = _f32(rope_sign)
    rope_partner = np.ascontiguousarray(rope_partner, dtype=np.int32)
    assert rope_theta.shape == (Hkv, D) and rope_partner.shape == (Hkv, D) and rope_sign.shape == (Hkv, D)
    out = np.empty((B, Hq, D), dtype=np.float64)
    rc = lib().kvo_decode_attention_rope(C.c_int32(B), C.c_int32(Hkv), C.c_int32(Hq), C.c_int32(D),
                                         C.c_int32(n), C.c_int32(p), C.c_int64(S_max),
                                         _p(k_mant, C.c_uint8), _p(k_exp, C.c_uint8),
                                         _p(v_mant, C.c_uint8), _p(v_exp, C.c_uint8),
                                         _p(q, C.c_float), _p(seq_len, C.c_int64),
                                         C.c_double(float(softmax_scale)),
                                         _p(perm_k, C.c_int32), _p(perm_v, C.c_int32),
                                         _p(rope_theta, C.c_float), _p(rope_partner, C.c_int32),
                                         _p(rope_sign, C.c_float), _p(out, C.c_double))
    if rc != 0:
        raise ValueError("kvo_decode_attention_rope rc=%d" % rc)
    return out


def scores(k_mant_rows, k_exp_rows, D, n, p, q_perm, softmax_scale):
    """k_mant_rows: uint8 [L][D*p/8], k_exp_rows: uint8 [L][D/n], q_perm: float64 [D]."""
    L = k_mant_rows.shape[0]
    q_perm = np.ascontiguousarray(q_perm, dtype=np.float64)
    k_mant_rows = np.ascontiguousarray(k_mant_rows)
    k_exp_rows = np.ascontiguousarray(k_exp_rows)
    s = np.empty((L,), dtype=np.float64)
    rc = lib().kvo_scores(C.c_int32(D), C.c_int32(n), C.c_int32(p), _p(k_mant_rows, C.c_uint8),
                          _p(k_exp_rows, C.c_uint8), C.c_int64(L), _p(q_perm, C.c_double),
                          C.c_double(float(softmax_scale)), _p(s, C.c_double))
    if rc != 0:
        raise ValueError("kvo_scores rc=%d" % rc)
    return s
