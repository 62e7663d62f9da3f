"""ctypes front-end of the C oracle (oracle/sparq_oracle.c) plus the definitional
KV-append oracle.  TEST INFRASTRUCTURE ONLY: used by tests/, the smoke check and the
benchmark's cpu_baseline leg.  It imports nothing from the product package and the
product package imports nothing from here.

Inputs are numpy arrays of raw 16-bit codes (dtype uint16) together with a dtype code
(0 = IEEE binary16, 1 = bfloat16); all arithmetic is fp64.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

F16, BF16 = 0, 1
NO_REALLOC, GQA_SHARED = 1, 2
TAU_SQRT_DH, TAU_SQRT_R = 8, 16

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        # SPARQ_ORACLE_SANITIZED=1: the AddressSanitizer + UBSan build (the process must preload libasan)
        path = _build.build(sanitize=bool(os.environ.get("SPARQ_ORACLE_SANITIZED")))
        L = ctypes.CDLL(path)
        c_int, c_uint, c_long, vp = ctypes.c_int, ctypes.c_uint, ctypes.c_long, ctypes.c_void_p
        L.oracle_to_double.argtypes = [c_int, vp, c_long, vp]
        L.oracle_mean_value.argtypes = [c_int, c_int, c_int, c_int, c_int, vp, vp, vp]
        L.oracle_dense_decode.argtypes = [c_int] * 6 + [vp] * 5
        L.oracle_sparq_decode.argtypes = [c_int] * 9 + [c_uint] + [vp] * 6 + [c_int] + [vp] * 6
        L.oracle_num_threads.restype = c_int
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _u16(a, shape):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "pass raw 16-bit codes (tensor.view(torch.int16).numpy().view(np.uint16))"
    assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


def _i32(a, shape):
    a = np.ascontiguousarray(a, dtype=np.int32)
    assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


def to_double(codes: np.ndarray, dtype: int) -> np.ndarray:
    """Exact widening of 16-bit codes by the oracle's own converter."""
    codes = np.ascontiguousarray(codes, dtype=np.uint16)
    out = np.empty(codes.shape, dtype=np.float64)
    rc = lib().oracle_to_double(dtype, _ptr(codes), codes.size, _ptr(out))
    assert rc == 0
    return out


def num_threads() -> int:
    return int(lib().oracle_num_threads())


@dataclass
class SparqResult:
    y: np.ndarray        # [B,H,d_h] fp64
    alpha: np.ndarray    # [B,H]
    tau: np.ndarray      # [B,H]
    i1: np.ndarray       # [B,H,r]  ascending channel indices
    i2: np.ndarray       # [B,H,k_stride] ascending positions, -1 padded
    z: np.ndarray | None # [B,H,S_max] approximate logits (dot / tau), 0 beyond the sequence


def sparq_decode(K, V, q, seq_lens, *, r, k, dtype, flags=0, k_per_seq=None, given_i2=None,
                 want_z=False, local_window=0) -> SparqResult:
    """SparQ decode step (Section 4, Steps 1-3) for a whole batch."""
    B, H_kv, S_max, d_h = K.shape
    H = q.shape[1]
    K = _u16(K, (B, H_kv, S_max, d_h)); V = _u16(V, (B, H_kv, S_max, d_h)); q = _u16(q, (B, H, d_h))
    seq_lens = _i32(seq_lens, (B,))
    kps = None if k_per_seq is None else _i32(k_per_seq, (B,))
    kb = kps if kps is not None else np.full(B, k, dtype=np.int32)
    k_stride = int(max(1, np.max(np.minimum(kb, seq_lens))))
    if given_i2 is not None:
        given_i2 = np.ascontiguousarray(given_i2, dtype=np.int32)
        assert given_i2.shape[:2] == (B, H)
        k_stride = given_i2.shape[2]
    y = np.empty((B, H, d_h)); alpha = np.empty((B, H)); tau = np.empty((B, H))
    i1 = np.empty((B, H, r), dtype=np.int32); i2 = np.empty((B, H, k_stride), dtype=np.int32)
    z = np.empty((B, H, S_max)) if want_z else None
    rc = lib().oracle_sparq_decode(B, H, H_kv, S_max, d_h, r, k, local_window, dtype, flags, _ptr(K), _ptr(V), _ptr(q),
                                   _ptr(seq_lens), _ptr(kps), _ptr(given_i2), k_stride,
                                   _ptr(y), _ptr(alpha), _ptr(tau), _ptr(i1), _ptr(i2), _ptr(z))
    if rc != 0:
        raise ValueError(f"oracle_sparq_decode: invalid arguments (code {rc})")
    return SparqResult(y, alpha, tau, i1, i2, z)


def dense_decode(K, V, q, seq_lens, *, dtype) -> np.ndarray:
    """Dense single-query attention, Eq. (2)."""
    B, H_kv, S_max, d_h = K.shape
    H = q.shape[1]
    K = _u16(K, (B, H_kv, S_max, d_h)); V = _u16(V, (B, H_kv, S_max, d_h)); q = _u16(q, (B, H, d_h))
    seq_lens = _i32(seq_lens, (B,))
    y = np.empty((B, H, d_h))
    rc = lib().oracle_dense_decode(B, H, H_kv, S_max, d_h, dtype, _ptr(K), _ptr(V), _ptr(q), _ptr(seq_lens), _ptr(y))
    if rc != 0:
        raise ValueError(f"oracle_dense_decode: invalid arguments (code {rc})")
    return y


def mean_value(V, seq_lens, *, dtype) -> np.ndarray:
    """v-bar = (1/S) sum_i v_i per (batch, KV head), Section 3 'Mean value reallocation'."""
    B, H_kv, S_max, d_h = V.shape
    V = _u16(V, (B, H_kv, S_max, d_h)); seq_lens = _i32(seq_lens, (B,))
    out = np.empty((B, H_kv, d_h))
    rc = lib().oracle_mean_value(B, H_kv, S_max, d_h, dtype, _ptr(V), _ptr(seq_lens), _ptr(out))
    assert rc == 0
    return out


def kv_append(K, Kt, V, seq_lens, k_new, v_new, *, dtype):
    """What the cache must hold after appending n_new rows per sequence, by definition:
    the rows land at positions S_b .. S_b+n_new-1 of K and V, Kt is the transpose of K on
    its last two axes, v-bar is the mean of the first S_b+n_new value rows (Section 3 and
    the 'Storing K twice' paragraph of Appendix F).  Arrays are raw uint16 codes; returns
    new copies (K, Kt, V, v_bar fp64, seq_lens)."""
    K = np.array(K, copy=True); Kt = np.array(Kt, copy=True); V = np.array(V, copy=True)
    seq = np.array(seq_lens, dtype=np.int32, copy=True)
    B, H_kv, S_max, d_h = K.shape
    k_new = np.asarray(k_new).reshape(B, H_kv, -1, d_h); v_new = np.asarray(v_new).reshape(B, H_kv, -1, d_h)
    n_new = k_new.shape[2]
    for b in range(B):
        s = int(seq[b])
        if s + n_new > S_max:
            continue   # sequence is full: left untouched
        K[b, :, s:s + n_new, :] = k_new[b]
        V[b, :, s:s + n_new, :] = v_new[b]
        Kt[b, :, :, s:s + n_new] = np.swapaxes(k_new[b], -1, -2)
        seq[b] = s + n_new
    return K, Kt, V, mean_value(V, seq, dtype=dtype), seq
