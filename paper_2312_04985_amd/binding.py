"""Thin ctypes binding over libsparq.so (include/sparq.h): same names, argument marshalling only.

torch supplies device memory (`tensor.data_ptr()`) and the current HIP stream; every step of
the decode path runs inside the library's kernels.  There is no fallback: if the library has
not been built, or a tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch   # imported before the library is loaded so both use the same HIP runtime

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsparq.so")

SPARQ_F16, SPARQ_BF16 = 0, 1
SPARQ_FLAG_NO_REALLOC, SPARQ_FLAG_GQA_SHARED, SPARQ_FLAG_RAGGED_BATCH = 1, 2, 4
SPARQ_FLAG_TAU_SQRT_DH, SPARQ_FLAG_TAU_SQRT_R, SPARQ_FLAG_SINGLE_K, SPARQ_FLAG_TILED_K = 8, 16, 32, 64
SPARQ_ERR_APPEND_FULL, SPARQ_ERR_EMPTY_SEQ, SPARQ_ERR_IDX_TRUNCATED, SPARQ_ERR_BAD_SEQ_LEN, SPARQ_ERR_INTERNAL = 1, 2, 4, 8, 16
SPARQ_OK, SPARQ_EINVAL, SPARQ_EUNSUPPORTED, SPARQ_EWORKSPACE, SPARQ_ELAUNCH, SPARQ_ETOOLARGE = 0, -1, -2, -3, -4, -5

EXPORTS = ["sparq_workspace_bytes", "sparq_workspace_init", "sparq_kv_append", "sparq_decode", "sparq_decode_noalloc", "sparq_decode_step",
           "dense_decode", "sparq_async_error", "sparq_copy_probe", "sparq_read_probe", "sparq_decode_plan",
           "sparq_stage_clocks", "sparq_status_string"]


class SparqShape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("H_kv", ctypes.c_int32),
                ("S_max", ctypes.c_int32), ("d_h", ctypes.c_int32), ("r", ctypes.c_int32),
                ("k", ctypes.c_int32), ("dtype", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("local_window", ctypes.c_int32), ("S_bound", ctypes.c_int32)]


class SparqCache(ctypes.Structure):
    _fields_ = [("K", ctypes.c_void_p), ("Kt", ctypes.c_void_p), ("V", ctypes.c_void_p),
                ("v_mean", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p)]


class SparqError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn}: {status_string(status)} ({status})")


_lib = None


def load() -> ctypes.CDLL:
    """Load libsparq.so built in-tree (paper_2312_04985_amd/build.py).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2312_04985_amd.build` "
                                "(or __graft_entry__.build()) first; there is no CPU fallback")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    shp, cch = ctypes.POINTER(SparqShape), ctypes.POINTER(SparqCache)
    L.sparq_workspace_bytes.argtypes = [shp, ctypes.POINTER(sz)]
    L.sparq_workspace_init.argtypes = [vp, sz, vp]
    L.sparq_kv_append.argtypes = [shp, cch, vp, vp, i32, vp, vp, sz, vp]
    L.sparq_decode.argtypes = [shp, cch, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
    L.sparq_decode_noalloc.argtypes = [shp, cch, vp, vp, vp, vp, vp, i32, vp, vp, vp]
    L.sparq_decode_step.argtypes = [shp, cch, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
    L.dense_decode.argtypes = [shp, cch, vp, vp, vp, sz, vp]
    L.sparq_async_error.argtypes = [vp, ctypes.POINTER(i32), vp]
    L.sparq_copy_probe.argtypes = [vp, vp, sz, vp]
    L.sparq_read_probe.argtypes = [vp, sz, vp, sz, vp]
    L.sparq_status_string.argtypes = [ctypes.c_int]
    L.sparq_decode_plan.argtypes = [shp]
    L.sparq_stage_clocks.argtypes = [shp, ctypes.POINTER(sz), ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.sparq_decode_plan.restype = ctypes.c_char_p
    L.sparq_status_string.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("sparq_status_string", "sparq_decode_plan"):
            getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def sparq_decode_plan(shape: SparqShape) -> str:
    return load().sparq_decode_plan(ctypes.byref(shape)).decode()


def sparq_stage_clocks(shape: SparqShape):
    """(offset_bytes, n_workgroups, stamps_per_workgroup) of the time stamps a profiling build leaves in the workspace."""
    off, n, m = ctypes.c_size_t(0), ctypes.c_int32(0), ctypes.c_int32(0)
    _check("sparq_stage_clocks", load().sparq_stage_clocks(ctypes.byref(shape), ctypes.byref(off), ctypes.byref(n), ctypes.byref(m)))
    return off.value, n.value, m.value


def status_string(status: int) -> str:
    return load().sparq_status_string(int(status)).decode()


def _check(fn: str, status: int) -> None:
    if status != SPARQ_OK:
        raise SparqError(fn, status)


def _dev(t: Optional[torch.Tensor], name: str, dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live in GPU memory (got {t.device}); the library has no CPU path")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def make_shape(B, H, H_kv, S_max, d_h, r, k, dtype, flags=0, local_window=0, S_bound=0) -> SparqShape:
    code = {torch.float16: SPARQ_F16, torch.bfloat16: SPARQ_BF16}.get(dtype, dtype)
    return SparqShape(B, H, H_kv, S_max, d_h, r, k, int(code), flags, local_window, S_bound)


def make_cache(K, Kt, V, v_mean, seq_lens) -> SparqCache:
    return SparqCache(_dev(K, "K"), _dev(Kt, "Kt"), _dev(V, "V"), _dev(v_mean, "v_mean", torch.float32),
                      _dev(seq_lens, "seq_lens", torch.int32))


def sparq_workspace_bytes(shape: SparqShape) -> int:
    out = ctypes.c_size_t(0)
    _check("sparq_workspace_bytes", load().sparq_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return int(out.value)


def sparq_workspace_init(workspace: torch.Tensor, stream=None) -> None:
    _check("sparq_workspace_init",
           load().sparq_workspace_init(_dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                       _stream(stream)))


def sparq_kv_append(shape, cache, k_new, v_new, n_new, n_new_per_seq, workspace, stream=None) -> None:
    _check("sparq_kv_append",
           load().sparq_kv_append(ctypes.byref(shape), ctypes.byref(cache), _dev(k_new, "k_new"), _dev(v_new, "v_new"),
                                  int(n_new), _dev(n_new_per_seq, "n_new_per_seq", torch.int32),
                                  _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                  _stream(stream)))


def sparq_decode(shape, cache, q, k_per_seq, out, alpha_out, idx_out, chan_out, workspace, stream=None) -> None:
    idx_stride = 0 if idx_out is None else idx_out.shape[-1]
    _check("sparq_decode",
           load().sparq_decode(ctypes.byref(shape), ctypes.byref(cache), _dev(q, "q"),
                               _dev(k_per_seq, "k_per_seq", torch.int32), _dev(out, "out"),
                               _dev(alpha_out, "alpha_out", torch.float32), _dev(idx_out, "idx_out", torch.int32),
                               idx_stride, _dev(chan_out, "chan_out", torch.int32),
                               _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                               _stream(stream)))


def sparq_decode_noalloc(shape, cache, q, k_per_seq, out, alpha_out, idx_out, chan_out, error_word=None, stream=None) -> None:
    """sparq_decode on the library's built-in scratch buffer (no workspace argument, nothing allocated)."""
    idx_stride = 0 if idx_out is None else idx_out.shape[-1]
    _check("sparq_decode_noalloc",
           load().sparq_decode_noalloc(ctypes.byref(shape), ctypes.byref(cache), _dev(q, "q"),
                                       _dev(k_per_seq, "k_per_seq", torch.int32), _dev(out, "out"),
                                       _dev(alpha_out, "alpha_out", torch.float32), _dev(idx_out, "idx_out", torch.int32),
                                       idx_stride, _dev(chan_out, "chan_out", torch.int32),
                                       _dev(error_word, "error_word", torch.int32), _stream(stream)))


def sparq_decode_step(shape, cache, k_new, v_new, v_mean_next, seq_lens_next, q, k_per_seq, out, alpha_out,
                      idx_out, chan_out, workspace, stream=None) -> None:
    idx_stride = 0 if idx_out is None else idx_out.shape[-1]
    _check("sparq_decode_step",
           load().sparq_decode_step(ctypes.byref(shape), ctypes.byref(cache), _dev(k_new, "k_new"), _dev(v_new, "v_new"),
                                    _dev(v_mean_next, "v_mean_next", torch.float32),
                                    _dev(seq_lens_next, "seq_lens_next", torch.int32), _dev(q, "q"),
                                    _dev(k_per_seq, "k_per_seq", torch.int32), _dev(out, "out"),
                                    _dev(alpha_out, "alpha_out", torch.float32), _dev(idx_out, "idx_out", torch.int32),
                                    idx_stride, _dev(chan_out, "chan_out", torch.int32),
                                    _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                    _stream(stream)))


def dense_decode(shape, cache, q, out, workspace, stream=None) -> None:
    _check("dense_decode",
           load().dense_decode(ctypes.byref(shape), ctypes.byref(cache), _dev(q, "q"), _dev(out, "out"),
                               _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                               _stream(stream)))


def sparq_async_error(workspace, stream=None) -> int:
    flag = ctypes.c_int32(0)
    _check("sparq_async_error", load().sparq_async_error(_dev(workspace, "workspace"), ctypes.byref(flag), _stream(stream)))
    return int(flag.value)


def sparq_copy_probe(dst, src, n_bytes: int, stream=None) -> None:
    _check("sparq_copy_probe", load().sparq_copy_probe(_dev(dst, "dst"), _dev(src, "src"), int(n_bytes), _stream(stream)))


def sparq_read_probe(src, n_bytes: int, sink, stream=None) -> None:
    _check("sparq_read_probe", load().sparq_read_probe(_dev(src, "src"), int(n_bytes), _dev(sink, "sink"),
                                                       sink.numel() * sink.element_size(), _stream(stream)))
