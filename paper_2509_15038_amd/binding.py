"""ctypes binding of libcurdkv.so: the same entry points as include/curdkv.h,
argument marshalling only.  Every step of the path runs in the HIP kernels.

torch appears here only as the owner of device memory and streams: tensors are
passed as raw pointers.  If the compiled library is missing the import of any
entry point fails loudly; there is no fallback.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcurdkv.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_HIP, ERR_OOM, ERR_TOO_LARGE = 0, -1, -2, -3, -4, -5
DTYPE_F32, DTYPE_BF16 = 0, 1
_DTYPES = {"fp32": DTYPE_F32, "bf16": DTYPE_BF16}

EXPORTS = ["curdkv_create", "curdkv_destroy", "curdkv_sketch_host", "curdkv_set_sketch",
           "curdkv_uses_fused_kernel", "curdkv_scores", "curdkv_fold", "curdkv_select", "curdkv_compact", "curdkv_compress",
           "curdkv_adaptive_budgets", "curdkv_adaptive_budgets_noalloc", "curdkv_compress_adaptive", "curdkv_scores_append", "curdkv_normalise", "curdkv_strerror"]


class CurdkvConfig(C.Structure):
    _fields_ = [("layers", C.c_int32), ("kv_heads", C.c_int32), ("group_size", C.c_int32),
                ("head_dim", C.c_int32), ("sketch_dim", C.c_int32), ("dtype", C.c_int32),
                ("score_source", C.c_int32), ("no_projection", C.c_int32),
                ("max_tokens", C.c_int64), ("seed", C.c_uint64)]


class CurdkvError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2509_15038_amd.build` "
            "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    cfgp = C.POINTER(CurdkvConfig)
    L.curdkv_create.argtypes = [C.POINTER(vp), cfgp]
    L.curdkv_destroy.argtypes = [vp]
    L.curdkv_sketch_host.argtypes = [cfgp, i32, i32, vp]
    L.curdkv_set_sketch.argtypes = [vp, i32, i32, vp]
    L.curdkv_uses_fused_kernel.argtypes = [vp, i64]
    L.curdkv_scores.argtypes = [vp, vp, vp, i64, vp, vp]
    L.curdkv_fold.argtypes = [vp, vp, i64, vp, vp]
    L.curdkv_select.argtypes = [vp, vp, i64, vp, i32, vp, vp, vp]
    L.curdkv_compact.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp]
    L.curdkv_compress.argtypes = [vp, vp, vp, i64, vp, i32, vp, vp, vp, vp, vp, vp]
    L.curdkv_adaptive_budgets.argtypes = [vp, vp, i64, i32, i32, C.c_double, vp, vp]
    L.curdkv_adaptive_budgets_noalloc.argtypes = [vp, vp, i64, i32, i32, C.c_double, vp, vp]
    L.curdkv_compress_adaptive.argtypes = [vp, vp, vp, i64, i32, i32, C.c_double, vp, vp, vp, vp, vp, vp, vp]
    L.curdkv_scores_append.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp, vp]
    L.curdkv_normalise.argtypes = [vp, vp, vp, i64, i64, vp, vp]
    L.curdkv_strerror.argtypes = [C.c_int]
    L.curdkv_strerror.restype = C.c_char_p
    for name in EXPORTS[:-1]:
        getattr(L, name).restype = C.c_int
    _lib = L
    return L


def strerror(code: int) -> str:
    return lib().curdkv_strerror(int(code)).decode()


SCORE_KV, SCORE_KEY, SCORE_VALUE = 0, 1, 2
_SOURCES = {"kv": SCORE_KV, "k": SCORE_KEY, "v": SCORE_VALUE}


def make_config(layers, kv_heads, group_size, head_dim, sketch_dim, dtype, max_tokens, seed,
                source="kv", projection=True):
    return CurdkvConfig(int(layers), int(kv_heads), int(group_size), int(head_dim),
                        int(sketch_dim), _DTYPES[dtype] if isinstance(dtype, str) else int(dtype),
                        _SOURCES[source] if isinstance(source, str) else int(source),
                        0 if projection else 1,
                        int(max_tokens), int(seed) & 0xFFFFFFFFFFFFFFFF)


def curdkv_sketch_host(cfg: CurdkvConfig, layer: int, head: int) -> np.ndarray:
    """G of one (layer, head) as float32 [head_dim, sketch_dim]; host only, no GPU."""
    out = np.empty((cfg.head_dim, cfg.sketch_dim), dtype=np.float32)
    rc = lib().curdkv_sketch_host(C.byref(cfg), layer, head, out.ctypes.data)
    if rc != OK:
        raise CurdkvError(rc, "curdkv_sketch_host")
    return out


def _ptr(t) -> int:
    """Device (torch) or host (numpy) buffer -> address; None -> NULL."""
    if t is None:
        return 0
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class Context:
    """Owns one curdkv_ctx.  Methods mirror the C entry points and return the raw
    status code through CurdkvError on failure."""

    def __init__(self, layers, kv_heads, group_size, head_dim, sketch_dim, dtype, max_tokens, seed,
                 source="kv", projection=True):
        self.cfg = make_config(layers, kv_heads, group_size, head_dim, sketch_dim, dtype,
                               max_tokens, seed, source, projection)
        self._h = C.c_void_p()
        self._destroy = lib().curdkv_destroy        # kept here: module globals may be gone at interpreter exit
        rc = lib().curdkv_create(C.byref(self._h), C.byref(self.cfg))
        if rc != OK:
            self._h = None
            raise CurdkvError(rc, "curdkv_create")

    def close(self):
        h = getattr(self, "_h", None)
        if h is not None and h.value:
            self._h = None
            self._destroy(h)

    __del__ = close

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    @property
    def heads(self) -> int:
        return self.cfg.layers * self.cfg.kv_heads

    def set_sketch(self, layer: int, head: int, G: np.ndarray):
        G = np.ascontiguousarray(G, dtype=np.float32)
        assert G.shape == (self.cfg.head_dim, self.cfg.sketch_dim)
        rc = lib().curdkv_set_sketch(self._h, layer, head, G.ctypes.data)
        if rc != OK:
            raise CurdkvError(rc, "curdkv_set_sketch")

    def scores(self, K, V, n: int, scores, stream=None):
        rc = lib().curdkv_scores(self._h, _ptr(K), _ptr(V), int(n), _ptr(scores), _stream(stream))
        if rc != OK:
            raise CurdkvError(rc, "curdkv_scores")

    def fold(self, scores_q, n: int, scores, stream=None):
        rc = lib().curdkv_fold(self._h, _ptr(scores_q), int(n), _ptr(scores), _stream(stream))
        if rc != OK:
            raise CurdkvError(rc, "curdkv_fold")

    def select(self, scores, n: int, budgets: np.ndarray, n_sink: int, offsets: np.ndarray,
               indices, stream=None):
        assert budgets.dtype == np.int32 and offsets.dtype == np.int64
        assert budgets.size == self.heads and offsets.size == self.heads + 1
        rc = lib().curdkv_select(self._h, _ptr(scores), int(n), budgets.ctypes.data, int(n_sink),
                                 offsets.ctypes.data, _ptr(indices), _stream(stream))
        if rc != OK:
            raise CurdkvError(rc, "curdkv_select")

    def compact(self, K, V, n: int, indices, offsets: np.ndarray, K_out, V_out, stream=None):
        assert offsets.dtype == np.int64 and offsets.size == self.heads + 1
        rc = lib().curdkv_compact(self._h, _ptr(K), _ptr(V), int(n), _ptr(indices),
                                  offsets.ctypes.data, _ptr(K_out), _ptr(V_out), _stream(stream))
        if rc != OK:
            raise CurdkvError(rc, "curdkv_compact")

    def compress(self, K, V, n: int, budgets: np.ndarray, n_sink: int, offsets: np.ndarray,
                 scores, indices, K_out, V_out, stream=None):
        assert budgets.dtype == np.int32 and offsets.dtype == np.int64
        assert budgets.size == self.heads and offsets.size == self.heads + 1
        rc = lib().curdkv_compress(self._h, _ptr(K), _ptr(V), int(n), budgets.ctypes.data,
                                   int(n_sink), offsets.ctypes.data, _ptr(scores), _ptr(indices),
                                   _ptr(K_out), _ptr(V_out), _stream(stream))
        if rc != OK:
            raise CurdkvError(rc, "curdkv_compress")

    def uses_fused_kernel(self, n: int) -> bool:
        rc = lib().curdkv_uses_fused_kernel(self._h, int(n))
        if rc < 0:
            raise CurdkvError(rc, "curdkv_uses_fused_kernel")
        return bool(rc)

    def adaptive_budgets(self, scores, n: int, budget: int, n_sink: int, alpha: float, budgets_out,
                         stream=None):
        rc = lib().curdkv_adaptive_budgets(self._h, _ptr(scores), int(n), int(budget), int(n_sink),
                                           float(alpha), _ptr(budgets_out), _stream(stream))
        if rc != OK:
            raise CurdkvError(rc, "curdkv_adaptive_budgets")

    def adaptive_budgets_noalloc(self, scores, n: int, budget: int, n_sink: int, alpha: float, budgets_out,
                                 stream=None):
        rc = lib().curdkv_adaptive_budgets_noalloc(self._h, _ptr(scores), int(n), int(budget), int(n_sink),
                                                   float(alpha), _ptr(budgets_out), _stream(stream))
        if rc != OK:
            raise CurdkvError(rc, "curdkv_adaptive_budgets_noalloc")

    def compress_adaptive(self, K, V, n: int, budget: int, n_sink: int, alpha: float, scores,
                          budgets_out, offsets_out, indices, K_out, V_out, stream=None):
        rc = lib().curdkv_compress_adaptive(self._h, _ptr(K), _ptr(V), int(n), int(budget), int(n_sink),
                                            float(alpha), _ptr(scores), _ptr(budgets_out),
                                            _ptr(offsets_out), _ptr(indices), _ptr(K_out), _ptr(V_out),
                                            _stream(stream))
        if rc != OK:
            raise CurdkvError(rc, "curdkv_compress_adaptive")

    def scores_append(self, K_new, V_new, m: int, n_old: int, stride: int, raw, sums, stream=None):
        rc = lib().curdkv_scores_append(self._h, _ptr(K_new), _ptr(V_new), int(m), int(n_old),
                                        int(stride), _ptr(raw), _ptr(sums), _stream(stream))
        if rc != OK:
            raise CurdkvError(rc, "curdkv_scores_append")

    def normalise(self, raw, sums, stride: int, n: int, scores, stream=None):
        rc = lib().curdkv_normalise(self._h, _ptr(raw), _ptr(sums), int(stride), int(n),
                                    _ptr(scores), _stream(stream))
        if rc != OK:
            raise CurdkvError(rc, "curdkv_normalise")
