"""ctypes front end of the CPU oracle (``blockffn_oracle.c``).

TEST INFRASTRUCTURE.  Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py`` may import this package.  It never imports the HIP package and the HIP
package never imports it.

All arguments are host numpy arrays.  Weights are fp32 arrays or uint16 arrays holding bf16
bit patterns, laid out one row per output feature (``w_router [E][d]``, ``w_up`` / ``w_gate``
``[E][d_e][d]``, ``w_down [E][d][d_e]``).
"""

from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "blockffn_oracle.c")
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None
_native = False


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over chunks/tokens only, no fast-math)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def use_native_build() -> str:
    """Switch this process to a build of the SAME source with ``-O3 -march=native`` for the host it
    runs on: the build the timed CPU baseline uses.  It is compiled on the spot into the host's
    temp directory (code for this host's instruction set must not travel to another machine) and
    keeps ISO floating-point semantics (-std=c11: no contraction, no fast-math), so it computes
    what the -O2 build computes."""
    global _lib, _native
    import tempfile
    so = os.path.join(tempfile.gettempdir(), "liboracle_native_%d.so" % os.getuid())
    cmd = ["gcc", "-O3", "-march=native", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", so, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    _lib = ctypes.CDLL(so)
    for name in ("oracle_router", "oracle_chunk_union", "oracle_sparse_ffn", "oracle_dense_ffn"):
        getattr(_lib, name).restype = ctypes.c_int
    _native = True
    return so


class _Layer(ctypes.Structure):
    _fields_ = [
        ("d", ctypes.c_int32), ("n_experts", ctypes.c_int32), ("d_e", ctypes.c_int32),
        ("wdtype", ctypes.c_int32), ("gated", ctypes.c_int32), ("pad_", ctypes.c_int32),
        ("eps", ctypes.c_double),
        ("w_router", ctypes.c_void_p), ("b_router", ctypes.c_void_p), ("g_rms", ctypes.c_void_p),
        ("w_up", ctypes.c_void_p), ("w_gate", ctypes.c_void_p), ("w_down", ctypes.c_void_p),
    ]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_SO)
        for name in ("oracle_router", "oracle_chunk_union", "oracle_sparse_ffn", "oracle_dense_ffn"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


class Layer:
    """One layer's parameters, kept alive for the lifetime of the object."""

    def __init__(self, w_router, w_up, w_down, w_gate=None, b_router=None, g_rms=None, eps=1e-6):
        self.wdtype = 1 if w_router.dtype == np.uint16 else 0
        want = np.uint16 if self.wdtype else np.float32
        self.E, self.d = w_router.shape
        self.d_e = w_up.shape[1]
        assert w_up.shape == (self.E, self.d_e, self.d)
        assert w_down.shape == (self.E, self.d, self.d_e)
        assert w_gate is None or w_gate.shape == w_up.shape
        assert self.E <= 1024 and self.d_e <= 4096
        self._keep = []
        def c(a, dt):
            if a is None:
                return None
            a = np.ascontiguousarray(a, dtype=dt)
            self._keep.append(a)
            return a
        self.w_router, self.w_up, self.w_down = c(w_router, want), c(w_up, want), c(w_down, want)
        self.w_gate = c(w_gate, want)
        self.b_router, self.g_rms = c(b_router, np.float32), c(g_rms, np.float32)
        self.gated = self.w_gate is not None
        self.eps = float(eps)
        self.W = (self.E + 63) // 64
        self.c = _Layer(self.d, self.E, self.d_e, self.wdtype, int(self.gated), 0, self.eps,
                        _ptr(self.w_router), _ptr(self.b_router), _ptr(self.g_rms),
                        _ptr(self.w_up), _ptr(self.w_gate), _ptr(self.w_down))


def router(L: Layer, x: np.ndarray, return_a0: bool = False):
    """Eq. 3: returns (scores fp32 [T][E], token_mask uint64 [T][W]) and optionally A^0 fp64."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    T = x.shape[0]
    assert x.shape == (T, L.d)
    scores = np.empty((T, L.E), np.float32)
    mask = np.empty((T, L.W), np.uint64)
    a0 = np.empty((T, L.E), np.float64) if return_a0 else None
    rc = lib.oracle_router(ctypes.byref(L.c), _ptr(x), ctypes.c_int64(T), _ptr(scores), _ptr(mask), _ptr(a0))
    assert rc == 0
    return (scores, mask, a0) if return_a0 else (scores, mask)


def chunk_union(token_mask: np.ndarray, k: int, E: int, stats: Optional[np.ndarray] = None):
    """Union(x) per chunk: (union_mask [C][W], active_idx [C][E] ascending with -1 tail,
    n_active [C]); ``stats`` (int64[2]) is added to: [inactive (token,expert) pairs,
    inactive (chunk,expert) pairs]."""
    lib = _load()
    token_mask = np.ascontiguousarray(token_mask, dtype=np.uint64)
    T, W = token_mask.shape
    assert W == (E + 63) // 64 and T % k == 0
    C = T // k
    union = np.empty((C, W), np.uint64)
    idx = np.empty((C, E), np.int32)
    n = np.empty((C,), np.int32)
    if stats is not None:
        assert stats.dtype == np.int64 and stats.shape == (2,)
    rc = lib.oracle_chunk_union(_ptr(token_mask), ctypes.c_int64(C), ctypes.c_int32(k), ctypes.c_int32(E),
                                _ptr(union), _ptr(idx), _ptr(n), _ptr(stats))
    assert rc == 0
    return union, idx, n


def sparse_ffn(L: Layer, x, scores, token_mask, active_idx, n_active, k: int) -> np.ndarray:
    """Chunk-sparse FFN (Sec. 3.3): y fp64 [T][d]."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    token_mask = np.ascontiguousarray(token_mask, dtype=np.uint64)
    active_idx = np.ascontiguousarray(active_idx, dtype=np.int32)
    n_active = np.ascontiguousarray(n_active, dtype=np.int32)
    T = x.shape[0]
    assert T % k == 0 and scores.shape == (T, L.E) and token_mask.shape == (T, L.W)
    C = T // k
    assert active_idx.shape == (C, L.E) and n_active.shape == (C,)
    y = np.empty((T, L.d), np.float64)
    rc = lib.oracle_sparse_ffn(ctypes.byref(L.c), _ptr(x), _ptr(scores), _ptr(token_mask), _ptr(active_idx),
                               _ptr(n_active), ctypes.c_int64(C), ctypes.c_int32(k), _ptr(y))
    assert rc == 0
    return y


def dense_ffn(L: Layer, x, scores) -> np.ndarray:
    """Eq. 1 with every expert evaluated: y fp64 [T][d]."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    T = x.shape[0]
    assert scores.shape == (T, L.E)
    y = np.empty((T, L.d), np.float64)
    rc = lib.oracle_dense_ffn(ctypes.byref(L.c), _ptr(x), _ptr(scores), ctypes.c_int64(T), _ptr(y))
    assert rc == 0
    return y


def forward(L: Layer, x, k: int):
    """Router -> union -> chunk-sparse FFN; returns a dict of every intermediate."""
    scores, mask = router(L, x)
    stats = np.zeros(2, np.int64)
    union, idx, n = chunk_union(mask, k, L.E, stats)
    y = sparse_ffn(L, x, scores, mask, idx, n, k)
    return dict(scores=scores, token_mask=mask, union_mask=union, active_idx=idx, n_active=n, stats=stats, y=y)
