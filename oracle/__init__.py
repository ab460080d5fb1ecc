"""ctypes front end of the CPU oracle (``svdp_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this module;
it is called by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The arithmetic is all in the C file; this
wrapper only marshals numpy arrays (float32 in, float64 out).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "svdp_oracle.c")
_SO = os.path.join(_HERE, "libsvdp_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, OpenMP across independent outputs)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_SO)
        c_int, c_vp = ctypes.c_int, ctypes.c_void_p
        L.oracle_dense_ffn.argtypes = [c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp, c_int, c_vp, c_vp]
        L.oracle_dense_ffn.restype = None
        L.oracle_predict.argtypes = [c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp, c_vp]
        L.oracle_predict.restype = None
        L.oracle_compact.argtypes = [c_int, c_int, c_vp, c_vp, c_vp]
        L.oracle_compact.restype = c_int
        L.oracle_sparse_ffn.argtypes = [c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp, c_vp, c_int, c_int, c_vp, c_vp]
        L.oracle_sparse_ffn.restype = None
        L.oracle_stack_glue.argtypes = [c_int, c_vp, c_vp, c_vp, ctypes.c_double, c_vp]
        L.oracle_stack_glue.restype = None
        _lib = L
    return _lib


def set_threads(n: int) -> None:
    """Number of OpenMP threads the C oracle uses from now on (timing only; the results do not depend on it)."""
    _load()
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def _f32(a, shape=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _x2(x, d) -> np.ndarray:
    x = _f32(x)
    if x.ndim == 1:
        x = x[None, :]
    assert x.ndim == 2 and x.shape[1] == d, (x.shape, d)
    return x


def dense_ffn(W_gate, W_up, W_downT, x, drelu: bool = False, return_z: bool = False):
    """y [B][d] (float64) of the dense ReGLU FFN; x is [B][d] or [d]."""
    W_gate = _f32(W_gate)
    D, d = W_gate.shape
    W_up, W_downT, x = _f32(W_up, (D, d)), _f32(W_downT, (D, d)), _x2(x, d)
    B = x.shape[0]
    y = np.empty((B, d), dtype=np.float64)
    z = np.empty((B, D), dtype=np.float64) if return_z else None
    _load().oracle_dense_ffn(d, D, B, _p(W_gate), _p(W_up), _p(W_downT), _p(x), int(drelu), _p(y), _p(z))
    return (y, z) if return_z else y


def predict(P, Q, b, x) -> np.ndarray:
    """Predictor scores s [B][D] (float64)."""
    P = _f32(P)
    d, r = P.shape
    Q = _f32(Q)
    D = Q.shape[0]
    assert Q.shape == (D, r)
    b, x = _f32(b, (D,)), _x2(x, d)
    B = x.shape[0]
    s = np.empty((B, D), dtype=np.float64)
    _load().oracle_predict(d, D, r, B, _p(P), _p(Q), _p(b), _p(x), _p(s))
    return s


def compact(s) -> Tuple[np.ndarray, np.ndarray]:
    """(mask [D] uint8, idx [nnz] int32 ascending) of the union mask of scores s [B][D]."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    if s.ndim == 1:
        s = s[None, :]
    B, D = s.shape
    m = np.zeros(D, dtype=np.uint8)
    idx = np.zeros(max(D, 1), dtype=np.int32)
    nnz = _load().oracle_compact(D, B, _p(s), _p(m), _p(idx))
    return m, idx[:nnz].copy()


def sparse_ffn(W_gate, W_up, W_downT, x, idx, drelu: bool = False, return_h: bool = False):
    """y [B][d] (float64) of the sparse FFN over the index list idx (shared by the batch)."""
    W_gate = _f32(W_gate)
    D, d = W_gate.shape
    W_up, W_downT, x = _f32(W_up, (D, d)), _f32(W_downT, (D, d)), _x2(x, d)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    nnz = int(idx.shape[0])
    assert nnz == 0 or (idx.min() >= 0 and idx.max() < D)
    B = x.shape[0]
    y = np.empty((B, d), dtype=np.float64)
    h = np.empty((B, max(nnz, 1)), dtype=np.float64) if return_h else None
    idx_arg = idx if nnz else np.zeros(1, dtype=np.int32)
    _load().oracle_sparse_ffn(d, D, B, _p(W_gate), _p(W_up), _p(W_downT), _p(x), _p(idx_arg), nnz,
                              int(drelu), _p(y), _p(h))
    return (y, h[:, :nnz]) if return_h else y


def stack_glue(x, y, shift, eps: float = 1e-6) -> np.ndarray:
    """RMS-normalised residual x + y plus a shift vector (glue of the stacked benchmark)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.ascontiguousarray(y, dtype=np.float64)
    shift = np.ascontiguousarray(shift, dtype=np.float64)
    out = np.empty_like(x)
    _load().oracle_stack_glue(x.shape[0], _p(x), _p(y), _p(shift), float(eps), _p(out))
    return out


def ffn_step(layer_f32: dict, x, drelu: bool = False):
    """Whole decode step: scores -> union mask -> index list -> sparse FFN.  Returns (s, mask, idx, y)."""
    s = predict(layer_f32["P"], layer_f32["Q"], layer_f32["b"], x)
    m, idx = compact(s)
    y = sparse_ffn(layer_f32["W_gate"], layer_f32["W_up"], layer_f32["W_downT"], x, idx, drelu=drelu)
    return s, m, idx, y
