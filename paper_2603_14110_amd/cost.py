"""Multiplication and HBM-byte accounting for the sparse decode step.

``mults_dense`` / ``mults_sparse`` are the paper's complexity model (Sec. 4.2,
"Algorithmic Complexity"): a dense ReGLU FFN costs 3dD multiplications, the
sparse path r(d+D) for the predictor, d(1-s)D for the gate rows and 2d(1-s')D
for the up and down rows, with s the predicted and s' the realised sparsity.

``bytes_sparse`` / ``bytes_dense`` count the bytes the method has to read and
write per step (weights and predictor factors really touched, the bias, the
tokens in and the outputs out); they are what the benchmark divides by the
measured time to get achieved GB/s.
"""
from __future__ import annotations


def mults_dense(d: int, D: int) -> float:
    return 3.0 * d * D


def mults_sparse(d: int, D: int, r: int, s_pred: float, s_real: float) -> float:
    return r * (d + D) + d * (1.0 - s_pred) * D + 2.0 * d * (1.0 - s_real) * D


def bytes_predictor(d: int, D: int, r: int, w: int) -> int:
    """P [d][r] and Q [D][r] in w-byte elements plus the fp32 bias."""
    return (d * r + D * r) * w + 4 * D


def bytes_rows(d: int, nnz: int, w: int) -> int:
    """nnz rows each of W_gate, W_up and W_down^T."""
    return 3 * nnz * d * w


def bytes_rows_sequential(d: int, nnz, alive, w: int):
    """Sequential pipeline (Sec. 4.2): the gate row of every listed neuron, the up and down rows only of
    the `alive` ones whose gate came out positive."""
    return (nnz + 2 * alive) * d * w


def bytes_io(d: int, B: int, w: int) -> int:
    """x in (storage dtype) and y out (fp32)."""
    return B * d * w + 4 * B * d


def bytes_sparse(d: int, D: int, r: int, nnz: int, B: int, w: int) -> int:
    return bytes_predictor(d, D, r, w) + bytes_rows(d, nnz, w) + bytes_io(d, B, w)


def bytes_dense(d: int, D: int, B: int, w: int) -> int:
    return 3 * d * D * w + bytes_io(d, B, w)
