"""CPU oracle of the offline predictor build: data-aware factorisation (Alg. 1)
and greedy bias calibration (Alg. 2, App. A "Greedy threshold selection").

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` and by the ``cpu_baseline`` leg
of ``bench.py --calibrate``; nothing in the product package imports it.

Plain numpy, fp64, the algorithms' steps in the paper's order and notation.
LAPACK routines (Cholesky, SVD, triangular solve) and a stable sort serve as
steps.  Two places fix a precision because a floating-point comparison decides
an integer there: the step costs of the greedy loop and the group sums of the
Kendall check are sums of fp32 weights accumulated left to right in fp32 (the
precision the GPU kernels take the same decisions in); everything else is fp64.

Tokens are rows here: ``X`` is ``[T][d]`` (the paper's ``X`` is ``d x N``).
"""
from __future__ import annotations

import heapq
from typing import Dict, Tuple

import numpy as np
import scipy.linalg


# ---------------------------------------------------------------------------
# Alg. 1: building SVD predictors with data whitening (Sec. 4.1)
# ---------------------------------------------------------------------------
def whitened_factors(W_gate: np.ndarray, X: np.ndarray, r: int) -> Tuple[np.ndarray, np.ndarray]:
    """A [D][r], B [r][d] with A B ~= W_gate, minimising ||W X^T - A B X^T||_F over rank-r products.

    S = Cholesky(X^T X) (lower triangular, S S^T = the paper's X X^T); U, Sigma, V = SVD(W_gate S);
    A = U_r Sigma_r; B = V_r^T S^-1.
    """
    W = np.asarray(W_gate, dtype=np.float64)
    Xr = np.asarray(X, dtype=np.float64)
    S = np.linalg.cholesky(Xr.T @ Xr)
    U, sig, Vt = np.linalg.svd(W @ S, full_matrices=False)
    A = U[:, :r] * sig[:r]
    # B = V_r^T S^-1  <=>  B S = V_r^T  <=>  S^T B^T = V_r
    B = scipy.linalg.solve_triangular(S.T, Vt[:r].T, lower=False).T
    return A, B


# ---------------------------------------------------------------------------
# Alg. 2, first two lines: neurons' importance and predictor outputs
# ---------------------------------------------------------------------------
def damage_weights(W_gate: np.ndarray, W_up: np.ndarray, W_downT: np.ndarray, X: np.ndarray) -> np.ndarray:
    """w[i][t] = |ReLU(W_gate[i,:] x_t) * (W_up[i,:] x_t)|^2 * ||W_down[:, i]||_2^2   (App. A, damage weight).

    W_downT is [D][d]: row i is column i of W_down.
    """
    Wg, Wu, Wd, Xr = (np.asarray(a, dtype=np.float64) for a in (W_gate, W_up, W_downT, X))
    g = Wg @ Xr.T
    u = Wu @ Xr.T
    z = np.maximum(g, 0.0) * u
    col_norm2 = np.sum(Wd * Wd, axis=1)
    return z * z * col_norm2[:, None]


def proxy_scores(A: np.ndarray, B: np.ndarray, X: np.ndarray) -> np.ndarray:
    """s[i][t] = (A B x_t)_i, the inner product first (B x), as the predictor evaluates it."""
    A, B, Xr = (np.asarray(a, dtype=np.float64) for a in (A, B, X))
    return A @ (B @ Xr.T)


# ---------------------------------------------------------------------------
# Alg. 2: greedy bias calibration
# ---------------------------------------------------------------------------
def _seq_sum_f32(block: np.ndarray) -> np.ndarray:
    """Row-wise left-to-right fp32 sum of an fp32 array [n][m]."""
    acc = np.zeros(block.shape[0], dtype=np.float32)
    for j in range(block.shape[1]):
        acc = (acc + block[:, j]).astype(np.float32)
    return acc


def required_drops(sparsity: float, D: int, T: int) -> int:
    """Smallest integer n with n / (D T) >= sparsity: the loop of Alg. 2 runs while the count is below it."""
    n = int(np.ceil(sparsity * D * T))
    while n > 0 and (n - 1) >= sparsity * D * T:
        n -= 1
    return min(max(n, 0), D * T)


def greedy_bias(w: np.ndarray, s: np.ndarray, need: int, eta: int) -> Dict[str, np.ndarray]:
    """Alg. 2 from its sort onward, on given weights w [D][T] and proxy scores s [D][T] (both taken as fp32).

    need = the number of (neuron, sample) pairs with s <= tau at which the while loop stops
    (``required_drops(sparsity, D, T)``).  Readings of the printed algorithm: the pointer update is
    k <- min(k + eta, T) (the listing prints max); the arg min takes the smallest neuron index among
    equal costs; a neuron without any positive weight starts (and stays) at k = T; sorting is stable
    (equal scores keep sample order); the count of dropped pairs is the literal #{t : s <= tau}.
    Returns b = -tau, the pointers k (1-based counts), tau, the number of greedy steps and the final count.
    """
    w = np.ascontiguousarray(w, dtype=np.float32)
    s = np.ascontiguousarray(s, dtype=np.float32)
    D, T = s.shape
    assert w.shape == (D, T) and eta >= 1
    order = np.argsort(s, axis=1, kind="stable")
    ss = np.take_along_axis(s, order, axis=1)            # s_{i,(1)} <= ... <= s_{i,(T)}
    ww = np.take_along_axis(w, order, axis=1)

    k = np.empty(D, dtype=np.int64)                       # k_i = min{k : w_{i,(k)} > 0}
    for i in range(D):
        pos = np.flatnonzero(ww[i] > 0)
        k[i] = pos[0] + 1 if pos.size else T

    def dropped(i: int, ki: int) -> int:                  # #{t : s_i^(t) <= s_{i,(ki)}}
        return int(np.searchsorted(ss[i], ss[i, ki - 1], side="right"))

    def step_cost(i: int) -> float:                       # C_i(k + eta) - C_i(k) with the padding of Alg. 2
        if k[i] >= T:
            return float("inf")
        seg = ww[i, k[i]:min(k[i] + eta, T)]
        return float(_seq_sum_f32(seg[None, :])[0])

    total = sum(dropped(i, int(k[i])) for i in range(D))
    heap = [(step_cost(i), i) for i in range(D)]
    heapq.heapify(heap)
    steps = 0
    while total < need:
        cost, i = heapq.heappop(heap)                     # greedy step: smallest cost, then smallest index
        if cost == float("inf"):
            break
        knew = min(int(k[i]) + eta, T)
        total += dropped(i, knew) - dropped(i, int(k[i]))
        k[i] = knew
        steps += 1
        heapq.heappush(heap, (step_cost(i), i))
    tau = ss[np.arange(D), k - 1].astype(np.float32)
    return {"b": -tau, "k": k.astype(np.int32), "tau": tau, "steps": steps, "count": int(total)}


def calibration_loss(w: np.ndarray, s: np.ndarray, tau: np.ndarray) -> float:
    """L(tau) = sum_t sum_i w_i^(t) 1[s_i^(t) <= tau_i]   (App. A, empirical loss), fp64."""
    w = np.asarray(w, dtype=np.float64)
    return float(np.sum(w * (np.asarray(s) <= np.asarray(tau)[:, None])))


# ---------------------------------------------------------------------------
# App. A, remark on the role of the rank-r approximation: Kendall check
# ---------------------------------------------------------------------------
def kendall_tau(w: np.ndarray, s: np.ndarray, eta: int) -> np.ndarray:
    """tau_i^K = 1 - K_d / (M (M - 1)) for every neuron: K_d = number of pairs m1 < m2 of the
    non-overlapping eta-step sums S_i^(m) (samples sorted by proxy score, M = floor(T / eta)) that are
    strictly out of order (S^(m1) > S^(m2)).  The normalisation is the printed one, under which a
    fully reversed sequence gives 0.5.  M < 2 gives 1.  Group sums are fp32, accumulated left to right."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    s = np.ascontiguousarray(s, dtype=np.float32)
    D, T = s.shape
    M = T // eta
    if M < 2:
        return np.ones(D, dtype=np.float64)
    order = np.argsort(s, axis=1, kind="stable")
    ww = np.take_along_axis(w, order, axis=1)[:, :M * eta].reshape(D, M, eta)
    S = np.stack([_seq_sum_f32(ww[:, m, :]) for m in range(M)], axis=1)     # [D][M]
    out = np.empty(D, dtype=np.float64)
    iu = np.triu_indices(M, k=1)
    for i in range(D):
        kd = int(np.count_nonzero(S[i][iu[0]] > S[i][iu[1]]))
        out[i] = 1.0 - kd / (M * (M - 1))
    return out
