"""Pins of the offline-build oracle (oracle/calib.py: Alg. 1 and Alg. 2 of the paper) against
what the paper and the mathematics fix: a hand-worked example, brute force on tiny instances,
closed forms of the whitened truncation error, library routines, and the runtime oracle."""
import itertools

import numpy as np
import pytest
import scipy.stats

from conftest import read_golden
from oracle import calib


# ---------------------------------------------------------------- Alg. 2 -----
def test_worked_example_by_hand():
    g = read_golden("calibration_worked_example.txt")
    s, w, eta = g["s"], g["w"], int(g["eta"])
    for tag in ("a", "b"):
        need = calib.required_drops(float(g[f"sparsity_{tag}"]), 2, 6)
        assert need == int(g[f"need_{tag}"])
        out = calib.greedy_bias(w, s, need, eta)
        assert out["k"].tolist() == g[f"k_{tag}"].astype(int).tolist()
        assert out["tau"].tolist() == g[f"tau_{tag}"].tolist()
        assert out["steps"] == int(g[f"steps_{tag}"])
        assert out["count"] == need
        assert np.array_equal(out["b"], -out["tau"])
        assert calib.calibration_loss(w, s, out["tau"]) == float(g[f"loss_{tag}"])
    # no greedy step at all: the pointers are the first positive weights
    out = calib.greedy_bias(w, s, 0, eta)
    assert out["k"].tolist() == g["k_start"].astype(int).tolist() and out["steps"] == 0


def _brute_force_min_loss(ww_sorted, K, kmin):
    """min over k_i in [kmin_i, T], sum k_i = K of sum_i C_i(k_i) (App. A, fixed drop budget problem)."""
    D, T = ww_sorted.shape
    C = np.concatenate([np.zeros((D, 1)), np.cumsum(ww_sorted, axis=1)], axis=1)
    best = None
    for ks in itertools.product(*[range(kmin[i], T + 1) for i in range(D)]):
        if sum(ks) == K:
            v = sum(C[i, ks[i]] for i in range(D))
            best = v if best is None else min(best, v)
    return best


@pytest.mark.parametrize("seed", range(6))
def test_greedy_is_optimal_under_monotone_marginals(seed):
    """App. A theorem: with non-decreasing marginal weights per neuron the greedy choice attains the
    minimum of the fixed-budget problem -- checked against enumeration of every feasible pointer vector."""
    rng = np.random.default_rng(seed)
    D, T = 3, 5
    s = rng.standard_normal((D, T)).astype(np.float32)      # the oracle takes scores as fp32
    order = np.argsort(s, axis=1)
    ww = np.sort(rng.integers(1, 9, (D, T)).astype(np.float64), axis=1)       # monotone after sorting by s
    w = np.empty_like(ww)
    np.put_along_axis(w, order, ww, axis=1)
    for K in range(D, D * T + 1):                                             # all weights > 0: k starts at 1
        out = calib.greedy_bias(w, s, K, 1)
        assert out["count"] == K and int(out["k"].sum()) == K
        got = calib.calibration_loss(w, s, out["tau"])
        assert got == _brute_force_min_loss(ww, K, [1] * D), (seed, K)


def test_greedy_invariants_and_readings():
    rng = np.random.default_rng(3)
    D, T, eta = 40, 64, 4
    s = rng.standard_normal((D, T)).astype(np.float32)
    g = s + 0.3 * rng.standard_normal((D, T))
    w = (np.maximum(g, 0) ** 2 * rng.uniform(0.5, 2, (D, 1))).astype(np.float32)
    w[7] = 0.0                                                                # a neuron that is never active
    prev_k, prev_loss = None, -1.0
    for sp in (0.3, 0.6, 0.8, 0.95, 1.0):
        need = calib.required_drops(sp, D, T)
        out = calib.greedy_bias(w, s, need, eta)
        k, tau = out["k"], out["tau"]
        cnt = int(np.sum(s <= tau[:, None]))
        assert cnt == out["count"] >= need                                    # the loop's exit condition
        assert np.all((1 <= k) & (k <= T))                                    # min(k + eta, T), not max
        assert k[7] == T                                                      # nothing to lose: fully dropped
        for i in range(D):
            assert tau[i] == np.sort(s[i])[k[i] - 1]                          # tau is the k-th smallest score
        loss = calib.calibration_loss(w, s, tau)
        if prev_k is not None:
            assert np.all(k >= prev_k) and loss >= prev_loss                  # more sparsity: pointers only advance
        prev_k, prev_loss = k, loss
        if out["steps"]:
            # one step fewer would not have reached the target: replay and stop early
            less = calib.greedy_bias(w, s, out["count"] - eta * 2 if out["count"] - eta * 2 > 0 else 0, eta)
            assert less["steps"] < out["steps"]
    assert prev_k.tolist() == [T] * D                                         # sparsity 1: everything dropped


def test_equal_costs_take_the_smallest_index():
    s = np.tile(np.arange(4, dtype=np.float32), (3, 1))
    w = np.ones((3, 4), dtype=np.float32)
    out = calib.greedy_bias(w, s, 3 + 2, 1)            # start: 3 pairs; two steps, all costs equal
    assert out["k"].tolist() == [3, 1, 1]              # the arg min is re-evaluated: neuron 0 both times
    w[0, 2] = 2.0                                      # neuron 0's second step now costs more
    assert calib.greedy_bias(w, s, 3 + 2, 1)["k"].tolist() == [2, 2, 1]


def test_score_ties_count_literally():
    """tau = s_(k) drops every sample with s <= tau, also those tied with it beyond position k."""
    s = np.array([[0.0, 1.0, 1.0, 1.0, 2.0]], dtype=np.float32)
    w = np.array([[1.0, 1.0, 1.0, 1.0, 1.0]], dtype=np.float32)
    out = calib.greedy_bias(w, s, 2, 1)
    assert out["k"].tolist() == [2] and out["count"] == 4


def test_required_drops():
    assert calib.required_drops(0.5, 2, 6) == 6
    assert calib.required_drops(0.75, 2, 6) == 9
    assert calib.required_drops(0.8, 2, 6) == 10
    assert calib.required_drops(0.0, 5, 5) == 0 and calib.required_drops(1.0, 5, 5) == 25


def test_kendall_against_scipy_and_closed_forms():
    rng = np.random.default_rng(0)
    D, T, eta = 5, 96, 4
    M = T // eta
    s = np.tile(np.arange(T, dtype=np.float32), (D, 1))                      # already sorted
    w = rng.uniform(0, 1, (D, T)).astype(np.float32)
    w[0] = np.arange(T)                                                       # increasing group sums
    w[1] = np.arange(T)[::-1]                                                 # decreasing
    tk = calib.kendall_tau(w, s, eta)
    assert tk[0] == 1.0 and tk[1] == 0.5
    for i in range(2, D):
        S = w[i].astype(np.float64).reshape(M, eta).sum(axis=1)
        tau_b = scipy.stats.kendalltau(np.arange(M), S).statistic            # no ties: (conc - disc) / pairs
        kd = (1.0 - tau_b) / 2.0 * (M * (M - 1) / 2.0)
        assert abs(tk[i] - (1.0 - kd / (M * (M - 1)))) < 1e-12
    assert np.all(calib.kendall_tau(w, s, T) == 1.0)                          # a single group


# ---------------------------------------------------- weights and scores -----
def test_damage_weight_is_the_squared_norm_of_the_dropped_contribution(oracle):
    """App. A, origin of the weight: dropping hidden coordinate i removes z_i W_down[:, i] from the
    output, whose squared norm is w_i -- through the runtime oracle's dense and sparse FFN."""
    rng = np.random.default_rng(1)
    d, D, T = 16, 24, 5
    Wg, Wu, Wd = (rng.standard_normal((D, d)).astype(np.float32) for _ in range(3))
    X = rng.standard_normal((T, d)).astype(np.float32)
    w = calib.damage_weights(Wg, Wu, Wd, X)
    assert w.shape == (D, T) and np.all(w >= 0)
    y_full = oracle.dense_ffn(Wg, Wu, Wd, X)
    for i in (0, 5, 23):
        lst = np.array([j for j in range(D) if j != i], dtype=np.int32)
        y_drop = oracle.sparse_ffn(Wg, Wu, Wd, X, lst)
        gate = X.astype(np.float64) @ Wg[i].astype(np.float64)
        # on tokens where neuron i is inactive the sparse path over "all but i" equals dense; otherwise it differs by v_i
        diff2 = np.sum((y_full - y_drop) ** 2, axis=1)
        assert np.allclose(diff2, w[i], rtol=1e-9, atol=1e-12)
        assert np.all((w[i] == 0) == (gate <= 0))


def test_proxy_scores_are_the_runtime_predictor_without_bias(oracle):
    rng = np.random.default_rng(2)
    d, D, r, T = 12, 20, 4, 7
    A = rng.standard_normal((D, r)).astype(np.float32)
    B = rng.standard_normal((r, d)).astype(np.float32)
    X = rng.standard_normal((T, d)).astype(np.float32)
    s = calib.proxy_scores(A, B, X)
    s_rt = oracle.predict(np.ascontiguousarray(B.T), A, np.zeros(D, np.float32), X)     # P = B^T, Q = A
    assert np.allclose(s.T, s_rt, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- Alg. 1 -----
def _correlated_tokens(rng, T, d):
    L = rng.standard_normal((d, d)) * (0.9 ** np.arange(d))[None, :]          # strongly anisotropic covariance
    return rng.standard_normal((T, d)) @ L.T


def test_whitened_factors_closed_forms():
    rng = np.random.default_rng(4)
    d, D, T = 24, 40, 200
    W = rng.standard_normal((D, d))
    X = _correlated_tokens(rng, T, d)
    S = np.linalg.cholesky(X.T @ X)
    Z = np.linalg.solve(S, X.T)                                               # S^-1 X: orthonormal rows
    assert np.allclose(Z @ Z.T, np.eye(d), atol=1e-8)
    sig = np.linalg.svd(W @ S, compute_uv=False)
    A, B = calib.whitened_factors(W, X, d)
    assert A.shape == (D, d) and B.shape == (d, d)
    assert np.allclose(A @ B, W, atol=1e-8)                                   # full rank: exact
    for r in (1, 4, 12):
        A, B = calib.whitened_factors(W, X, r)
        assert A.shape == (D, r) and B.shape == (r, d)
        err = np.linalg.norm((W - A @ B) @ X.T)
        assert abs(err - np.sqrt(np.sum(sig[r:] ** 2))) < 1e-7 * sig[0]       # = tail of the whitened spectrum
        # optimal among rank-r products on this data: beats the plain truncated SVD of W and perturbations
        U, sv, Vt = np.linalg.svd(W, full_matrices=False)
        plain = (U[:, :r] * sv[:r]) @ Vt[:r]
        assert err < np.linalg.norm((W - plain) @ X.T)
        for _ in range(3):
            A2, B2 = A + 1e-3 * rng.standard_normal(A.shape), B + 1e-3 * rng.standard_normal(B.shape)
            assert err <= np.linalg.norm((W - A2 @ B2) @ X.T)


def test_whitening_with_isotropic_data_is_the_plain_truncation():
    rng = np.random.default_rng(5)
    d, D, r = 10, 14, 3
    W = rng.standard_normal((D, d))
    Qm, _ = np.linalg.qr(rng.standard_normal((50, d)))                        # X^T X = 4 I
    A, B = calib.whitened_factors(W, 2.0 * Qm, r)
    U, sv, Vt = np.linalg.svd(W, full_matrices=False)
    assert np.allclose(A @ B, (U[:, :r] * sv[:r]) @ Vt[:r], atol=1e-10)
