"""Comparison rules shared by the GPU parity tests and the smoke entry.

Mask / index list: bit-exact, except for neurons whose oracle score lies inside
the band |s| < 1e-4 * max|s| of its token (fp32 vs fp64 rounding may decide
those either way).  For a batch the mask is the union over tokens: a neuron is
firmly on if some token scores >= band, firmly off if every token scores
<= -band (or is NaN), otherwise it is not compared.
y: relative L2 error against the oracle evaluated on the *GPU's* index list,
<= 1e-5 for fp32 storage and <= 1e-2 for bf16 storage.
"""
import numpy as np

BAND = 1e-4
Y_TOL = {"f32": 1e-5, "bf16": 1e-2}


def firm_sets(s_oracle: np.ndarray):
    s = np.atleast_2d(np.asarray(s_oracle, dtype=np.float64))
    band = BAND * np.nanmax(np.abs(s), axis=1, keepdims=True)
    firm_on = (s >= band).any(axis=0)
    firm_off = ((s <= -band) | np.isnan(s)).all(axis=0)
    return firm_on, firm_off


def mask_bits(mask_words: np.ndarray, D: int) -> np.ndarray:
    w = np.ascontiguousarray(mask_words).view(np.uint64)
    bits = ((w[:, None] >> np.arange(64, dtype=np.uint64)[None, :]) & np.uint64(1)).astype(bool)
    return bits.reshape(-1)[:D]


def check_mask_and_idx(s_oracle, mask_words, idx, nnz, D):
    """Returns the GPU's index list (validated) as an int32 array."""
    firm_on, firm_off = firm_sets(s_oracle)
    bits = mask_bits(mask_words, D)
    assert not (firm_on & ~bits).any(), "a firmly active neuron is missing from the mask"
    assert not (firm_off & bits).any(), "a firmly inactive neuron is in the mask"
    nnz = int(nnz)
    lst = np.asarray(idx[:nnz], dtype=np.int64)
    assert np.array_equal(lst, np.flatnonzero(bits)), "index list is not the ascending list of mask bits"
    return lst.astype(np.int32)


def rel_l2(y, y_ref):
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    num = np.linalg.norm(y - y_ref, axis=-1)
    den = np.linalg.norm(y_ref, axis=-1)
    d = y_ref.shape[-1]
    return np.where(den > 0, num / np.where(den > 0, den, 1.0), num / (1e-6 * np.sqrt(d)) * 1.0)


def fp32_forward_bound(f32, X, lst, gamma=4 * 2.0 ** -24):
    """First-order forward error bound (per token, L2) of evaluating the sparse FFN over the
    list `lst` with fp32 products and sums: each dot product g_i, u_i carries an absolute error
    of at most gamma * sum_j |w_ij x_j|, which propagates through h_i = ReLU(g_i) u_i and the
    down projection.  Used only where the list is arbitrary (stress tests): an adversarial
    list can make y the result of cancelling terms, so that a bound relative to |y| alone
    does not exist in fp32."""
    lst = np.asarray(lst, dtype=np.int64)
    X = np.atleast_2d(np.asarray(X, dtype=np.float64))
    if lst.size == 0:
        return np.zeros(X.shape[0])
    Wg, Wu, Wd = (f32[k][lst].astype(np.float64) for k in ("W_gate", "W_up", "W_downT"))
    g, u = X @ Wg.T, X @ Wu.T
    G, U = np.abs(X) @ np.abs(Wg).T, np.abs(X) @ np.abs(Wu).T
    dh = gamma * (G * np.abs(u) + U * np.maximum(g, 0.0))
    h = np.maximum(g, 0.0) * np.abs(u)
    return (dh + gamma * h) @ np.linalg.norm(Wd, axis=1)


def check_y(y_gpu, y_ref, dtype: str, slack=None):
    """Per-token relative L2 error (absolute <= 1e-6*sqrt(d) when the reference is zero).
    `slack` (per token, absolute) is added to the allowance for arbitrary-list stress tests."""
    y_gpu = np.atleast_2d(np.asarray(y_gpu, dtype=np.float64))
    y_ref = np.atleast_2d(np.asarray(y_ref, dtype=np.float64))
    tol = Y_TOL[dtype]
    for t in range(y_ref.shape[0]):
        den = np.linalg.norm(y_ref[t])
        err = np.linalg.norm(y_gpu[t] - y_ref[t])
        extra = 0.0 if slack is None else float(slack[t])
        if den > 0:
            assert err <= tol * den + extra, f"token {t}: relative L2 error {err / den:.3e} > {tol} (slack {extra:.2e})"
        else:
            assert err <= 1e-6 * np.sqrt(y_ref.shape[1]) + extra, f"token {t}: |y| = {err:.3e} but reference is zero"
