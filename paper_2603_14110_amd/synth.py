"""Seeded synthetic ReGLU-FFN layers and decode tokens.

This module only *prepares inputs*: weight matrices, the offline low-rank
predictor factors (plain truncated SVD of the gate matrix, i.e. the offline
factorisation of the paper's Sec. 4.1 / Alg. 1 with the whitening matrix set to
the identity), a per-neuron bias, and token vectors.  It is used by the tests,
the smoke entry and the benchmark to feed *both* the CPU oracle and the HIP
library with identical bit patterns.  None of the decode-time path (predictor
scores per token, mask, index list, sparse or dense FFN) is implemented here;
those live only in ``oracle/`` and in ``csrc/``.

The synthetic layers stand in for the ~90 %-sparse ReGLU models the paper
evaluates (hidden/intermediate sizes from the paper's model table, App. D):
their weights and activations are not available, so a low-rank-plus-shift gate
matrix is generated whose pre-activations are negative for a prescribed
fraction of (token, neuron) pairs.

Everything is numpy, float64, and deterministic given ``seed``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np
import scipy.linalg

# ----------------------------------------------------------------------------
# storage dtypes (bit-level helpers, no arithmetic of the method)
# ----------------------------------------------------------------------------

F32 = "f32"
BF16 = "bf16"


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 -> bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact decode of bfloat16 bit patterns into float32."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """float64/float32 array -> storage array (float32, or uint16 bf16 bits)."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == F32:
        return a32
    if dtype == BF16:
        return f32_to_bf16_bits(a32)
    raise ValueError(f"unknown dtype {dtype!r}")


def storage_to_f32(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float32 view of a storage array (what both the oracle and the GPU see)."""
    if dtype == F32:
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == BF16:
        return bf16_bits_to_f32(a)
    raise ValueError(f"unknown dtype {dtype!r}")


# ----------------------------------------------------------------------------
# workload descriptions
# ----------------------------------------------------------------------------


@dataclass(frozen=True)
class LayerSpec:
    """Shape and generator parameters of one synthetic FFN layer."""

    name: str
    d: int                  # hidden size d
    D: int                  # intermediate size D
    r: int                  # predictor rank
    dtype: str              # storage dtype of weights, predictor factors and tokens
    k_dom: int              # dominant rank of the synthetic gate matrix
    sparsity: float         # target fraction of negative gate pre-activations
    n_cal: int              # calibration tokens for alpha and the bias
    recall: float = 0.99    # per-neuron recall kept on the calibration tokens
    seed: int = 0


def workload(name: str, **over) -> LayerSpec:
    """The named single-layer workloads (shapes follow the paper's model table)."""
    table = {
        # tiny fp32 layer: parity config
        "tiny": LayerSpec("tiny", 256, 1024, 32, F32, 16, 0.90, 256, seed=0),
        # LLaMA-2-7B-shaped layer (d=4096, D=11008), rank swept 128/256/512
        "7b": LayerSpec("7b", 4096, 11008, 256, BF16, 64, 0.90, 1024, seed=1000),
        # 13B-shaped layer
        "13b": LayerSpec("13b", 5120, 13824, 320, BF16, 64, 0.92, 1024, seed=2000),
        # Mistral-7B-shaped layer (d=4096, D=14336)
        "mistral": LayerSpec("mistral", 4096, 14336, 256, BF16, 64, 0.90, 1024, seed=3000),
        # SparseQwen2-7B-shaped layer (d=3584, D=18944), the paper's rank for it
        "qwen": LayerSpec("qwen", 3584, 18944, 512, BF16, 64, 0.90, 1024, seed=5000),
    }
    spec = table[name]
    if over:
        spec = LayerSpec(**{**spec.__dict__, **over})
    return spec


@dataclass
class Layer:
    """One generated layer.  Arrays are in *storage* form (float32 or bf16 bits)."""

    spec: LayerSpec
    W_gate: np.ndarray      # [D][d]
    W_up: np.ndarray        # [D][d]
    W_downT: np.ndarray     # [D][d]  (row i = column i of W_down)
    P: np.ndarray           # [d][r]
    Q: np.ndarray           # [D][r]
    b: np.ndarray           # [D] float32
    u: np.ndarray           # [d] float64 unit vector (token mean direction / 2)
    alpha: float
    sigma: np.ndarray       # leading r+1 singular values of the stored W_gate (float64)
    extra: Dict[str, float] = field(default_factory=dict)

    def f32(self, name: str) -> np.ndarray:
        a = getattr(self, name)
        if name == "b":
            return a
        return storage_to_f32(a, self.spec.dtype)


# ----------------------------------------------------------------------------
# generator
# ----------------------------------------------------------------------------


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(stream)])


def make_tokens(spec: LayerSpec, u: np.ndarray, n: int, stream: int) -> np.ndarray:
    """n tokens x = 2u + N(0,1)^d in storage form, from RNG stream ``stream``."""
    g = _rng(spec.seed, stream)
    X = 2.0 * u[None, :] + g.standard_normal((n, spec.d))
    return to_storage(X, spec.dtype)


def truncated_svd_factors(W: np.ndarray, r: int, n_sigma: Optional[int] = None):
    """Rank-r factors of W (D x d) with W ~= Q @ P.T, P = U_r Sigma_r (d x r), Q = V_r (D x r).

    Row-vector convention: W^T = U Sigma V^T, so a token x gives scores (x P) Q^T.
    Computed from the eigen-decomposition of the d x d Gram matrix W^T W, which
    is exact enough in float64 for the leading part of the spectrum and an
    order of magnitude cheaper than a full LAPACK SVD of the D x d matrix.
    Returns (P, Q, sigma[:n_sigma]) with sigma descending.
    """
    D, d = W.shape
    n_sigma = min(d, (r + 1) if n_sigma is None else n_sigma)
    k = max(r, n_sigma)
    G = W.T @ W
    lam, U = scipy.linalg.eigh(G, subset_by_index=[d - k, d - 1])
    lam = lam[::-1]
    U = np.ascontiguousarray(U[:, ::-1])
    sig = np.sqrt(np.maximum(lam, 0.0))
    Ur = U[:, :r]
    P = Ur * sig[None, :r]
    Q = (W @ Ur) / sig[None, :r]
    return P, Q, sig[:n_sigma]


def _solve_alpha(G0: np.ndarray, c: np.ndarray, target: float) -> float:
    """Bisection for alpha with mean[(G0 - alpha*c) < 0] = target."""
    def frac(a):
        return float(np.mean(G0 < a * c[:, None]))
    lo, hi = 0.0, 1.0
    while frac(hi) < target and hi < 1e9:
        hi *= 2.0
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if frac(mid) < target:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def calibrate_bias(S: np.ndarray, G: np.ndarray, recall: float) -> np.ndarray:
    """Per-neuron bias from calibration scores S and true gate values G (both [n_cal][D]).

    For neuron i, up to floor((1-recall) * n_pos_i) of its truly active
    calibration tokens may be missed: the threshold is the next-smallest score
    among the active ones and b_i sits just above its negative, so that
    score + b_i > 0 holds for every kept token.  A neuron that is never active
    on the calibration tokens gets b_i = -max score (it never fires on them).
    """
    n, D = S.shape
    pos = G > 0.0
    n_pos = pos.sum(axis=0)
    miss = np.floor((1.0 - recall) * n_pos + 1e-9).astype(np.int64)
    Spos = np.where(pos, S, np.inf)
    Spos.sort(axis=0)
    rows = np.minimum(miss, n - 1)
    tau = Spos[rows, np.arange(D)]
    never = n_pos == 0
    tau = np.where(never, S.max(axis=0), tau)
    b = (-tau).astype(np.float32)
    # make sure the float32 bias is strictly above -tau for kept neurons
    fix = (~never) & (b.astype(np.float64) <= -tau)
    b[fix] = np.nextafter(b[fix], np.float32(np.inf))
    # and not above -max for never-active ones
    fixn = never & (b.astype(np.float64) > -tau)
    b[fixn] = np.nextafter(b[fixn], np.float32(-np.inf))
    return b


def make_layer(spec: LayerSpec) -> Layer:
    """Generate one layer (weights, predictor factors, bias) from ``spec.seed``."""
    d, D, r, k = spec.d, spec.D, spec.r, spec.k_dom
    g = _rng(spec.seed, 0)
    u = g.standard_normal(d)
    u /= np.linalg.norm(u)
    std_ab = float(k) ** -0.25            # entries of A, B have variance 1/sqrt(k)
    A = g.standard_normal((D, k)) * std_ab
    Bm = g.standard_normal((d, k)) * std_ab
    W0 = 0.8 * (A @ Bm.T)
    W0 += (0.2 / np.sqrt(d)) * g.standard_normal((D, d))
    W_up = to_storage(g.standard_normal((D, d), dtype=np.float32) / np.float32(np.sqrt(d)), spec.dtype)
    W_downT = to_storage(g.standard_normal((D, d), dtype=np.float32) / np.float32(np.sqrt(d)), spec.dtype)

    Xc_st = make_tokens(spec, u, spec.n_cal, stream=1)
    Xc = storage_to_f32(Xc_st, spec.dtype).astype(np.float64)

    G0 = Xc @ W0.T
    c = Xc @ u
    alpha = _solve_alpha(G0, c, spec.sparsity)
    del G0
    W0 -= alpha * u[None, :]              # W_gate = W0 - alpha * 1 u^T
    W_gate_st = to_storage(W0, spec.dtype)
    del W0
    Wg = storage_to_f32(W_gate_st, spec.dtype).astype(np.float64)

    P, Q, sig = truncated_svd_factors(Wg, r)
    P_st = to_storage(P, spec.dtype)
    Q_st = to_storage(Q, spec.dtype)
    Pq = storage_to_f32(P_st, spec.dtype).astype(np.float64)
    Qq = storage_to_f32(Q_st, spec.dtype).astype(np.float64)

    G = Xc @ Wg.T
    S = (Xc @ Pq) @ Qq.T
    b = calibrate_bias(S, G, spec.recall)
    extra = {
        "cal_true_sparsity": float(np.mean(G <= 0.0)),
        "cal_pred_density": float(np.mean(S + b[None, :].astype(np.float64) > 0.0)),
    }
    return Layer(spec, W_gate_st, W_up, W_downT, P_st, Q_st, b, u, float(alpha), sig, extra)


def load_or_make(spec: LayerSpec, cache_dir: Optional[str] = None) -> Layer:
    """make_layer with an on-disk cache (uncompressed .npz keyed by the spec): the
    full-size layers take tens of seconds to generate and are shared by tests and bench."""
    import hashlib
    import os

    cache_dir = cache_dir or os.environ.get("SVDP_CACHE_DIR", "/tmp/svdp_synth_cache")
    key = hashlib.sha1(repr(sorted(spec.__dict__.items())).encode()).hexdigest()[:16]
    path = os.path.join(cache_dir, f"{spec.name}_{key}.npz")
    names = ("W_gate", "W_up", "W_downT", "P", "Q", "b", "u", "sigma")
    if os.path.exists(path):
        try:
            with np.load(path, allow_pickle=False) as z:
                arrs = {k: z[k] for k in names}
                alpha = float(z["alpha"])
                extra = {k[6:]: float(z[k]) for k in z.files if k.startswith("extra_")}
            return Layer(spec, arrs["W_gate"], arrs["W_up"], arrs["W_downT"], arrs["P"], arrs["Q"], arrs["b"],
                         arrs["u"], alpha, arrs["sigma"], extra)
        except Exception:
            pass
    layer = make_layer(spec)
    try:
        os.makedirs(cache_dir, exist_ok=True)
        tmp = path + f".tmp{os.getpid()}.npz"
        np.savez(tmp, alpha=np.float64(layer.alpha), **{k: getattr(layer, k) for k in names},
                 **{"extra_" + k: np.float64(v) for k, v in layer.extra.items()})
        os.replace(tmp, path)
    except OSError:
        pass
    return layer


def timed_tokens(layer: Layer, n: int) -> np.ndarray:
    """The decode tokens used for parity and timing (RNG stream 2, disjoint from calibration)."""
    return make_tokens(layer.spec, layer.u, n, stream=2)
