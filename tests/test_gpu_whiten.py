"""GPU parity of the offline predictor build with data whitening (Alg. 1, svdp_whiten_factors) against the CPU
oracle (oracle/calib.py: Cholesky factor, LAPACK SVD, triangular solve).  Both take the Cholesky factor the
algorithm prints, so the pair is fixed up to the signs of the singular vectors (and rotations inside clusters of
nearly equal singular values).  What is compared is what Alg. 1 defines - the product A B, the error on the data
||(W - A B) X^T||_F that it minimises, the singular values of the whitened matrix - and, up to sign, the leading
columns of the two factors themselves."""
import numpy as np
import pytest

from paper_2603_14110_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from oracle import calib
    from paper_2603_14110_amd import binding

    assert torch.cuda.is_available(), "these tests need a GPU"
    binding.lib()
    return binding, torch, calib


def _tokens(rng, n, d, decay):
    mix = rng.standard_normal((d, d)) * (decay ** np.arange(d))[None, :]          # anisotropic second moments
    mean = rng.standard_normal(d) * 0.3
    return mean + rng.standard_normal((n, d)) @ mix.T * 0.35


CASES = [  # d, D, T, r, storage, decay of the token spectrum
    (64, 192, 64, 8, "f32", 0.95),            # T = d: the smallest calibration set the method takes
    (128, 448, 400, 16, "bf16", 0.97),
    (256, 1024, 1024, 32, "bf16", 0.97),      # the shape of the end-to-end calibration test
    (256, 640, 300, 256, "f32", 0.98),        # full rank: A B = W
    (512, 1536, 2048, 64, "bf16", 0.99),
]


@pytest.mark.parametrize("d,D,T,r,dt,decay", CASES)
def test_whitened_factors_against_oracle(env, d, D, T, r, dt, decay):
    binding, torch, calib = env
    rng = np.random.default_rng(1000 + d + r)
    W_st = synth.to_storage(rng.standard_normal((D, d)) / np.sqrt(d), dt)
    X_st = synth.to_storage(_tokens(rng, T, d, decay), dt)
    W, X = synth.storage_to_f32(W_st, dt).astype(np.float64), synth.storage_to_f32(X_st, dt).astype(np.float64)
    A, B = calib.whitened_factors(W, X, r)
    P, Q, sigma, sweeps = binding.whiten_factors(binding.to_device(W_st, dt), binding.to_device(X_st, dt), r)
    P, Q = P.cpu().numpy().astype(np.float64), Q.cpu().numpy().astype(np.float64)
    assert P.shape == (d, r) and Q.shape == (D, r) and sweeps[0] == 0 and 1 <= sweeps[1] <= 24, sweeps
    AB, QP = A @ B, Q @ P.T
    # the product the predictor evaluates (fp32 outputs: a few 1e-7 per factor element)
    assert np.linalg.norm(QP - AB) <= 2e-5 * np.linalg.norm(AB)
    # the objective of Alg. 1, against the oracle's optimum
    err_or, err = np.linalg.norm((W - AB) @ X.T), np.linalg.norm((W - QP) @ X.T)
    scale = np.linalg.norm(W @ X.T)
    assert abs(err - err_or) <= 2e-5 * scale, (err, err_or, scale)
    if r == d:
        assert err <= 2e-5 * scale
    # singular values of W S (any factor S of the second moments gives the same ones) = column norms of A
    sv_or = np.linalg.norm(A, axis=0)
    assert np.all(np.abs(sigma - sv_or) <= 1e-5 * sv_or[0]), np.abs(sigma - sv_or).max() / sv_or[0]
    assert np.all(np.diff(sigma) <= 1e-6 * sigma[0])
    # the leading, well separated columns of the factors themselves, up to sign (Q = A, P = B^T)
    for k in range(min(r, 3)):
        if k + 1 < len(sv_or) and sv_or[k] - sv_or[k + 1] < 0.05 * sv_or[k]:
            break
        sgn = np.sign(np.dot(Q[:, k], A[:, k]))
        assert np.linalg.norm(sgn * Q[:, k] - A[:, k]) <= 1e-4 * np.linalg.norm(A[:, k]), k
        assert np.linalg.norm(sgn * P[:, k] - B[k, :]) <= 1e-4 * np.linalg.norm(B[k, :]), k
    # Q's columns are orthogonal with those norms (Q = U_r Sigma_r)
    G = Q.T @ Q
    assert np.linalg.norm(G - np.diag(np.diag(G))) <= 1e-5 * np.linalg.norm(G)


def test_whitening_beats_plain_truncation_on_correlated_tokens(env):
    """Sec. 4.1's claim on data made to show it, with the GPU's factors: at the same rank the data-aware pair
    has the smaller error on the tokens than the plain truncated SVD of the weights."""
    binding, torch, calib = env
    rng = np.random.default_rng(77)
    d, D, T, r = 256, 768, 1024, 24
    W = rng.standard_normal((D, d)) / np.sqrt(d)
    X = _tokens(rng, T, d, 0.98)
    P, Q, _, _ = binding.whiten_factors(torch.from_numpy(W.astype(np.float32)).cuda(),
                                        torch.from_numpy(X.astype(np.float32)).cuda(), r)
    W32, X32 = W.astype(np.float32).astype(np.float64), X.astype(np.float32).astype(np.float64)
    QP = Q.cpu().numpy().astype(np.float64) @ P.cpu().numpy().astype(np.float64).T
    U, sv, Vt = np.linalg.svd(W32, full_matrices=False)
    plain = (U[:, :r] * sv[:r]) @ Vt[:r]
    assert np.linalg.norm((W32 - QP) @ X32.T) < 0.8 * np.linalg.norm((W32 - plain) @ X32.T)


def test_whiten_rejects_what_it_cannot_take(env):
    binding, torch, calib = env
    L = binding.lib()
    a = 0x1000
    INVALID, UNSUPPORTED, WORKSPACE = 1, 2, 3
    assert L.svdp_whiten_workspace_bytes(100, 256, 512, 8) == 0          # d not a multiple of 64
    assert L.svdp_whiten_workspace_bytes(128, 256, 100, 8) == 0          # fewer tokens than dimensions
    assert L.svdp_whiten_workspace_bytes(128, 256, 512, 200) == 0        # rank above d
    n = L.svdp_whiten_workspace_bytes(128, 256, 512, 8)
    assert n > 0 and n % 256 == 0
    assert L.svdp_whiten_factors(None, a, 128, 256, 512, 8, 1, a, a, None, None, a, n, None) == INVALID
    assert L.svdp_whiten_factors(a, a, 100, 256, 512, 8, 1, a, a, None, None, a, n, None) == UNSUPPORTED
    assert L.svdp_whiten_factors(a, a, 128, 256, 512, 8, 1, a, a, None, None, a, 64, None) == WORKSPACE
    # rank-deficient second moments (every token the same): refused by the factorisation
    W = torch.randn(256, 128, device="cuda")
    X = torch.ones(512, 128, device="cuda")
    with pytest.raises(binding.SvdpError, match="unsupported"):
        binding.whiten_factors(W, X, 8)
