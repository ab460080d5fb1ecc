"""CPU pins of the oracle: everything here fixes the oracle against something
other than itself - library routines (numpy matmul / flatnonzero), a
hand-worked example, and identities and bounds the paper states."""
import numpy as np
import pytest

from conftest import read_golden
from paper_2603_14110_amd import cost, synth


def _rand_layer(rng, d, D, r, scale=1.0):
    Wg = rng.standard_normal((D, d)).astype(np.float32) * scale
    Wu = rng.standard_normal((D, d)).astype(np.float32)
    WdT = rng.standard_normal((D, d)).astype(np.float32)
    P = rng.standard_normal((d, r)).astype(np.float32)
    Q = rng.standard_normal((D, r)).astype(np.float32)
    b = rng.standard_normal(D).astype(np.float32)
    return Wg, Wu, WdT, P, Q, b


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


# ---- hand-worked example (tests/golden/tiny_worked_example.txt) -------------


def test_hand_worked_example(oracle):
    g = read_golden("tiny_worked_example.txt")
    y, z = oracle.dense_ffn(g["W_gate"], g["W_up"], g["W_downT"], g["x"], return_z=True)
    assert np.array_equal(z[0], g["z"])
    assert np.array_equal(y[0], g["y_dense"])
    s = oracle.predict(g["P"].reshape(2, 1), g["Q"].reshape(3, 1), g["b"], g["x"])
    assert np.array_equal(s[0], g["s"])
    m, idx = oracle.compact(s)
    assert np.array_equal(m, g["mask"].astype(np.uint8))
    assert np.array_equal(idx, g["idx"].astype(np.int32))
    ys = oracle.sparse_ffn(g["W_gate"], g["W_up"], g["W_downT"], g["x"], idx)
    assert np.array_equal(ys[0], g["y_sparse"])


def test_complexity_worked_example():
    g = read_golden("complexity_worked_example.txt")
    d, D, r = int(g["d"]), int(g["D"]), int(g["r"])
    ratio = cost.mults_dense(d, D) / cost.mults_sparse(d, D, r, g["s_pred"], g["s_real"])
    assert round(ratio, 1) == g["ratio_printed"]
    assert abs(ratio - 3.818) < 1e-3


# ---- reductions to library routines (Alg. 4 is matmul / nonzero / selrows) ----


@pytest.mark.parametrize("d,D,r,B", [(8, 16, 4, 1), (24, 40, 8, 3), (64, 192, 16, 8)])
def test_against_numpy_routines(oracle, d, D, r, B):
    rng = np.random.default_rng(d * 1000 + D)
    Wg, Wu, WdT, P, Q, b = _rand_layer(rng, d, D, r)
    x = rng.standard_normal((B, d)).astype(np.float32)
    W64 = [a.astype(np.float64) for a in (Wg, Wu, WdT, P, Q, b, x)]
    Wg6, Wu6, WdT6, P6, Q6, b6, x6 = W64
    # dense: three matmuls
    y_np = (np.maximum(x6 @ Wg6.T, 0.0) * (x6 @ Wu6.T)) @ WdT6
    y = oracle.dense_ffn(Wg, Wu, WdT, x)
    assert _rel(y, y_np) < 1e-13
    yd = oracle.dense_ffn(Wg, Wu, WdT, x, drelu=True)
    yd_np = (np.maximum(x6 @ Wg6.T, 0.0) * np.maximum(x6 @ Wu6.T, 0.0)) @ WdT6
    assert _rel(yd, yd_np) < 1e-13
    # predictor: two matmuls and the bias
    s_np = (x6 @ P6) @ Q6.T + b6
    s = oracle.predict(P, Q, b, x)
    assert np.max(np.abs(s - s_np)) < 1e-12 * max(1.0, np.abs(s_np).max())
    # compaction: flatnonzero of the union mask
    m, idx = oracle.compact(s)
    assert np.array_equal(idx, np.flatnonzero((s > 0).any(axis=0)).astype(np.int32))
    assert np.array_equal(m.astype(bool), (s > 0).any(axis=0))
    # sparse: selrows + matmul over an arbitrary list shared by the batch
    sel = np.sort(rng.choice(D, size=D // 3, replace=False)).astype(np.int32)
    ys_np = (np.maximum(x6 @ Wg6[sel].T, 0.0) * (x6 @ Wu6[sel].T)) @ WdT6[sel]
    ys, h = oracle.sparse_ffn(Wg, Wu, WdT, x, sel, return_h=True)
    assert _rel(ys, ys_np) < 1e-13
    assert h.shape == (B, sel.size)
    assert _rel(h, np.maximum(x6 @ Wg6[sel].T, 0.0) * (x6 @ Wu6[sel].T)) < 1e-13


def test_compact_ties_nan_and_extremes(oracle):
    s = np.array([[0.0, -0.0, np.nan, 1e-300, -1e-300, np.inf, -np.inf, 5.0]])
    m, idx = oracle.compact(s)
    assert m.tolist() == [0, 0, 0, 1, 0, 1, 0, 1]
    assert idx.tolist() == [3, 5, 7]
    m, idx = oracle.compact(-np.ones((2, 64)))
    assert m.sum() == 0 and idx.size == 0
    m, idx = oracle.compact(np.ones((2, 64)))
    assert idx.tolist() == list(range(64))
    # union: a neuron is on if any token switches it on
    s = -np.ones((3, 6))
    s[0, 1] = 1
    s[2, 4] = 2
    s[1, 1] = 3
    assert oracle.compact(s)[1].tolist() == [1, 4]


def test_empty_and_full_lists(oracle):
    rng = np.random.default_rng(5)
    Wg, Wu, WdT, *_ = _rand_layer(rng, 16, 32, 4)
    x = rng.standard_normal((2, 16)).astype(np.float32)
    y0 = oracle.sparse_ffn(Wg, Wu, WdT, x, np.zeros(0, np.int32))
    assert np.array_equal(y0, np.zeros((2, 16)))
    yf = oracle.sparse_ffn(Wg, Wu, WdT, x, np.arange(32, dtype=np.int32))
    assert _rel(yf, oracle.dense_ffn(Wg, Wu, WdT, x)) < 1e-13


# ---- invariants the paper fixes ------------------------------------------------


def test_true_sign_mask_gives_dense_output(oracle):
    """Sec. 3: selecting the rows with positive gate is algebraically the dense FFN."""
    rng = np.random.default_rng(11)
    d, D = 48, 160
    Wg, Wu, WdT, *_ = _rand_layer(rng, d, D, 4)
    x = rng.standard_normal((4, d)).astype(np.float32)
    y_dense = oracle.dense_ffn(Wg, Wu, WdT, x)
    gate = x.astype(np.float64) @ Wg.astype(np.float64).T
    for t in range(4):
        idx = np.flatnonzero(gate[t] > 0).astype(np.int32)
        assert 0 < idx.size < D
        ys = oracle.sparse_ffn(Wg, Wu, WdT, x[t], idx)
        assert _rel(ys[0], y_dense[t]) < 1e-12
        # dropping one truly active neuron must change the output
        ys2 = oracle.sparse_ffn(Wg, Wu, WdT, x[t], idx[1:])
        assert _rel(ys2[0], y_dense[t]) > 1e-6
    # union of the tokens' true masks: every token still gets its dense output
    uni = np.flatnonzero((gate > 0).any(axis=0)).astype(np.int32)
    assert _rel(oracle.sparse_ffn(Wg, Wu, WdT, x, uni), y_dense) < 1e-12


def test_full_rank_zero_bias_mask_is_gate_sign(oracle):
    """Cor. A.7: at rank r = d the truncated SVD is exact (sigma_{r+1} = 0), so with
    b = 0 the predictor mask is the sign pattern of the gate pre-activation."""
    rng = np.random.default_rng(12)
    d, D = 32, 96
    Wg = rng.standard_normal((D, d))
    P, Q, sig = synth.truncated_svd_factors(Wg, d)
    assert np.allclose(Q @ P.T, Wg, atol=1e-9)
    x = rng.standard_normal((8, d)).astype(np.float32)
    s = oracle.predict(P, Q, np.zeros(D, np.float32), x)          # factors rounded to fp32
    gate = x.astype(np.float64) @ Wg.T
    firm = np.abs(gate) > 1e-4 * np.abs(gate).max(axis=1, keepdims=True)
    assert firm.mean() > 0.99
    assert np.array_equal((s > 0)[firm], (gate > 0)[firm])
    for t in range(8):
        m, idx = oracle.compact(s[t])
        keep = firm[t]
        assert np.array_equal(m.astype(bool)[keep], (gate[t] > 0)[keep])


def _gating_terms(oracle, rng, d, D, r, b):
    W = rng.standard_normal((D, d))
    P, Q, sig = synth.truncated_svd_factors(W, r)
    W32, P32, Q32 = W.astype(np.float32), P.astype(np.float32), Q.astype(np.float32)
    x = rng.standard_normal(d).astype(np.float32)
    s = oracle.predict(P32, Q32, b, x)[0]
    m, idx = oracle.compact(s)
    # A(x) = ReLU(W x) from the dense oracle's gate branch: W_up = rows of ones/d trick is
    # avoided; use z with W_up chosen so that W_up x = 1 for every neuron.
    Wu = np.tile((x / np.dot(x, x)).astype(np.float64), (D, 1))
    _, z = oracle.dense_ffn(W32, Wu.astype(np.float32), np.zeros((D, d), np.float32), x, return_z=True)
    up = Wu.astype(np.float32).astype(np.float64) @ x.astype(np.float64)
    A = z[0] / up                                     # ReLU(W x), exact to rounding
    Wr = Q32.astype(np.float64) @ P32.astype(np.float64).T
    return W32.astype(np.float64), Wr, x.astype(np.float64), s, m.astype(bool), A, sig


def test_exact_gating_error_and_bounds(oracle):
    """App. A: Prop. A.1 (exact error), Lemma A.3 (shifted residual bound),
    Cor. A.7 (truncated-SVD bound) - these fail if the bias enters with the wrong
    sign, the inequality is not strict the right way, or P/Q are transposed."""
    rng = np.random.default_rng(13)
    d, D, r = 24, 80, 6
    for case in range(6):
        if case % 3 == 0:
            b = -np.abs(rng.standard_normal(D)).astype(np.float32) - 0.01      # b < 0
        elif case % 3 == 1:
            b = np.abs(rng.standard_normal(D)).astype(np.float32)              # b >= 0
        else:
            b = rng.standard_normal(D).astype(np.float32)
        W, Wr, x, s, m, A, sig = _gating_terms(oracle, rng, d, D, r, b)
        gate = W @ x
        assert np.allclose(A, np.maximum(gate, 0.0), rtol=1e-9, atol=1e-9)
        err = np.linalg.norm(A - A * m)
        # Prop. A.1: ||A - B_b||^2 = sum (Wx)_+^2 * 1[(W_r x + b) <= 0]
        sr = Wr @ x + b.astype(np.float64)
        assert np.allclose(s, sr, atol=1e-9)
        assert abs(err**2 - np.sum(np.maximum(gate, 0.0) ** 2 * (sr <= 0))) < 1e-9
        # Lemma A.3
        res = (W - Wr) @ x
        bound = np.linalg.norm(np.maximum(res - b, 0.0))
        assert err <= bound + 1e-9 <= np.linalg.norm(res - b) + 2e-9
        # Cor. A.7 with ||Delta W||_2 = sigma_{r+1} (fp32 rounding of the factors adds ~1e-6)
        nx = np.linalg.norm(x)
        if case % 3 == 0:
            assert err / nx <= sig[r] + np.linalg.norm(b) / nx + 1e-4
        elif case % 3 == 1:
            assert err / nx <= np.max(np.maximum(sig[r] - b / nx, 0.0)) + 1e-4
    # a large positive bias keeps every neuron (error 0); a large negative one drops all
    b = np.full(D, 1e4, np.float32)
    W, Wr, x, s, m, A, sig = _gating_terms(oracle, rng, d, D, r, b)
    assert m.all()
    W, Wr, x, s, m, A, sig = _gating_terms(oracle, rng, d, D, r, -b)
    assert not m.any()


def test_monotone_in_bias(oracle):
    """Prop. A.2: lowering the bias can only shrink the mask and grow the error."""
    rng = np.random.default_rng(14)
    d, D, r = 16, 64, 4
    Wg, Wu, WdT, P, Q, b = _rand_layer(rng, d, D, r)
    x = rng.standard_normal(d).astype(np.float32)
    gate = np.maximum(x.astype(np.float64) @ Wg.astype(np.float64).T, 0.0)
    prev_mask, prev_err = None, None
    for c in [0.0, 0.3, 1.0, 3.0, 10.0]:
        m, _ = oracle.compact(oracle.predict(P, Q, b - np.float32(c), x))
        m = m.astype(bool)
        err = np.linalg.norm(gate * ~m)
        if prev_mask is not None:
            assert not (m & ~prev_mask).any()
            assert err >= prev_err - 1e-12
        prev_mask, prev_err = m, err


def test_union_semantics(oracle):
    """A batch shares one list: each token is computed exactly over the union, i.e. its
    own-mask output plus the exact contributions of the neurons other tokens switched on."""
    rng = np.random.default_rng(15)
    d, D, r, B = 32, 128, 8, 4
    Wg, Wu, WdT, P, Q, b = _rand_layer(rng, d, D, r)
    x = rng.standard_normal((B, d)).astype(np.float32)
    s = oracle.predict(P, Q, b, x)
    _, uni = oracle.compact(s)
    y_uni = oracle.sparse_ffn(Wg, Wu, WdT, x, uni)
    _, z = oracle.dense_ffn(Wg, Wu, WdT, x, return_z=True)
    for t in range(B):
        _, own = oracle.compact(s[t])
        assert set(own.tolist()) <= set(uni.tolist())
        y_own = oracle.sparse_ffn(Wg, Wu, WdT, x[t], own)[0]
        extra = np.setdiff1d(uni, own)
        corr = z[t, extra] @ WdT.astype(np.float64)[extra]
        assert _rel(y_uni[t], y_own + corr) < 1e-12
        # B = 1 through the batch path is the single-token path, bit for bit
        assert np.array_equal(oracle.sparse_ffn(Wg, Wu, WdT, x[t:t + 1], own)[0], y_own)


def test_homogeneity_and_permutation(oracle):
    """ReGLU is positively homogeneous of degree 2 in x; the output does not depend on the
    order of the neurons (permute rows of all three matrices, the bias and Q together)."""
    rng = np.random.default_rng(16)
    d, D, r = 16, 64, 4
    Wg, Wu, WdT, P, Q, b = _rand_layer(rng, d, D, r)
    x = rng.standard_normal(d).astype(np.float32)
    y = oracle.dense_ffn(Wg, Wu, WdT, x)
    assert _rel(oracle.dense_ffn(Wg, Wu, WdT, 2.0 * x), 4.0 * y) < 1e-13
    perm = rng.permutation(D)
    assert _rel(oracle.dense_ffn(Wg[perm], Wu[perm], WdT[perm], x), y) < 1e-12
    s = oracle.predict(P, Q, b, x)
    sp = oracle.predict(P, Q[perm], b[perm], x)
    assert np.allclose(sp[0], s[0][perm], atol=1e-12)
    _, idx = oracle.compact(s)
    _, idxp = oracle.compact(sp)
    assert sorted(perm[idxp].tolist()) == idx.tolist()
    assert _rel(oracle.sparse_ffn(Wg[perm], Wu[perm], WdT[perm], x, idxp),
                oracle.sparse_ffn(Wg, Wu, WdT, x, idx)) < 1e-12


def test_planted_mistakes_are_caught(oracle):
    """The pins above must be able to fail: emulate plausible oracle mistakes in numpy and
    check they disagree with the oracle on the same inputs."""
    rng = np.random.default_rng(17)
    d, D, r = 12, 20, 4
    Wg, Wu, WdT, P, Q, b = _rand_layer(rng, d, D, r)
    x = rng.standard_normal(d).astype(np.float32)
    x6, Wg6, Wu6, WdT6 = (a.astype(np.float64) for a in (x, Wg, Wu, WdT))
    y = oracle.dense_ffn(Wg, Wu, WdT, x)[0]
    wrong_relu_on_up = (x6 @ Wg6.T * np.maximum(x6 @ Wu6.T, 0)) @ WdT6
    wrong_no_relu = ((x6 @ Wg6.T) * (x6 @ Wu6.T)) @ WdT6
    assert _rel(wrong_relu_on_up, y) > 1e-3 and _rel(wrong_no_relu, y) > 1e-3
    s = oracle.predict(P, Q, b, x)[0]
    assert np.abs(((x6 @ P) @ Q.T - b) - s).max() > 1e-3      # bias sign


def test_stack_glue_closed_forms(oracle):
    rng = np.random.default_rng(18)
    d = 64
    x, y = rng.standard_normal(d), rng.standard_normal(d)
    out = oracle.stack_glue(x, y, np.zeros(d), eps=0.0)
    assert abs(np.sqrt(np.mean(out**2)) - 1.0) < 1e-12          # unit RMS
    assert np.allclose(out, (x + y) / np.sqrt(np.mean((x + y) ** 2)), atol=1e-13)
    out2 = oracle.stack_glue(3 * x, 3 * y, np.zeros(d), eps=0.0)
    assert np.allclose(out, out2, atol=1e-13)                    # scale invariance
    sh = rng.standard_normal(d)
    assert np.allclose(oracle.stack_glue(x, y, sh, eps=0.0), out + sh, atol=1e-13)
    v = np.full(d, 2.0)
    assert np.allclose(oracle.stack_glue(v, 0 * v, np.zeros(d), eps=1e-6), 2.0 / np.sqrt(4.0 + 1e-6))
