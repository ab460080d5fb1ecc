"""GPU parity of the offline bias calibration (svdp_calib_bias) against the CPU oracle's
priority-queue loop (oracle/calib.py, Alg. 2): pointers, thresholds and step counts bit for bit."""
import numpy as np
import pytest

from conftest import read_golden

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from oracle import calib
    from paper_2603_14110_amd import binding

    assert torch.cuda.is_available(), "these tests need a GPU"
    binding.lib()
    return binding, torch, calib


def _run(env, w, s, eta, need, kendall=False):
    binding, torch, calib = env
    wd = torch.from_numpy(np.ascontiguousarray(w, dtype=np.float32)).cuda()
    sd = torch.from_numpy(np.ascontiguousarray(s, dtype=np.float32)).cuda()
    b, k, steps, kend = binding.calib_bias(wd, sd, eta, need, want_kendall=kendall)
    torch.cuda.synchronize()
    return b.cpu().numpy(), k.cpu().numpy(), int(steps.item()), None if kend is None else kend.cpu().numpy()


def _check(env, w, s, eta, need, kendall=False):
    binding, torch, calib = env
    ref = calib.greedy_bias(w, s, need, eta)
    b, k, steps, kend = _run(env, w, s, eta, need, kendall)
    assert np.array_equal(k, ref["k"]), (eta, need, np.flatnonzero(k != ref["k"])[:8])
    assert np.array_equal(b.view(np.uint32), ref["b"].view(np.uint32))
    assert steps == ref["steps"]
    if kendall:
        assert np.allclose(kend, calib.kendall_tau(w, s, eta), rtol=0, atol=2e-7)
    return ref


def _stats(rng, D, T, corr=0.3, dead=()):
    """Scores and weights with the structure of the real statistics: the weight grows with the true gate,
    which the score tracks up to noise; about half the samples of a neuron have zero weight."""
    s = rng.standard_normal((D, T)).astype(np.float32)
    g = s + corr * rng.standard_normal((D, T)).astype(np.float32)
    w = (np.maximum(g, 0) ** 2 * rng.uniform(0.2, 3.0, (D, 1))).astype(np.float32)
    for i in dead:
        w[i] = 0.0
    return w, s


def test_worked_example(env):
    binding, torch, calib = env
    g = read_golden("calibration_worked_example.txt")
    for tag in ("a", "b"):
        b, k, steps, _ = _run(env, g["w"], g["s"], int(g["eta"]), int(g[f"need_{tag}"]))
        assert k.tolist() == g[f"k_{tag}"].astype(int).tolist()
        assert (-b).tolist() == g[f"tau_{tag}"].tolist()
        assert steps == int(g[f"steps_{tag}"])


@pytest.mark.parametrize("D,T,eta", [(1, 1, 1), (3, 7, 2), (64, 100, 1), (50, 129, 4), (300, 512, 8), (97, 1000, 16),
                                      (40, 2048, 32), (12, 4096, 64), (33, 333, 400)])
def test_against_the_priority_queue_loop(env, D, T, eta):
    binding, torch, calib = env
    rng = np.random.default_rng(D * 7919 + T)
    w, s = _stats(rng, D, T, dead=(0,) if D > 2 else ())
    for sp in (0.0, 0.35, 0.6, 0.9, 0.97, 1.0):
        need = binding.calib_need(sp, D, T)
        assert need == calib.required_drops(sp, D, T)
        ref = _check(env, w, s, eta, need, kendall=(sp == 0.6))
        if sp == 1.0:
            assert ref["k"].tolist() == [T] * D


def test_ties_everywhere(env):
    """Small integers: equal scores (stable order, literal counting of s <= tau), equal costs across and
    within neurons (smallest index first, a cheaper step behind a dearer one), signed zeros."""
    binding, torch, calib = env
    rng = np.random.default_rng(5)
    D, T = 37, 96
    s = rng.integers(-3, 4, (D, T)).astype(np.float32)
    s[s == 0] = np.where(rng.random(np.count_nonzero(s == 0)) < 0.5, -0.0, 0.0)
    w = rng.integers(0, 4, (D, T)).astype(np.float32)
    for eta in (1, 3, 8):
        for need in (0, 500, 1500, 2500, 3300, D * T - 1, D * T):
            _check(env, w, s, eta, need, kendall=(need == 1500))


def test_non_monotone_costs(env):
    """Weights unrelated to the scores: step costs go up and down, so the order is decided by the running
    maximum (a cheap step hidden behind an expensive one follows it immediately)."""
    binding, torch, calib = env
    rng = np.random.default_rng(8)
    D, T = 120, 256
    s = rng.standard_normal((D, T)).astype(np.float32)
    w = rng.exponential(1.0, (D, T)).astype(np.float32) * (rng.random((D, T)) < 0.7)
    for eta in (1, 4, 16):
        for sp in (0.2, 0.5, 0.8, 0.99):
            _check(env, w, s, eta, binding.calib_need(sp, D, T))


def test_validation(env):
    binding, torch, calib = env
    L = binding.lib()
    assert L.svdp_calib_workspace_bytes(10, 4097, 1) == 0
    assert L.svdp_calib_workspace_bytes(0, 16, 1) == 0 and L.svdp_calib_workspace_bytes(4, 16, 0) == 0
    w = torch.zeros(4, 8, device="cuda")
    with pytest.raises(binding.SvdpError):
        binding.calib_bias(w, w.clone(), 0, 3)


# ------------------------------------------------------------ statistics (svdp_calib_stats) -----
def _bf16_layer(env, seed, d, D, r, T):
    binding, torch, calib = env
    from paper_2603_14110_amd import synth

    rng = np.random.default_rng(seed)
    st = lambda a: synth.to_storage(a, "bf16")
    Wg, Wu, Wd = (st(rng.standard_normal((D, d)) / np.sqrt(d)) for _ in range(3))
    P, Q = st(rng.standard_normal((d, r)) / np.sqrt(d)), st(rng.standard_normal((D, r)))
    X = st(rng.standard_normal((T, d)) + 0.5)
    f = {k: synth.storage_to_f32(v, "bf16") for k, v in dict(W_gate=Wg, W_up=Wu, W_downT=Wd, P=P, Q=Q, X=X).items()}
    dev = binding.DeviceLayer(*(binding.to_device(a, "bf16") for a in (P, Q)), torch.zeros(D, device="cuda"),
                              *(binding.to_device(a, "bf16") for a in (Wg, Wu, Wd)))
    return f, dev, binding.to_device(X, "bf16")


STAT_SHAPES = [(64, 128, 32, 50), (264, 640, 40, 130), (1024, 2560, 72, 300), (512, 4160, 256, 257), (72, 64, 8, 1)]


@pytest.mark.parametrize("shape", STAT_SHAPES)
def test_stats_against_the_oracle(env, shape):
    binding, torch, calib = env
    d, D, r, T = shape
    f, dev, Xd = _bf16_layer(env, 100 + d, d, D, r, T)
    w, s = binding.calib_stats(dev, Xd)
    torch.cuda.synchronize()
    w, s = w.cpu().numpy().astype(np.float64), s.cpu().numpy().astype(np.float64)
    assert w.shape == (D, T) and s.shape == (D, T)
    # proxy scores: A = Q, B = P^T; the tolerance of the runtime predictor's scores
    s_or = calib.proxy_scores(f["Q"], f["P"].T, f["X"])
    assert np.all(np.abs(s - s_or) <= 2e-5 * np.abs(s_or).max(axis=0, keepdims=True))
    # damage weights: forward error bound of fp32 accumulation of exact products, carried through z^2 * norm
    w_or = calib.damage_weights(f["W_gate"], f["W_up"], f["W_downT"], f["X"])
    Xa = np.abs(f["X"].astype(np.float64))
    gam = d * 2.0 ** -24 / 4
    eg, eu = gam * (np.abs(f["W_gate"]).astype(np.float64) @ Xa.T), gam * (np.abs(f["W_up"]).astype(np.float64) @ Xa.T)
    g = f["W_gate"].astype(np.float64) @ f["X"].astype(np.float64).T
    u = f["W_up"].astype(np.float64) @ f["X"].astype(np.float64).T
    cn = np.sum(f["W_downT"].astype(np.float64) ** 2, axis=1)[:, None]
    z = np.maximum(g, 0) * u
    dz = eg * np.abs(u) + eu * np.maximum(g, 0) + eg * eu
    bound = cn * (2 * np.abs(z) * dz + dz * dz) * 1.01 + 1e-5 * w_or
    assert np.all(np.abs(w - w_or) <= bound), float(np.max(np.abs(w - w_or) - bound))
    assert np.all(w >= 0) and np.all((w == 0) | (g > -eg))


def test_statistics_then_calibration_end_to_end(env):
    """The two GPU calls chained, against the oracle's pipeline on its own fp64 statistics: the pointers may
    differ where costs agree to rounding, the achieved sparsity and the loss may not."""
    binding, torch, calib = env
    d, D, r, T, eta = 256, 1024, 32, 512, 8
    f, dev, Xd = _bf16_layer(env, 9, d, D, r, T)
    w, s = binding.calib_stats(dev, Xd)
    need = binding.calib_need(0.85, D, T)
    b, k, steps, _ = binding.calib_bias(w, s, eta, need)
    torch.cuda.synchronize()
    w_or = calib.damage_weights(f["W_gate"], f["W_up"], f["W_downT"], f["X"])
    s_or = calib.proxy_scores(f["Q"], f["P"].T, f["X"])
    ref = calib.greedy_bias(w_or, s_or, need, eta)
    tau = -b.cpu().numpy()
    got_cnt = int(np.sum(s_or.astype(np.float32) <= tau[:, None]))
    assert abs(got_cnt - ref["count"]) <= 2e-3 * D * T
    l_gpu, l_ref = calib.calibration_loss(w_or, s_or.astype(np.float32), tau), calib.calibration_loss(
        w_or, s_or.astype(np.float32), ref["tau"])
    assert abs(l_gpu - l_ref) <= 1e-2 * l_ref
    assert np.mean(k.cpu().numpy() == ref["k"]) > 0.9
    # and exactly the oracle's loop on the GPU's own statistics
    ref2 = calib.greedy_bias(w.cpu().numpy(), s.cpu().numpy(), need, eta)
    assert np.array_equal(k.cpu().numpy(), ref2["k"]) and steps.item() == ref2["steps"]


def test_stats_reject_fp32_layers(env):
    binding, torch, calib = env
    from paper_2603_14110_amd import synth

    L = synth.make_layer(synth.workload("tiny"))
    dev = binding.DeviceLayer.from_synth(L)
    with pytest.raises(binding.SvdpError):
        binding.calib_stats(dev, binding.to_device(synth.timed_tokens(L, 4), "f32"))


def test_full_size_layer_as_benchmarked(env):
    """The 7B-shaped layer with the calibration set bench.py --calibrate uses (2048 tokens, eta = 16,
    sparsity level 0.9): statistics on sampled neurons against the oracle, then pointers, bias and
    step count of the whole layer against the priority-queue loop on the GPU's statistics."""
    binding, torch, calib = env
    from paper_2603_14110_amd import synth

    L = synth.load_or_make(synth.workload("7b"))
    sp = L.spec
    dev = binding.DeviceLayer.from_synth(L)
    T, eta = 2048, 16
    Xc = synth.make_tokens(sp, L.u, T, 1)
    w, s = binding.calib_stats(dev, binding.to_device(Xc, sp.dtype))
    need = binding.calib_need(0.9, sp.D, T)
    b, k, steps, kend = binding.calib_bias(w, s, eta, need, want_kendall=True)
    torch.cuda.synchronize()
    wh, sh = w.cpu().numpy(), s.cpu().numpy()
    # sampled neurons: first, last, tile borders of the contraction kernel, random ones
    rng = np.random.default_rng(0)
    rows = np.unique(np.concatenate([[0, 127, 128, sp.D - 129, sp.D - 1], rng.choice(sp.D, 40, replace=False)]))
    Xf = synth.storage_to_f32(Xc, sp.dtype)
    f = {n: L.f32(n)[rows] for n in ("W_gate", "W_up", "W_downT", "Q")}
    s_or = calib.proxy_scores(f["Q"], L.f32("P").T, Xf)
    smax = np.abs(sh).max(axis=0, keepdims=True)                     # per token, over all neurons
    assert np.all(np.abs(sh[rows] - s_or) <= 2e-5 * smax)
    w_or = calib.damage_weights(f["W_gate"], f["W_up"], f["W_downT"], Xf)
    X64, Xa = Xf.astype(np.float64), np.abs(Xf.astype(np.float64))
    gam = sp.d * 2.0 ** -24 / 4
    g, u = f["W_gate"].astype(np.float64) @ X64.T, f["W_up"].astype(np.float64) @ X64.T
    eg, eu = gam * (np.abs(f["W_gate"]).astype(np.float64) @ Xa.T), gam * (np.abs(f["W_up"]).astype(np.float64) @ Xa.T)
    cn = np.sum(f["W_downT"].astype(np.float64) ** 2, axis=1)[:, None]
    dz = eg * np.abs(u) + eu * np.maximum(g, 0) + eg * eu
    bound = cn * (2 * np.abs(np.maximum(g, 0) * u) * dz + dz * dz) * 1.01 + 1e-5 * w_or
    assert np.all(np.abs(wh[rows] - w_or) <= bound)
    # the whole layer's calibration against the sequential loop on the same statistics
    ref = calib.greedy_bias(wh, sh, need, eta)
    assert np.array_equal(k.cpu().numpy(), ref["k"])
    assert np.array_equal(b.cpu().numpy().view(np.uint32), ref["b"].view(np.uint32))
    assert steps.item() == ref["steps"] and ref["count"] >= need
    assert np.allclose(kend.cpu().numpy()[rows], calib.kendall_tau(wh[rows], sh[rows], eta), rtol=0, atol=2e-7)


def test_offline_build_then_decode(env, oracle):
    """The method end to end on one small layer, every stage on the GPU: factors from the whitened factorisation
    (Alg. 1, svdp_whiten_factors, on correlated calibration tokens), bias from the greedy calibration (Alg. 2),
    then the decode step on held-out tokens.  Checks what the construction promises: the calibration set is dropped at exactly
    the requested level, the predictor built with whitening loses less damage than the plain truncation at the
    same rank and sparsity level, and the sparse output stays close to the dense one."""
    binding, torch, calib = env
    from paper_2603_14110_amd import synth

    rng = np.random.default_rng(21)
    d, D, r, T, eta, level = 256, 1024, 32, 1024, 4, 0.85
    st = lambda a: synth.to_storage(a, "bf16")
    f32 = lambda a: synth.storage_to_f32(a, "bf16")
    Wg, Wu, Wd = (st(rng.standard_normal((D, d)) / np.sqrt(d)) for _ in range(3))
    mix = rng.standard_normal((d, d)) * (0.97 ** np.arange(d))[None, :]            # anisotropic token covariance
    mean = rng.standard_normal(d) * 0.3
    tokens = lambda n: st(mean + rng.standard_normal((n, d)) @ mix.T * 0.35)
    Xcal, Xtest = tokens(T), tokens(64)
    lost, dens, outs = {}, {}, {}
    for name in ("whitened", "plain"):
        if name == "whitened":
            Pw, Qw, _, _ = binding.whiten_factors(binding.to_device(Wg, "bf16"), binding.to_device(Xcal, "bf16"), r)
            A, B = Qw.cpu().numpy().astype(np.float64), Pw.cpu().numpy().astype(np.float64).T
        else:
            U, sv, Vt = np.linalg.svd(f32(Wg).astype(np.float64), full_matrices=False)
            A, B = U[:, :r] * sv[:r], Vt[:r]
        P, Q = st(B.T), st(A)                                                      # s = (x P) Q^T = A B x
        zero_b = torch.zeros(D, device="cuda")
        dev = binding.DeviceLayer(binding.to_device(P, "bf16"), binding.to_device(Q, "bf16"), zero_b,
                                  *(binding.to_device(a, "bf16") for a in (Wg, Wu, Wd)))
        w, s = binding.calib_stats(dev, binding.to_device(Xcal, "bf16"))
        need = binding.calib_need(level, D, T)
        b, k, steps, _ = binding.calib_bias(w, s, eta, need)
        torch.cuda.synchronize()
        # exactly the requested level on the calibration set: the last step reached it, one fewer did not
        cnt = int((s + b[:, None] <= 0).sum().item())
        assert need <= cnt < need + eta * 64
        lost[name] = float((w * (s + b[:, None] <= 0)).sum() / w.sum())
        # decode on held-out tokens with the calibrated bias
        layer = binding.DeviceLayer(dev.tensors["P"], dev.tensors["Q"], b, dev.tensors["W_gate"], dev.tensors["W_up"],
                                    dev.tensors["W_downT"])
        Xt = binding.to_device(Xtest, "bf16")
        nnz = torch.zeros(1, dtype=torch.int32, device="cuda")
        ys, ns = [], []
        for t in range(64):
            ys.append(binding.ffn_step(layer, Xt[t], nnz=nnz).clone())
            ns.append(nnz.item())
        y_sparse = torch.cat(ys).cpu().numpy().astype(np.float64)
        y_dense = oracle.dense_ffn(f32(Wg), f32(Wu), f32(Wd), f32(Xtest))
        outs[name] = np.linalg.norm(y_sparse - y_dense) / np.linalg.norm(y_dense)
        dens[name] = float(np.mean(ns)) / D
        # the step's own arithmetic is exact for its list: compare one token with the oracle on that list
        s_or = oracle.predict(f32(P), f32(Q), b.cpu().numpy(), f32(Xtest)[:1])
        lst = np.flatnonzero(s_or[0] > 0).astype(np.int32)
        if abs(lst.size - ns[0]) == 0:
            y_ref = oracle.sparse_ffn(f32(Wg), f32(Wu), f32(Wd), f32(Xtest)[:1], lst)
            assert np.linalg.norm(y_sparse[0] - y_ref[0]) <= 1e-2 * np.linalg.norm(y_ref[0])
    assert all(0.05 < v < 0.30 for v in dens.values()), dens                       # near 1 - level on held-out tokens
    assert lost["whitened"] < lost["plain"], lost                                  # Sec. 4.1: whitening helps on correlated data
    assert outs["whitened"] < outs["plain"] and outs["whitened"] < 0.5, outs
