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
