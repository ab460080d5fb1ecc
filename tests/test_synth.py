"""CPU checks of the seeded input generator (tiny workload and small variants)."""
import numpy as np
import pytest

from paper_2603_14110_amd import synth


def test_bf16_roundtrip_and_rounding():
    a = np.array([1.0, -2.5, 3.140625, 1e-3, 65504.0, 0.0, -0.0], dtype=np.float32)
    bits = synth.f32_to_bf16_bits(a)
    back = synth.bf16_bits_to_f32(bits)
    assert np.all(np.abs(back - a) <= np.abs(a) * 2.0**-8)
    assert np.array_equal(synth.f32_to_bf16_bits(back), bits)          # idempotent
    # ties to even: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7 -> rounds to 1 (even mantissa)
    assert synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(np.array([1.0 + 2.0**-8], np.float32)))[0] == 1.0
    assert synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(np.array([1.0 + 3 * 2.0**-8], np.float32)))[0] == 1.0 + 2.0**-6
    import torch
    t = torch.randn(4096, dtype=torch.float32)
    ref = t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(synth.f32_to_bf16_bits(t.numpy()), ref)


def test_truncated_svd_matches_lapack():
    rng = np.random.default_rng(0)
    W = rng.standard_normal((96, 40))
    r = 8
    P, Q, sig = synth.truncated_svd_factors(W, r)
    U, S, Vt = np.linalg.svd(W, full_matrices=False)
    assert np.allclose(sig, S[: r + 1], rtol=1e-9)
    Wr = (U[:, :r] * S[:r]) @ Vt[:r]
    assert np.allclose(Q @ P.T, Wr, atol=1e-9)
    # Eckart-Young (Cor. A.7): the spectral norm of the residual is sigma_{r+1}
    assert abs(np.linalg.norm(W - Q @ P.T, 2) - S[r]) < 1e-9
    assert np.allclose(Q.T @ Q, np.eye(r), atol=1e-9)                  # Q = V_r is orthonormal


@pytest.fixture(scope="module")
def tiny():
    return synth.make_layer(synth.workload("tiny"))


def test_tiny_layer_statistics(tiny, oracle):
    L = tiny
    sp = L.spec
    assert L.W_gate.shape == (sp.D, sp.d) and L.P.shape == (sp.d, sp.r) and L.Q.shape == (sp.D, sp.r)
    assert L.b.dtype == np.float32 and L.W_gate.dtype == np.float32
    assert abs(L.extra["cal_true_sparsity"] - sp.sparsity) < 0.005
    # recall on the calibration tokens, evaluated by the oracle (not by the generator's own code)
    Xc = synth.storage_to_f32(synth.make_tokens(sp, L.u, sp.n_cal, stream=1), sp.dtype)
    s = oracle.predict(L.f32("P"), L.f32("Q"), L.b, Xc)
    gate = Xc.astype(np.float64) @ L.f32("W_gate").astype(np.float64).T
    pos = gate > 0
    recall = ((s > 0) & pos).sum() / pos.sum()
    assert recall >= 0.99
    per_neuron_miss = (pos & ~(s > 0)).sum(axis=0)
    assert np.all(per_neuron_miss <= np.floor(0.01 * pos.sum(axis=0) + 1e-9))
    # timed tokens: about 10 % predicted density, token dependent
    X = synth.storage_to_f32(synth.timed_tokens(L, 64), sp.dtype)
    dens = (oracle.predict(L.f32("P"), L.f32("Q"), L.b, X) > 0).mean(axis=1)
    assert 0.03 < dens.mean() < 0.25
    assert not np.array_equal(synth.timed_tokens(L, 4), synth.make_tokens(sp, L.u, 4, stream=1))


def test_generator_is_deterministic():
    sp = synth.workload("tiny", d=64, D=128, r=8, n_cal=64)
    a, b = synth.make_layer(sp), synth.make_layer(sp)
    for k in ("W_gate", "W_up", "W_downT", "P", "Q", "b"):
        assert np.array_equal(getattr(a, k), getattr(b, k))
    c = synth.make_layer(synth.workload("tiny", d=64, D=128, r=8, n_cal=64, seed=7))
    assert not np.array_equal(a.W_gate, c.W_gate)


def test_bf16_layer_storage():
    sp = synth.workload("tiny", d=64, D=128, r=8, n_cal=64, dtype=synth.BF16)
    L = synth.make_layer(sp)
    assert L.W_gate.dtype == np.uint16 and L.P.dtype == np.uint16
    w = L.f32("W_gate")
    assert np.array_equal(synth.f32_to_bf16_bits(w), L.W_gate)
