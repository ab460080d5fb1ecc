"""GPU parity of the kernels on the matrix cores (SVDP_FLAG_ENGINE_MATRIX) against the CPU
oracle: every entry point that runs them, on seeded random layers whose row chunks
span several 16-row tiles with ragged ends, for every batch size and predictor rank."""
import numpy as np
import pytest

import parity
from paper_2603_14110_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env(oracle):
    import torch
    from paper_2603_14110_amd import binding

    assert torch.cuda.is_available(), "these tests need a GPU"
    binding.lib()
    return binding, torch, oracle


class RandomLayer:
    """Plain random bf16 layer (no generator structure): weights ~ N(0, 1/d), a bias that keeps
    about a third of the neurons on."""

    def __init__(self, binding, torch, seed, d, D, r, B):
        rng = np.random.default_rng(seed)
        dt = "bf16"
        st = lambda a: synth.to_storage(a, dt)
        Wg, Wu, Wd = (st(rng.standard_normal((D, d)) / np.sqrt(d)) for _ in range(3))
        P, Q = st(rng.standard_normal((d, r)) / np.sqrt(d)), st(rng.standard_normal((D, r)))
        self.b = (rng.standard_normal(D) * 0.5 - 1.5).astype(np.float32)
        X = st(rng.standard_normal((B, d)))
        self.f = {k: synth.storage_to_f32(v, dt) for k, v in dict(W_gate=Wg, W_up=Wu, W_downT=Wd, P=P, Q=Q).items()}
        self.X = synth.storage_to_f32(X, dt)
        self.dev = binding.DeviceLayer(*(binding.to_device(a, dt) for a in (P, Q)), torch.from_numpy(self.b).cuda(),
                                       *(binding.to_device(a, dt) for a in (Wg, Wu, Wd)))
        self.Xd = binding.to_device(X, dt)
        self.d, self.D, self.B = d, D, B


# (d, D, r, B): d a multiple of 512; D/256 from under one tile to several tiles with a ragged end
SHAPES = [(512, 64, 8, 1), (512, 4160, 16, 8), (1024, 8704, 72, 8), (1536, 12352, 40, 5), (1024, 5184, 24, 4),
          (2048, 4608, 32, 3), (512, 16448, 16, 7), (1024, 2560, 64, 2), (3584, 6400, 48, 6), (512, 10048, 96, 8)]


@pytest.mark.parametrize("shape", SHAPES)
def test_matrix_engine_every_entry_point(env, shape):
    binding, torch, oracle = env
    d, D, r, B = shape
    c = RandomLayer(binding, torch, 77 + D, d, D, r, B)
    f = c.f
    s_or = oracle.predict(f["P"], f["Q"], c.b, c.X)
    results = {}
    MATRIX, VECTOR = binding.FLAG_ENGINE_MATRIX, binding.FLAG_ENGINE_VECTOR
    for engine in (MATRIX, VECTOR):
        dev = c.dev.with_flags(engine)
        # the whole step
        mask = torch.zeros(D // 64, dtype=torch.int64, device="cuda")
        idx = torch.full((D,), -1, dtype=torch.int32, device="cuda")
        nnz = torch.zeros(1, dtype=torch.int32, device="cuda")
        y = binding.ffn_step(dev, c.Xd, mask=mask, idx=idx, nnz=nnz)
        lst = parity.check_mask_and_idx(s_or, mask.cpu().numpy(), idx.cpu().numpy(), nnz.item(), D)
        y_ref = oracle.sparse_ffn(f["W_gate"], f["W_up"], f["W_downT"], c.X, lst)
        parity.check_y(y.cpu().numpy(), y_ref, "bf16", slack=parity.fp32_forward_bound(f, c.X, lst))
        assert torch.equal(y, binding.ffn_step(dev, c.Xd))              # optional outputs change nothing
        # dense baseline
        yd = binding.dense_ffn(dev, c.Xd)
        parity.check_y(yd.cpu().numpy(), oracle.dense_ffn(f["W_gate"], f["W_up"], f["W_downT"], c.X), "bf16",
                       slack=parity.fp32_forward_bound(f, c.X, np.arange(D)))
        # dReLU variant
        dl = c.dev.with_flags(binding.FLAG_DRELU | engine)
        mask2 = torch.zeros(D // 64, dtype=torch.int64, device="cuda")
        idx2 = torch.full((D,), -1, dtype=torch.int32, device="cuda")
        nnz2 = torch.zeros(1, dtype=torch.int32, device="cuda")
        y2 = binding.ffn_step(dl, c.Xd, mask=mask2, idx=idx2, nnz=nnz2)
        lst2 = parity.check_mask_and_idx(s_or, mask2.cpu().numpy(), idx2.cpu().numpy(), nnz2.item(), D)
        parity.check_y(y2.cpu().numpy(),
                       oracle.sparse_ffn(f["W_gate"], f["W_up"], f["W_downT"], c.X, lst2, drelu=True), "bf16",
                       slack=parity.fp32_forward_bound(f, c.X, lst2))
        results[engine] = (lst, y.cpu().numpy(), yd.cpu().numpy())
    # the two engines: same list, y equal to fp32 rounding
    assert np.array_equal(results[MATRIX][0], results[VECTOR][0])
    for k in (1, 2):
        a, b = results[MATRIX][k].astype(np.float64), results[VECTOR][k].astype(np.float64)
        assert np.linalg.norm(a - b) <= 2e-5 * max(np.linalg.norm(b), 1e-30)


@pytest.mark.parametrize("shape", SHAPES[1:4])
def test_matrix_engine_arbitrary_lists(env, shape):
    binding, torch, oracle = env
    d, D, r, B = shape
    c = RandomLayer(binding, torch, 5 + D, d, D, r, 8)
    f = c.f
    rng = np.random.default_rng(D)
    lists = [np.zeros(0, np.int32), np.array([D - 1], np.int32), np.arange(D, dtype=np.int32),
             np.arange(0, D, 17, dtype=np.int32), np.sort(rng.choice(D, D // 2 + 3, replace=False)).astype(np.int32),
             np.sort(rng.choice(D, 255, replace=False)).astype(np.int32),          # fewer rows than blocks
             np.sort(rng.choice(D, 257, replace=False)).astype(np.int32),
             rng.permutation(D)[: D // 7].astype(np.int32)]                        # unsorted lists are allowed
    dev = c.dev.with_flags(binding.FLAG_ENGINE_MATRIX)
    for Bq in (1, 2, 3, 4, 8):
        for lst in lists:
            idx = torch.zeros(D, dtype=torch.int32, device="cuda")
            idx[: lst.size] = torch.from_numpy(lst).cuda()
            nnz = torch.tensor([lst.size], dtype=torch.int32, device="cuda")
            y = binding.sparse_ffn(dev, c.Xd[:Bq], idx, nnz).cpu().numpy()
            y_ref = oracle.sparse_ffn(f["W_gate"], f["W_up"], f["W_downT"], c.X[:Bq], lst)
            parity.check_y(y, y_ref, "bf16", slack=parity.fp32_forward_bound(f, c.X[:Bq], lst))
            if lst.size == 0:
                assert not y.any()


# (d, D, r, B): ranks the score kernel on the matrix cores takes (multiples of 32 up to 512) and two it does not
SCORE_SHAPES = [(256, 1024, 32, 1), (512, 2048, 128, 8), (264, 640, 256, 5), (512, 4096, 320, 3), (128, 832, 512, 8),
                (128, 256, 544, 4), (96, 192, 48, 2), (1024, 3072, 256, 7)]


@pytest.mark.parametrize("shape", SCORE_SHAPES)
def test_matrix_engine_scores(env, shape):
    """svdp_predict and the mask of svdp_ffn_step with the score kernel on the matrix cores."""
    binding, torch, oracle = env
    d, D, r, B = shape
    c = RandomLayer(binding, torch, 31 + r, d, D, r, B)
    f = c.f
    s_or = oracle.predict(f["P"], f["Q"], c.b, c.X)
    dev = c.dev.with_flags(binding.FLAG_ENGINE_MATRIX)
    for Bq in sorted({1, B}):
        s = binding.predict(dev, c.Xd[:Bq]).cpu().numpy().astype(np.float64)
        assert s.shape == (Bq, D)
        assert np.all(np.abs(s - s_or[:Bq]) <= 2e-5 * np.abs(s_or[:Bq]).max(axis=1, keepdims=True))
        mask = torch.zeros(D // 64, dtype=torch.int64, device="cuda")
        idx = torch.full((D,), -1, dtype=torch.int32, device="cuda")
        nnz = torch.zeros(1, dtype=torch.int32, device="cuda")
        y = binding.ffn_step(dev, c.Xd[:Bq], mask=mask, idx=idx, nnz=nnz)
        lst = parity.check_mask_and_idx(s_or[:Bq], mask.cpu().numpy(), idx.cpu().numpy(), nnz.item(), D)
        y_ref = oracle.sparse_ffn(f["W_gate"], f["W_up"], f["W_downT"], c.X[:Bq], lst)
        parity.check_y(y.cpu().numpy(), y_ref, "bf16", slack=parity.fp32_forward_bound(f, c.X[:Bq], lst))
        # svdp_compact on the materialised scores gives the step's list
        m2, i2, n2 = binding.compact(binding.predict(dev, c.Xd[:Bq]))
        assert torch.equal(m2, mask) and n2.item() == nnz.item()
        assert torch.equal(i2[: nnz.item()], idx[: nnz.item()])


def test_engine_selection_and_determinism(env):
    """No engine flag = matrix cores from 5 tokens up (batch capacity 8), vector units below; layers the matrix
    kernel does not take (fp32 storage, d not a multiple of 512, re-validation) run on the vector kernel whatever
    is asked for.  Seen through bit patterns: each engine is deterministic and the two differ in the
    last bits of y."""
    binding, torch, oracle = env
    c = RandomLayer(binding, torch, 11, 1024, 8704, 32, 8)
    MATRIX, VECTOR, AUTO = binding.FLAG_ENGINE_MATRIX, binding.FLAG_ENGINE_VECTOR, 0

    def run(engine, B, dev=None, flags=0):
        return binding.ffn_step((dev or c.dev).with_flags(engine | flags), c.Xd[:B]).clone()

    for B in (1, 2, 3, 4, 5, 8):
        ym, yv, ya = run(MATRIX, B), run(VECTOR, B), run(AUTO, B)
        assert torch.equal(ym, run(MATRIX, B)) and torch.equal(yv, run(VECTOR, B))
        assert not torch.equal(ym, yv)
        assert torch.equal(ya, ym if B >= 5 else yv)
    # re-validation: vector row kernel under every setting (the score kernel still follows the flag,
    # which can only move scores within rounding of zero; the lists agree on this layer)
    assert torch.equal(run(MATRIX, 8, flags=binding.FLAG_REVALIDATE), run(VECTOR, 8, flags=binding.FLAG_REVALIDATE))
    # d = 520: not a multiple of 512
    c2 = RandomLayer(binding, torch, 12, 520, 4160, 16, 8)
    assert torch.equal(binding.ffn_step(c2.dev.with_flags(MATRIX), c2.Xd), binding.ffn_step(c2.dev.with_flags(VECTOR), c2.Xd))


def test_two_host_threads_with_different_engines(env):
    """The library keeps no mode between calls: two host threads, each on its own stream and workspace, one
    asking for the vector units and one for the matrix cores, get the results they get when run alone."""
    import threading

    binding, torch, oracle = env
    c = RandomLayer(binding, torch, 13, 1024, 8704, 32, 8)
    devs = {k: c.dev.with_flags(k) for k in (binding.FLAG_ENGINE_MATRIX, binding.FLAG_ENGINE_VECTOR)}
    alone = {k: binding.ffn_step(d, c.Xd).clone() for k, d in devs.items()}
    torch.cuda.synchronize()
    assert not torch.equal(*alone.values())
    bad = []

    def worker(k):
        try:
            st = torch.cuda.Stream()
            ws = torch.empty(binding.workspace_bytes(devs[k], 8), dtype=torch.uint8, device="cuda")
            out = torch.empty(8, c.d, device="cuda")
            with torch.cuda.stream(st):
                for _ in range(50):
                    binding.ffn_step(devs[k], c.Xd, ws=ws, out=out)
                    st.synchronize()
                    if not torch.equal(out, alone[k]):
                        bad.append(k)
                        return
        except Exception as e:                  # a failure in a thread must fail the test
            bad.append((k, repr(e)))

    threads = [threading.Thread(target=worker, args=(k,)) for k in devs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not bad, bad


def test_matrix_engine_under_graph_replay(env):
    """The matrix-core kernels captured in a HIP graph (as bench.py runs them): every replay, with eager work
    in between, reproduces the eager result bit for bit; so do the sequential-pipeline kernel and calibration-free
    reruns on the same workspace."""
    binding, torch, oracle = env
    c = RandomLayer(binding, torch, 21, 1024, 6144, 64, 8)
    seq = c.dev.with_flags(binding.FLAG_REVALIDATE)
    ws = c.dev.workspace(8)
    xin = torch.zeros_like(c.Xd)
    outs = {k: torch.zeros(8, c.d, device="cuda") for k in ("step", "dense", "seq")}

    def work():
        binding.ffn_step(c.dev, xin, ws=ws, out=outs["step"])
        binding.dense_ffn(c.dev, xin, ws=ws, out=outs["dense"])
        binding.ffn_step(seq, xin, ws=ws, out=outs["seq"])

    variants = [c.Xd, torch.flip(c.Xd, dims=[0]), c.Xd * 0.5]
    eager = []
    for v in variants:
        xin.copy_(v)
        work()
        torch.cuda.synchronize()
        eager.append({k: t.clone() for k, t in outs.items()})
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        work()
        s.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            work()
    for rnd in range(3):
        for v, ref in zip(variants, eager):
            xin.copy_(v)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for k in outs:
                assert torch.equal(outs[k], ref[k]), (rnd, k)
            binding.ffn_step(c.dev, c.Xd[:3])                       # eager work between replays
