"""GPU parity: every entry point of libsvdp against the CPU oracle on the same
seeded inputs, element by element (rules in tests/parity.py)."""
import os

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
    binding.lib()          # raises if the HIP library is missing: no fallback
    return binding, torch, oracle


class Case:
    """A generated layer on both sides: float32 views for the oracle, device tensors for the library."""

    def __init__(self, binding, torch, spec, n_tok):
        self.spec = spec
        self.L = synth.load_or_make(spec) if spec.D >= 8192 else synth.make_layer(spec)
        self.f32 = {k: self.L.f32(k) for k in ("W_gate", "W_up", "W_downT", "P", "Q", "b")}
        self.dev = binding.DeviceLayer.from_synth(self.L)
        self.X_st = synth.timed_tokens(self.L, n_tok)
        self.X = synth.storage_to_f32(self.X_st, spec.dtype)
        self.Xd = binding.to_device(self.X_st, spec.dtype)


_cases = {}


def get_case(env, name, n_tok=64, **over):
    binding, torch, _ = env
    key = (name, n_tok, tuple(sorted(over.items())))
    if key not in _cases:
        _cases[key] = Case(binding, torch, synth.workload(name, **over), n_tok)
    return _cases[key]


SMALL = [
    ("tiny", {}),                                                             # d=256 D=1024 r=32 fp32
    ("tiny", dict(dtype="bf16")),
    ("tiny", dict(d=264, D=1088, r=40, dtype="bf16", seed=5)),                # ragged: nothing a power of two
    ("tiny", dict(d=100, D=192, r=12, seed=6, k_dom=8, n_cal=128)),           # fp32, d % 64 != 0
    ("tiny", dict(d=1024, D=2560, r=72, dtype="bf16", seed=7, k_dom=32)),     # several tiles per block
]


def step_check(env, c, B, t0, flags=0):
    """One decode step through svdp_ffn_step, checked completely (mask, list, y) against the oracle."""
    binding, torch, oracle = env
    dev = c.dev.with_flags(flags) if flags else c.dev
    x = c.Xd[t0:t0 + B]
    D = c.spec.D
    s_or = oracle.predict(c.f32["P"], c.f32["Q"], c.f32["b"], c.X[t0:t0 + B])
    mask = torch.zeros(D // 64, dtype=torch.int64, device="cuda")
    idx = torch.full((D,), -1, dtype=torch.int32, device="cuda")
    nnz = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    y = binding.ffn_step(dev, x, mask=mask, idx=idx, nnz=nnz)
    torch.cuda.synchronize()
    lst = parity.check_mask_and_idx(s_or, mask.cpu().numpy(), idx.cpu().numpy(), nnz.item(), D)
    y_ref = oracle.sparse_ffn(c.f32["W_gate"], c.f32["W_up"], c.f32["W_downT"], c.X[t0:t0 + B], lst,
                              drelu=bool(flags & 1))
    parity.check_y(y.cpu().numpy(), y_ref, c.spec.dtype)
    # the step without the optional outputs gives the same y, bit for bit
    y2 = binding.ffn_step(dev, x)
    assert torch.equal(y, y2)
    return lst, y


@pytest.mark.parametrize("name,over", SMALL)
def test_predict_scores(env, name, over):
    binding, torch, oracle = env
    c = get_case(env, name, **over)
    for B in (1, 2, 3, 8):
        s = binding.predict(c.dev, c.Xd[:B]).cpu().numpy().astype(np.float64)
        s_or = oracle.predict(c.f32["P"], c.f32["Q"], c.f32["b"], c.X[:B])
        scale = np.abs(s_or).max(axis=1, keepdims=True)
        assert np.all(np.abs(s - s_or) <= 2e-5 * scale), np.abs(s - s_or).max() / scale.max()


def test_compact_bit_exact(env):
    """Same fp32 scores on both sides -> the decision s > 0 is taken in the same precision: bit-exact."""
    binding, torch, oracle = env
    rng = np.random.default_rng(1)
    for B, D in [(1, 64), (1, 1024), (3, 11008), (8, 14336), (2, 64 * 1030)]:
        s = rng.standard_normal((B, D)).astype(np.float32) - np.float32(0.8 + 0.4 * (B > 2))
        s[0, :8] = [0.0, -0.0, np.nan, np.inf, -np.inf, 1e-45, -1e-45, 1.0]
        mask, idx, nnz = binding.compact(torch.from_numpy(s).cuda())
        m_or, idx_or = oracle.compact(s.astype(np.float64))
        n = int(nnz.item())
        assert n == idx_or.size
        assert np.array_equal(idx.cpu().numpy()[:n], idx_or)
        assert np.all(idx.cpu().numpy()[n:] == -1)                    # the tail is left untouched
        assert np.array_equal(parity.mask_bits(mask.cpu().numpy(), D), m_or.astype(bool))
    for fill in (-1.0, 1.0):                                            # empty and full
        s = torch.full((2, 1024), fill, device="cuda")
        mask, idx, nnz = binding.compact(s)
        assert nnz.item() == (1024 if fill > 0 else 0)
        if fill > 0:
            assert np.array_equal(idx.cpu().numpy(), np.arange(1024))


@pytest.mark.parametrize("name,over", SMALL)
def test_sparse_ffn_arbitrary_lists(env, name, over):
    binding, torch, oracle = env
    c = get_case(env, name, **over)
    D = c.spec.D
    rng = np.random.default_rng(2)
    lists = [np.zeros(0, np.int32), np.array([D - 1], np.int32), np.arange(D, dtype=np.int32),
             np.sort(rng.choice(D, D // 10, replace=False)).astype(np.int32),
             np.sort(rng.choice(D, D // 2 + 3, replace=False)).astype(np.int32),
             rng.permutation(D)[: D // 7].astype(np.int32)]            # unsorted lists are allowed
    for B in (1, 2, 5, 8):
        for lst in lists:
            idx = torch.zeros(D, dtype=torch.int32, device="cuda")
            idx[: lst.size] = torch.from_numpy(lst).cuda()
            nnz = torch.tensor([lst.size], dtype=torch.int32, device="cuda")
            y_ref = oracle.sparse_ffn(c.f32["W_gate"], c.f32["W_up"], c.f32["W_downT"], c.X[:B], lst)
            slack = parity.fp32_forward_bound(c.f32, c.X[:B], lst)
            y = binding.sparse_ffn(c.dev, c.Xd[:B], idx, nnz).cpu().numpy()
            parity.check_y(y, y_ref, c.spec.dtype, slack=slack)
            if lst.size == 0:
                assert not y.any()


@pytest.mark.parametrize("flags", [0, 2, 8])
def test_sparse_ffn_skips_entries_outside_the_layer(env, flags):
    """svdp_sparse_ffn documents that a list entry outside [0, D) is skipped on the device: the result is
    the oracle's over the valid entries, for the vector, sequential-pipeline and matrix-core row kernels."""
    binding, torch, oracle = env
    c = get_case(env, "tiny", d=1024, D=2560, r=72, dtype="bf16", seed=7, k_dom=32)
    D = c.spec.D
    rng = np.random.default_rng(5)
    good = np.sort(rng.choice(D, 600, replace=False)).astype(np.int32)
    lst = good.copy()
    bad_at = rng.choice(lst.size, 40, replace=False)
    lst[bad_at] = rng.choice(np.array([-1, -7, D, D + 1, 2**31 - 1, -2**31], dtype=np.int64), 40).astype(np.int32)
    valid = np.delete(good, bad_at)
    dev = c.dev.with_flags(flags)
    for B in (1, 3, 8):
        idx = torch.from_numpy(np.concatenate([lst, np.zeros(D - lst.size, np.int32)])).cuda()
        nnz = torch.tensor([lst.size], dtype=torch.int32, device="cuda")
        y = binding.sparse_ffn(dev, c.Xd[:B], idx, nnz).cpu().numpy()
        y_ref = oracle.sparse_ffn(c.f32["W_gate"], c.f32["W_up"], c.f32["W_downT"], c.X[:B], valid)
        parity.check_y(y, y_ref, c.spec.dtype, slack=parity.fp32_forward_bound(c.f32, c.X[:B], valid))
    # a list length beyond D is clamped on the device
    idx = torch.arange(D, dtype=torch.int32, device="cuda")
    y = binding.sparse_ffn(dev, c.Xd[:1], idx, torch.tensor([D + 1000], dtype=torch.int32, device="cuda")).cpu().numpy()
    parity.check_y(y, oracle.dense_ffn(c.f32["W_gate"], c.f32["W_up"], c.f32["W_downT"], c.X[:1]), c.spec.dtype)


@pytest.mark.parametrize("name,over", SMALL)
def test_dense_ffn(env, name, over):
    binding, torch, oracle = env
    c = get_case(env, name, **over)
    for B in (1, 4, 7):
        y_ref = oracle.dense_ffn(c.f32["W_gate"], c.f32["W_up"], c.f32["W_downT"], c.X[:B])
        y = binding.dense_ffn(c.dev, c.Xd[:B]).cpu().numpy()
        parity.check_y(y, y_ref, c.spec.dtype)
    yd = binding.dense_ffn(c.dev.with_flags(binding.FLAG_DRELU), c.Xd[:2]).cpu().numpy()
    parity.check_y(yd, oracle.dense_ffn(c.f32["W_gate"], c.f32["W_up"], c.f32["W_downT"], c.X[:2], drelu=True),
                   c.spec.dtype)


@pytest.mark.parametrize("name,over", SMALL)
def test_ffn_step_all_tokens(env, name, over):
    """Config-0 style run: every one of the 64 decode tokens, batch 1."""
    c = get_case(env, name, **over)
    dens = []
    for t in range(64):
        lst, _ = step_check(env, c, 1, t)
        dens.append(lst.size / c.spec.D)
    assert 0.02 < np.mean(dens) < 0.4


@pytest.mark.parametrize("B", [2, 3, 4, 8])
@pytest.mark.parametrize("name,over", SMALL[:3])
def test_ffn_step_union_batches(env, name, over, B):
    c = get_case(env, name, **over)
    for t0 in range(0, 64 - B + 1, 8):
        step_check(env, c, B, t0)


def test_random_shapes(env):
    """Seeded random shapes (ragged d and r, any B, both storage types, plain random weights):
    every entry point against the oracle.  Covers launch-shape arithmetic the named workloads miss."""
    binding, torch, oracle = env
    rng = np.random.default_rng(2024)
    for case in range(24):
        dt = "bf16" if case % 2 else "f32"
        e = 8 if dt == "bf16" else 4
        d = int(rng.integers(1, 160)) * e
        r = int(rng.integers(1, 20)) * e
        D = int(rng.integers(1, 40)) * 64
        B = int(rng.integers(1, 9))
        st = lambda a: synth.to_storage(a, dt)
        Wg, Wu, Wd = (st(rng.standard_normal((D, d)) / np.sqrt(d)) for _ in range(3))
        P, Q = st(rng.standard_normal((d, r)) / np.sqrt(d)), st(rng.standard_normal((D, r)))
        b = (rng.standard_normal(D) * 0.5 - 1.0).astype(np.float32)
        X = st(rng.standard_normal((B, d)))
        f = {k: synth.storage_to_f32(v, dt) for k, v in dict(W_gate=Wg, W_up=Wu, W_downT=Wd, P=P, Q=Q).items()}
        Xf = synth.storage_to_f32(X, dt)
        dev = binding.DeviceLayer(*(binding.to_device(a, dt) for a in (P, Q)), torch.from_numpy(b).cuda(),
                                  *(binding.to_device(a, dt) for a in (Wg, Wu, Wd)))
        Xd = binding.to_device(X, dt)
        s_or = oracle.predict(f["P"], f["Q"], b, Xf)
        s = binding.predict(dev, Xd).cpu().numpy().astype(np.float64)
        assert np.all(np.abs(s - s_or) <= 2e-5 * np.abs(s_or).max(axis=1, keepdims=True)), (case, d, r, D, B, dt)
        mask = torch.zeros(D // 64, dtype=torch.int64, device="cuda")
        idx = torch.full((D,), -1, dtype=torch.int32, device="cuda")
        nnz = torch.zeros(1, dtype=torch.int32, device="cuda")
        y = binding.ffn_step(dev, Xd, mask=mask, idx=idx, nnz=nnz)
        lst = parity.check_mask_and_idx(s_or, mask.cpu().numpy(), idx.cpu().numpy(), nnz.item(), D)
        y_ref = oracle.sparse_ffn(f["W_gate"], f["W_up"], f["W_downT"], Xf, lst)
        parity.check_y(y.cpu().numpy(), y_ref, dt, slack=parity.fp32_forward_bound(f, Xf, lst))
        yd = binding.dense_ffn(dev, Xd).cpu().numpy()
        parity.check_y(yd, oracle.dense_ffn(f["W_gate"], f["W_up"], f["W_downT"], Xf), dt,
                       slack=parity.fp32_forward_bound(f, Xf, np.arange(D)))


def test_step_equals_separate_calls(env):
    binding, torch, _ = env
    c = get_case(env, "tiny")
    for B in (1, 4):
        x = c.Xd[8:8 + B]
        s = binding.predict(c.dev, x)
        mask, idx, nnz = binding.compact(s)
        y_sep = binding.sparse_ffn(c.dev, x, idx, nnz)
        D = c.spec.D
        mask2 = torch.zeros(D // 64, dtype=torch.int64, device="cuda")
        idx2 = torch.full((D,), -1, dtype=torch.int32, device="cuda")
        nnz2 = torch.zeros(1, dtype=torch.int32, device="cuda")
        y = binding.ffn_step(c.dev, x, mask=mask2, idx=idx2, nnz=nnz2)
        assert torch.equal(mask, mask2) and torch.equal(nnz, nnz2)
        n = nnz.item()
        assert torch.equal(idx[:n], idx2[:n])
        assert torch.equal(y, y_sep)


def test_active_rows_from_mask_words(env):
    """svdp_active_rows: the sparse FFN from the step's own mask words gives the step's y bit for bit, for every
    row-kernel family (two-launch vector path, sequential pipeline, matrix cores); the form that enqueues only
    the dominant kernel (used to time it by itself) leaves y alone and does not disturb the next full call."""
    binding, torch, oracle = env
    c = get_case(env, "tiny", d=1024, D=2560, r=72, dtype="bf16", seed=7, k_dom=32)
    for flags in (0, binding.FLAG_REVALIDATE, binding.FLAG_ENGINE_MATRIX):
        dev = c.dev.with_flags(flags)
        for B in (1, 4, 8):
            x = c.Xd[2:2 + B]
            D = c.spec.D
            mask = torch.zeros(D // 64, dtype=torch.int64, device="cuda")
            ws = torch.zeros(binding.workspace_bytes(dev, B), dtype=torch.uint8, device="cuda")
            y = binding.ffn_step(dev, x, ws=ws, mask=mask).clone()
            ws.zero_()
            y2 = torch.full_like(y, 7.0)
            binding.active_rows(dev, x, mask, ws=ws, out=y2)
            assert torch.equal(y2, y)
            y3 = torch.full_like(y, 7.0)
            assert binding.active_rows(dev, x, mask, ws=ws, first_kernel_only=True) is None
            torch.cuda.synchronize()
            assert bool((y3 == 7.0).all())
            binding.active_rows(dev, x, mask, ws=ws, out=y3)
            assert torch.equal(y3, y)


def test_flags_drelu_and_revalidate(env):
    binding, torch, oracle = env
    c = get_case(env, "tiny", dtype="bf16")
    for B in (1, 4):
        step_check(env, c, B, 3, flags=binding.FLAG_DRELU)
        lst, y_plain = step_check(env, c, B, 3)
        lst2, y_rev = step_check(env, c, B, 3, flags=binding.FLAG_REVALIDATE)
        assert np.array_equal(lst, lst2)
        # skipping rows whose gate is <= 0 removes exact zeros from the sum: same values
        assert np.array_equal(y_plain.cpu().numpy(), y_rev.cpu().numpy())


@pytest.mark.parametrize("name,over", SMALL)
def test_sequential_pipeline(env, name, over):
    """SVDP_FLAG_REVALIDATE in the default launch organisation (its own row kernel): every entry point
    against the oracle, lists with many false positives (up to all D rows), and the values of the
    parallel pipeline bit for bit on the vector engine (the dropped terms are exact zeros)."""
    binding, torch, oracle = env
    c = get_case(env, name, **over)
    D = c.spec.D
    VEC = binding.FLAG_ENGINE_VECTOR
    seq = c.dev.with_flags(binding.FLAG_REVALIDATE | VEC)
    seq_d = c.dev.with_flags(binding.FLAG_REVALIDATE | binding.FLAG_DRELU | VEC)
    par = c.dev.with_flags(VEC)          # the parallel pipeline on the same (vector) engine
    rng = np.random.default_rng(11)
    lists = [np.zeros(0, np.int32), np.arange(D, dtype=np.int32), np.arange(1, D, 3, dtype=np.int32),
             np.sort(rng.choice(D, D // 2 + 1, replace=False)).astype(np.int32), rng.permutation(D)[:300].astype(np.int32)]
    for B in (1, 2, 5, 8):
        x = c.Xd[7:7 + B]
        Xf = c.X[7:7 + B]
        for t0 in (0, 16):                       # offsets the union-batch step tests also use
            step_check(env, c, B, t0, flags=binding.FLAG_REVALIDATE | VEC)
            if B <= 4:
                step_check(env, c, B, t0, flags=binding.FLAG_REVALIDATE | binding.FLAG_DRELU | VEC)
        assert torch.equal(binding.ffn_step(seq, x), binding.ffn_step(par, x))
        for lst in lists:
            idx = torch.zeros(D, dtype=torch.int32, device="cuda")
            idx[: lst.size] = torch.from_numpy(lst).cuda()
            nnz = torch.tensor([lst.size], dtype=torch.int32, device="cuda")
            y = binding.sparse_ffn(seq, x, idx, nnz)
            y_ref = oracle.sparse_ffn(c.f32["W_gate"], c.f32["W_up"], c.f32["W_downT"], Xf, lst)
            parity.check_y(y.cpu().numpy(), y_ref, c.spec.dtype, slack=parity.fp32_forward_bound(c.f32, Xf, lst))
            assert torch.equal(y, binding.sparse_ffn(par, x, idx, nnz))
            yd = binding.sparse_ffn(seq_d, x, idx, nnz).cpu().numpy()
            parity.check_y(yd, oracle.sparse_ffn(c.f32["W_gate"], c.f32["W_up"], c.f32["W_downT"], Xf, lst, drelu=True),
                           c.spec.dtype, slack=parity.fp32_forward_bound(c.f32, Xf, lst))
        # the dense entry point with the flag: every row's gate decides for itself (no predictor involved)
        yd = binding.dense_ffn(seq, x)
        parity.check_y(yd.cpu().numpy(), oracle.dense_ffn(c.f32["W_gate"], c.f32["W_up"], c.f32["W_downT"], Xf),
                       c.spec.dtype, slack=parity.fp32_forward_bound(c.f32, Xf, np.arange(D)))
        assert torch.equal(yd, binding.dense_ffn(par, x))


def test_deterministic(env):
    """Fixed summation order (App. C): bitwise identical output run to run."""
    binding, torch, _ = env
    c = get_case(env, "tiny", d=1024, D=2560, r=72, dtype="bf16", seed=7, k_dom=32)
    for B in (1, 8):
        ref = binding.ffn_step(c.dev, c.Xd[:B]).clone()
        refd = binding.dense_ffn(c.dev, c.Xd[:B]).clone()
        for _ in range(20):
            assert torch.equal(binding.ffn_step(c.dev, c.Xd[:B]), ref)
            assert torch.equal(binding.dense_ffn(c.dev, c.Xd[:B]), refd)


def test_degenerate_masks(env):
    """Nothing active (very negative bias) and everything active (very positive bias)."""
    binding, torch, oracle = env
    c = get_case(env, "tiny")
    t = c.dev.tensors
    for fill, expect in ((-1e6, 0), (1e6, c.spec.D)):
        b = torch.full_like(t["b"], fill)
        dev = binding.DeviceLayer(t["P"], t["Q"], b, t["W_gate"], t["W_up"], t["W_downT"])
        nnz = torch.zeros(1, dtype=torch.int32, device="cuda")
        y = binding.ffn_step(dev, c.Xd[:2], nnz=nnz).cpu().numpy()
        assert nnz.item() == expect
        if expect == 0:
            assert not y.any()
        else:
            parity.check_y(y, oracle.dense_ffn(c.f32["W_gate"], c.f32["W_up"], c.f32["W_downT"], c.X[:2]), "f32")


def test_stack_glue(env):
    binding, torch, oracle = env
    rng = np.random.default_rng(3)
    for d, dt in [(256, "f32"), (4096, "bf16"), (264, "bf16")]:
        x_st = synth.to_storage(rng.standard_normal(d), dt)
        y = rng.standard_normal(d).astype(np.float32)
        sh = rng.standard_normal(d).astype(np.float32)
        out = binding.stack_glue(binding.to_device(x_st, dt), torch.from_numpy(y).cuda(), torch.from_numpy(sh).cuda())
        ref = oracle.stack_glue(synth.storage_to_f32(x_st, dt), y, sh)
        got = out.float().cpu().numpy().astype(np.float64)
        tol = 2e-6 if dt == "f32" else 2.0 ** -8
        assert np.all(np.abs(got - ref) <= tol * np.maximum(np.abs(ref), 1.0))


# ---- full-size layers, in the launch configuration the benchmark times ----------------


# (workload, overrides, batch, first tokens of the steps checked)
FULL = [("7b", {}, 1, (0, 8, 16, 24)), ("7b", dict(r=128), 1, (0, 8, 16, 24)), ("7b", dict(r=512), 1, (0, 8, 16, 24)),
        ("13b", {}, 1, (0, 8, 16, 24)),
        ("mistral", {}, 1, (0, 8, 16, 24)), ("mistral", {}, 2, (0, 8, 16, 24)), ("mistral", {}, 4, (0, 8, 16, 24)),
        ("mistral", {}, 8, (0, 8, 16, 24)),
        # batch sizes that leave token slots of the 4- and 8-token kernels idle
        ("mistral", {}, 3, (32,)), ("mistral", {}, 5, (40,)), ("mistral", {}, 6, (48,)), ("mistral", {}, 7, (56,)),
        # the third shape of the paper's model table (App. D): D > 16384, so a lane of the row kernel's mask scan
        # owns more mask words than it keeps in registers; d is not a multiple of 4096 (ragged row batches)
        ("qwen", {}, 1, (0, 8, 16)), ("qwen", {}, 8, (0, 24))]


@pytest.mark.parametrize("name,over,B,offsets", FULL)
def test_full_size_sampled_tokens(env, name, over, B, offsets):
    """Full shapes; a sample of decode steps checked completely (mask, list, y) against the
    oracle, plus the dense baseline on one batch."""
    binding, torch, oracle = env
    c = get_case(env, name, n_tok=64, **over)
    for t0 in offsets:
        step_check(env, c, B, t0)
    y = binding.dense_ffn(c.dev, c.Xd[:B]).cpu().numpy()
    parity.check_y(y, oracle.dense_ffn(c.f32["W_gate"], c.f32["W_up"], c.f32["W_downT"], c.X[:B]), c.spec.dtype)


def test_full_size_fixed_sparsity_lists_qwen_shape(env):
    """The executor-table protocol as `bench.py --table4` runs it on the largest shape (d=3584, D=18944): random
    ascending lists at 50 % and 95 % sparsity through svdp_sparse_ffn, against the oracle."""
    binding, torch, oracle = env
    c = get_case(env, "qwen", n_tok=64)
    D = c.spec.D
    rng = np.random.default_rng(7)
    for sp in (0.50, 0.95):
        n = int(round((1.0 - sp) * D))
        lst = np.sort(rng.choice(D, n, replace=False)).astype(np.int32)
        idx = torch.zeros(D, dtype=torch.int32, device="cuda")
        idx[:n] = torch.from_numpy(lst).cuda()
        nnz = torch.tensor([n], dtype=torch.int32, device="cuda")
        y = binding.sparse_ffn(c.dev, c.Xd[:1], idx, nnz).cpu().numpy()
        y_ref = oracle.sparse_ffn(c.f32["W_gate"], c.f32["W_up"], c.f32["W_downT"], c.X[:1], lst)
        parity.check_y(y, y_ref, c.spec.dtype, slack=parity.fp32_forward_bound(c.f32, c.X[:1], lst))


def test_full_size_sequential_pipeline_weak_predictor(env):
    """7B shape with a rank-32 predictor (over-predicts about 4x), as `bench.py --rank 32 --flags 2` runs it:
    the sequential pipeline against the oracle on the predictor's own list, and bit for bit against the
    parallel pipeline."""
    binding, torch, oracle = env
    c = get_case(env, "7b", n_tok=64, r=32)
    seq = c.dev.with_flags(binding.FLAG_REVALIDATE)
    dens = []
    for B, t0 in ((1, 0), (1, 9), (2, 16), (4, 24)):
        lst, y = step_check(env, c, B, t0, flags=binding.FLAG_REVALIDATE)
        dens.append(lst.size / c.spec.D)
        assert torch.equal(y, binding.ffn_step(c.dev, c.Xd[t0:t0 + B]))
        assert torch.equal(binding.dense_ffn(seq, c.Xd[t0:t0 + B]), binding.dense_ffn(c.dev, c.Xd[t0:t0 + B]))
    assert np.mean(dens) > 0.2          # the weak predictor keeps far more than the ~10 % that are active
