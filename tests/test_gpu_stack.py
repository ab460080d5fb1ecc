"""GPU parity of a small stack of layers with the benchmark's glue, eager and as a replayed HIP graph."""
import numpy as np
import pytest

import parity
from paper_2603_14110_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def small_stack(oracle):
    import torch
    from paper_2603_14110_amd import binding, stack

    assert torch.cuda.is_available()
    binding.lib()
    specs = stack.stack_specs(4, base="tiny", seed0=7000, d=512, D=1536, r=48, dtype="bf16", k_dom=24, n_cal=256)
    layers = [synth.make_layer(sp) for sp in specs]
    return layers, stack.FFNStack.from_synth(layers), binding, torch


def oracle_stack(oracle, layers, x0_f32, teacher=None):
    """Oracle stack in fp64, activations re-rounded to the storage dtype between layers.
    Returns the per-layer inputs (as stored), scores, lists and outputs."""
    dt = layers[0].spec.dtype
    xs, out = [np.asarray(x0_f32, dtype=np.float32)], []
    for l, L in enumerate(layers):
        f = {k: L.f32(k) for k in ("W_gate", "W_up", "W_downT", "P", "Q", "b")}
        s, m, idx, y = oracle.ffn_step(f, xs[l])
        shift = 2.0 * layers[l + 1].u if l + 1 < len(layers) else np.zeros(L.spec.d)
        xn = oracle.stack_glue(xs[l].astype(np.float64), y[0], shift)
        xs.append(synth.storage_to_f32(synth.to_storage(xn, dt), dt))
        out.append((s, idx, y))
    return xs, out


def test_stack_teacher_forced_and_free_running(small_stack, oracle):
    layers, st, binding, torch = small_stack
    L0 = layers[0]
    X = synth.storage_to_f32(synth.timed_tokens(L0, 6), "bf16")
    Xd = binding.to_device(synth.timed_tokens(L0, 6), "bf16")
    for t in range(6):
        xs, out = oracle_stack(oracle, layers, X[t])
        # teacher-forced: the oracle's input of layer l goes into GPU layer l
        for l, L in enumerate(layers):
            D = L.spec.D
            xin = binding.to_device(synth.to_storage(xs[l], "bf16"), "bf16")
            mask = torch.zeros(D // 64, dtype=torch.int64, device="cuda")
            idx = torch.full((D,), -1, dtype=torch.int32, device="cuda")
            nnz = torch.zeros(1, dtype=torch.int32, device="cuda")
            y = binding.ffn_step(st.layers[l], xin, mask=mask, idx=idx, nnz=nnz)
            lst = parity.check_mask_and_idx(out[l][0], mask.cpu().numpy(), idx.cpu().numpy(), nnz.item(), D)
            f = {k: L.f32(k) for k in ("W_gate", "W_up", "W_downT")}
            y_ref = oracle.sparse_ffn(f["W_gate"], f["W_up"], f["W_downT"], xs[l], lst)
            parity.check_y(y.cpu().numpy(), y_ref, "bf16")
            xn = binding.stack_glue(xin, y, st.shifts[l]).float().cpu().numpy()
            ref = xs[l + 1]
            assert np.all(np.abs(xn - ref) <= 2.0 ** -7 * np.maximum(np.abs(ref), 1.0))
        # free-running: the whole stack on the GPU; compared loosely (a borderline neuron may flip)
        got = st.step(Xd[t]).float().cpu().numpy()
        assert np.linalg.norm(got - xs[-1]) <= 0.05 * np.linalg.norm(xs[-1])


def test_stack_graph_replay_matches_eager(small_stack):
    """The whole step captured in one HIP graph; every replay (with eager work in between)
    must reproduce the eager result bit for bit."""
    layers, st, binding, torch = small_stack
    Xd = binding.to_device(synth.timed_tokens(layers[0], 5), "bf16")
    eager = [st.step(Xd[t]).clone() for t in range(5)]
    xin = torch.zeros_like(Xd[0])
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        st.step(xin)
        s.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            out = st.step(xin)
    for rnd in range(3):
        for t in range(5):
            xin.copy_(Xd[t])
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager[t]), (rnd, t)
            assert torch.equal(st.step(Xd[t]), eager[t])     # eager work between replays


def test_dense_stack_close_to_sparse(small_stack):
    layers, st, binding, torch = small_stack
    Xd = binding.to_device(synth.timed_tokens(layers[0], 3), "bf16")
    for t in range(3):
        a = st.step(Xd[t]).float().clone()
        b = st.as_dense().step(Xd[t]).float()
        # the predictor keeps ~99 % of the truly active neurons: outputs are close, not equal
        assert torch.linalg.norm(a - b) <= 0.25 * torch.linalg.norm(b)


def test_glue_inside_the_step_gives_the_same_bits(small_stack):
    """svdp_ffn_step_glued: x_out equals svdp_stack_glue's output and y, mask and list equal
    svdp_ffn_step on it, bit for bit, for every batch size; the stack gives the same output with the glue
    fused into the next layer's first kernel or launched on its own."""
    layers, st, binding, torch = small_stack
    L = st.layers[1]
    d, D = L.d, L.D
    g = torch.Generator(device="cuda").manual_seed(3)
    for dt_layer in (L,):
        for B in (1, 2, 3, 8):
            xp = torch.randn(B, d, device="cuda", generator=g).to(torch.bfloat16)
            yp = torch.randn(B, d, device="cuda", generator=g) * 0.7
            shift = torch.randn(d, device="cuda", generator=g)
            x_ref = torch.stack([binding.stack_glue(xp[b], yp[b], shift) for b in range(B)])
            m1, m2 = (torch.zeros(D // 64, dtype=torch.int64, device="cuda") for _ in range(2))
            i1, i2 = (torch.full((D,), -1, dtype=torch.int32, device="cuda") for _ in range(2))
            n1, n2 = (torch.zeros(1, dtype=torch.int32, device="cuda") for _ in range(2))
            y_ref = binding.ffn_step(dt_layer, x_ref, mask=m1, idx=i1, nnz=n1)
            x_out = torch.zeros_like(xp)
            y = binding.ffn_step_glued(dt_layer, xp, yp, shift, x_out, mask=m2, idx=i2, nnz=n2)
            assert torch.equal(x_out, x_ref)
            assert torch.equal(y, y_ref) and torch.equal(m1, m2) and n1.item() == n2.item()
            assert torch.equal(i1[: n1.item()], i2[: n1.item()])
            # y may alias y_prev
            yp2 = yp.clone()
            binding.ffn_step_glued(dt_layer, xp, yp2, shift, x_out, out=yp2)
            assert torch.equal(yp2, y_ref)
    Xd = binding.to_device(synth.timed_tokens(layers[0], 4), "bf16")
    plain = st.with_glue_launches()
    assert st.fused_glue and not plain.fused_glue
    for t in range(4):
        assert torch.equal(st.step(Xd[t]).clone(), plain.step(Xd[t]))


def test_glued_step_fp32(oracle):
    """The fp32 storage path of the fused glue against the oracle's glue and step."""
    import torch
    from paper_2603_14110_amd import binding

    Ls = synth.make_layer(synth.workload("tiny"))
    dev = binding.DeviceLayer.from_synth(Ls)
    rng = np.random.default_rng(4)
    d = Ls.spec.d
    xp, yp, shift = (rng.standard_normal(d).astype(np.float32) for _ in range(3))
    x_out = torch.zeros(1, d, device="cuda")
    y = binding.ffn_step_glued(dev, torch.from_numpy(xp).cuda()[None], torch.from_numpy(yp).cuda()[None],
                               torch.from_numpy(shift).cuda(), x_out)
    x_or = oracle.stack_glue(xp, yp, shift)
    assert np.allclose(x_out.cpu().numpy()[0], x_or, rtol=1e-5, atol=1e-6)
    assert torch.equal(x_out[0], binding.stack_glue(torch.from_numpy(xp).cuda(), torch.from_numpy(yp).cuda(),
                                                    torch.from_numpy(shift).cuda()))
    assert torch.equal(y, binding.ffn_step(dev, x_out))


def test_real_stack_specs_teacher_forced(oracle):
    """Three layers of the 32-layer benchmark stack at full size (the lowest, a middle and the highest of the
    per-layer target sparsities drawn from U(0.80, 0.95)), each fed what the stack feeds it: the glue of a previous
    token and output, re-centred on the layer's own direction.  Teacher-forced: the oracle's glue output goes into
    svdp_ffn_step; svdp_ffn_step_glued forms the token itself and is checked against the oracle on the token it
    formed (one bf16 rounding apart from the oracle's)."""
    import torch
    from paper_2603_14110_amd import binding, stack

    binding.lib()
    specs = sorted(stack.stack_specs(32), key=lambda sp: sp.sparsity)
    rng = np.random.default_rng(41)
    for sp in (specs[0], specs[len(specs) // 2], specs[-1]):
        L = synth.load_or_make(sp)
        f = {k: L.f32(k) for k in ("W_gate", "W_up", "W_downT", "P", "Q", "b")}
        dev = binding.DeviceLayer.from_synth(L)
        d, D = sp.d, sp.D
        shift = (2.0 * L.u).astype(np.float32)
        dens = []
        for t in range(3):
            # previous layer's token and output: a token of the stream and an output of the FFN's typical size
            xp_st = synth.to_storage(2.0 * rng.standard_normal(d) / np.sqrt(d) + rng.standard_normal(d), "bf16")
            xp = synth.storage_to_f32(xp_st, "bf16")
            yp = (rng.standard_normal(d) * 0.8).astype(np.float32)
            x_or = oracle.stack_glue(xp.astype(np.float64), yp, shift)
            x_st = synth.to_storage(x_or, "bf16")
            x = synth.storage_to_f32(x_st, "bf16")
            # (a) the plain step on the oracle's token
            mask = torch.zeros(D // 64, dtype=torch.int64, device="cuda")
            idx = torch.full((D,), -1, dtype=torch.int32, device="cuda")
            nnz = torch.zeros(1, dtype=torch.int32, device="cuda")
            y = binding.ffn_step(dev, binding.to_device(x_st, "bf16"), mask=mask, idx=idx, nnz=nnz)
            s_or = oracle.predict(f["P"], f["Q"], f["b"], x[None])
            lst = parity.check_mask_and_idx(s_or, mask.cpu().numpy(), idx.cpu().numpy(), nnz.item(), D)
            parity.check_y(y.cpu().numpy(), oracle.sparse_ffn(f["W_gate"], f["W_up"], f["W_downT"], x[None], lst), "bf16")
            dens.append(lst.size / D)
            # (b) glue and step in the same launches
            x_out = torch.zeros(1, d, dtype=torch.bfloat16, device="cuda")
            mask2 = torch.zeros(D // 64, dtype=torch.int64, device="cuda")
            idx2 = torch.full((D,), -1, dtype=torch.int32, device="cuda")
            nnz2 = torch.zeros(1, dtype=torch.int32, device="cuda")
            y2 = binding.ffn_step_glued(dev, binding.to_device(xp_st, "bf16")[None], torch.from_numpy(yp).cuda()[None],
                                        torch.from_numpy(shift).cuda(), x_out, mask=mask2, idx=idx2, nnz=nnz2)
            xg = x_out.float().cpu().numpy()[0]
            assert np.all(np.abs(xg - x_or) <= 2.0 ** -8 * np.maximum(np.abs(x_or), 1.0))
            s2 = oracle.predict(f["P"], f["Q"], f["b"], xg[None])
            lst2 = parity.check_mask_and_idx(s2, mask2.cpu().numpy(), idx2.cpu().numpy(), nnz2.item(), D)
            parity.check_y(y2.cpu().numpy(), oracle.sparse_ffn(f["W_gate"], f["W_up"], f["W_downT"], xg[None], lst2), "bf16")
        # the realised density follows the layer's target (80 % to 95 % sparsity), loosely: three tokens
        assert 0.0 < np.mean(dens) < 0.6, (sp.sparsity, dens)
        del dev
        torch.cuda.empty_cache()
