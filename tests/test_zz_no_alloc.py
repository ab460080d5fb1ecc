"""svdp_ffn_step_static (the step with the scratch in the library's own static device array, for callers
that cannot allocate) against svdp_ffn_step on a caller-provided workspace: same kernels, so the outputs are
compared bit for bit (mask words, list length, list, y), on two calls in a row, the second with a smaller
input; then the same pair again, so that whatever the first round left in the array meets the second."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _random_layer(binding, torch, d, D, r, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    mk = lambda *sh: (torch.randn(*sh, device="cuda", generator=g) / d ** 0.5).to(torch.bfloat16)
    Q = torch.randn(D, r, device="cuda", generator=g).to(torch.bfloat16)
    b = torch.randn(D, device="cuda", generator=g) * 0.5 - 1.3          # about a tenth of the neurons on
    return binding.DeviceLayer(mk(d, r), Q, b, mk(D, d), mk(D, d), mk(D, d))


def _both(binding, torch, dev, x):
    D = dev.D
    outs = []
    for static in (False, True):
        mask = torch.zeros(D // 64, dtype=torch.int64, device="cuda")
        idx = torch.full((D,), -1, dtype=torch.int32, device="cuda")
        nnz = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        if static:
            y = binding.ffn_step_static(dev, x, mask=mask, idx=idx, nnz=nnz)
        else:
            y = binding.ffn_step(dev, x, mask=mask, idx=idx, nnz=nnz)
        torch.cuda.synchronize()
        outs.append((mask, idx, nnz, y))
    (m0, i0, n0, y0), (m1, i1, n1, y1) = outs
    assert torch.equal(m0, m1) and torch.equal(n0, n1) and torch.equal(i0, i1)
    assert torch.equal(y0, y1)
    assert 0 < n0.item() < D and bool(torch.isfinite(y0).all()) and float(y0.abs().max()) > 0
    return n0.item()


def test_static_scratch_step_equals_workspace_step():
    import torch
    from paper_2603_14110_amd import binding

    assert torch.cuda.is_available(), "this test needs a GPU"
    binding.lib()
    big = _random_layer(binding, torch, 4096, 11008, 256, seed=1)       # the 7B shape: 4.3 MB of scratch, batch 1
    small = _random_layer(binding, torch, 512, 2048, 64, seed=2)        # batch 3: another kernel family, less scratch
    g = torch.Generator(device="cuda").manual_seed(3)
    xb = torch.randn(1, 4096, device="cuda", generator=g).to(torch.bfloat16)
    xs = torch.randn(3, 512, device="cuda", generator=g).to(torch.bfloat16)
    assert binding.workspace_bytes(big, 1) <= binding.STATIC_SCRATCH_BYTES
    counts = []
    for _ in range(2):
        counts.append(_both(binding, torch, big, xb))
        counts.append(_both(binding, torch, small, xs))
    assert counts[0] == counts[2] and counts[1] == counts[3]
    # beyond the array: refused with the workspace status, nothing enqueued
    with pytest.raises(binding.SvdpError, match="workspace"):
        binding.ffn_step_static(big, torch.cat([xb, xb]))
    # and against the oracle, so that the pair is not merely equal to each other
    import oracle
    import parity

    D = small.D
    f = {k: v.float().cpu().numpy() for k, v in small.tensors.items()}
    X = xs.float().cpu().numpy()
    mask = torch.zeros(D // 64, dtype=torch.int64, device="cuda")
    idx = torch.full((D,), -1, dtype=torch.int32, device="cuda")
    nnz = torch.zeros(1, dtype=torch.int32, device="cuda")
    y = binding.ffn_step_static(small, xs, mask=mask, idx=idx, nnz=nnz)
    torch.cuda.synchronize()
    s_or = oracle.predict(f["P"], f["Q"], f["b"], X)
    lst = parity.check_mask_and_idx(s_or, mask.cpu().numpy(), idx.cpu().numpy(), nnz.item(), D)
    y_ref = oracle.sparse_ffn(f["W_gate"], f["W_up"], f["W_downT"], X, lst)
    parity.check_y(y.cpu().numpy(), y_ref, "bf16", slack=parity.fp32_forward_bound(f, X, lst))
