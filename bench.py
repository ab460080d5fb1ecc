#!/usr/bin/env python3
"""Benchmark of the sparse decode step on one MI355X.

A "step" is one pass of the whole hot path - predictor scores, union mask, index
list, gate/up on the active rows, down projection - for one batch of decode
tokens of one layer (for --workload stack: through all layers of the stack, glue
included).  K steps over K different seeded tokens are captured in one HIP graph
and replayed; a single layer's weights rotate over several copies at distinct
addresses so that a step never finds its rows in the 256 MB last-level cache
("cold" mode, the one the roofline fraction is quoted on; the stack is cold by
construction).

Prints ONE JSON line.  `value` is microseconds per token per layer (lower is
better); `roofline` is the algorithmic HBM bytes of a step (summed from the
measured list length of every step) divided by the measured time, against the
8 TB/s peak; `cpu_baseline` is the CPU oracle timed on a bounded sample of the
same tokens on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1024)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default="7b", choices=["tiny", "7b", "13b", "mistral", "stack"])
    ap.add_argument("--rank", type=int, default=0, help="predictor rank (0 = the workload's default)")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--layers", type=int, default=32, help="layers of --workload stack")
    ap.add_argument("--copies", type=int, default=16, help="weight copies rotated through (1 = hot cache)")
    ap.add_argument("--reps", type=int, default=5, help="graph replays; the median is reported")
    ap.add_argument("--flags", type=int, default=0)
    ap.add_argument("--glue-launches", action="store_true",
                    help="--workload stack: the glue between layers as launches of its own (default: inside the "
                         "next layer's first kernel)")
    ap.add_argument("--engine", default="auto", choices=["auto", "vector", "matrix"],
                    help="arithmetic units of the batch-sensitive kernels (SVDP_FLAG_ENGINE_* of the layer)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--table4", action="store_true",
                    help="instead of the step benchmark: FFN-only speed-up at fixed sparsity on the paper's three shapes")
    ap.add_argument("--calibrate", action="store_true",
                    help="time the offline bias calibration (Alg. 2) of the 7B-shaped layer instead of the decode step")
    ap.add_argument("--calib-tokens", type=int, default=2048)
    ap.add_argument("--calib-eta", type=int, default=16)
    ap.add_argument("--calib-sparsity", type=float, default=0.9)
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="also run one plain device copy of this many MiB (calibrates rocprofv3 byte counters)")
    return ap.parse_args()


def time_graph(torch, fn_step, n_steps, warmup, reps, use_graph=True):
    """Median milliseconds for n_steps calls of fn_step(k) (k = 0..n_steps-1), HIP events on the
    stream the kernels are launched on."""
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for k in range(min(warmup, n_steps)):
            fn_step(k)
        stream.synchronize()
        if use_graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for k in range(n_steps):
                    fn_step(k)
            run = g.replay
        else:
            def run():
                for k in range(n_steps):
                    fn_step(k)
        run()
        stream.synchronize()
        times = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            run()
            e1.record(stream)
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
    times.sort()
    return times[len(times) // 2], times


def cpu_baseline_layer(layer, X, B, seconds):
    """The oracle as it stands, timed on the host cores over a bounded sample of the tokens."""
    import oracle

    f = {k: layer.f32(k) for k in ("W_gate", "W_up", "W_downT", "P", "Q", "b")}
    oracle.ffn_step(f, X[:B])                      # load / page in
    n, t0 = 0, time.perf_counter()
    passes = 0
    while time.perf_counter() - t0 < seconds and passes < 8:
        k = 0
        while k + B <= X.shape[0] and time.perf_counter() - t0 < seconds:
            oracle.ffn_step(f, X[k:k + B])
            k += B
            n += B
        passes += 1
    dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
    return {"value": dt / n * 1e6, "unit": "us/token/layer", "cores": cores, "kind": "oracle",
            "sample": f"{n} token evaluations over the timed stream's tokens (in order, wrapping), batch {B}, "
                      f"{dt:.1f} s of wall time"}


def run_layer(a, torch, np, binding, cost, synth):
    over = {"r": a.rank} if a.rank else {}
    spec = synth.workload(a.workload, **over)
    B, K = a.batch, a.steps
    layer = synth.load_or_make(spec)
    w = 2 if spec.dtype == "bf16" else 4
    base = binding.DeviceLayer.from_synth(layer, flags=a.flags)
    copies = [base] + [base.clone() for _ in range(max(a.copies, 1) - 1)]
    X_st = synth.timed_tokens(layer, K * B)
    Xd = binding.to_device(X_st, spec.dtype).view(K, B, spec.d)
    Y = torch.zeros((K, B, spec.d), dtype=torch.float32, device="cuda")
    NNZ = torch.zeros((K, 1), dtype=torch.int32, device="cuda")
    MASK = torch.zeros((K, spec.D // 64), dtype=torch.int64, device="cuda")
    ws = base.workspace(B)

    def sparse_step(k):
        binding.ffn_step(copies[k % len(copies)], Xd[k], ws=ws, out=Y[k], nnz=NNZ[k], mask=MASK[k])

    def rows_only(k):          # the dominant kernel by itself, on the mask words the steps produced
        binding.active_rows(copies[k % len(copies)], Xd[k], MASK[k], ws=ws)

    engine_bits = a.flags & (binding.FLAG_ENGINE_VECTOR | binding.FLAG_ENGINE_MATRIX)
    plain = [c.with_flags(engine_bits) for c in copies]     # the dense baseline never takes the pipeline flags

    def dense_step(k):
        binding.dense_ffn(plain[k % len(plain)], Xd[k], ws=ws, out=Y[k])

    ms, all_ms = time_graph(torch, sparse_step, K, a.warmup, a.reps, not a.no_graph)
    nnz = NNZ.cpu().numpy().reshape(-1).astype(np.int64)
    ms_rows, _ = time_graph(torch, rows_only, K, a.warmup, max(3, a.reps // 2), not a.no_graph)
    Kd = min(K, 128)
    ms_dense, _ = time_graph(torch, dense_step, Kd, min(a.warmup, 8), max(3, a.reps // 2), not a.no_graph)
    bytes_mean = float(np.mean([cost.bytes_sparse(spec.d, spec.D, spec.r, int(n), B, w) for n in nnz]))
    rows_bytes = float(np.mean(cost.bytes_rows(spec.d, nnz, w)))
    alive = None
    if a.flags & binding.FLAG_REVALIDATE:
        # sequential pipeline: rows really read = gate rows of the list + up/down rows of those whose gate is
        # positive for some token of the batch (signs from an fp32 product of the stored values)
        Wg32 = base.tensors["W_gate"].float()
        bits = torch.arange(64, device="cuda", dtype=torch.int64)
        alive = np.zeros(K, dtype=np.int64)
        for k in range(K):
            on = ((MASK[k][:, None] >> bits[None, :]) & 1).reshape(-1).bool()
            pos = (Xd[k].float() @ Wg32.T > 0).any(dim=0)
            alive[k] = int((on & pos).sum().item())
        del Wg32
        rows_bytes = float(np.mean(cost.bytes_rows_sequential(spec.d, nnz, alive, w)))
        bytes_mean += rows_bytes - float(np.mean(cost.bytes_rows(spec.d, nnz, w)))
    res = dict(
        us_step=ms * 1e3 / K, us_dense=ms_dense * 1e3 / Kd, bytes_step=bytes_mean,
        bytes_dense=cost.bytes_dense(spec.d, spec.D, B, w), layers=1, all_ms=all_ms,
        density=nnz / spec.D, us_rows=ms_rows * 1e3 / K, bytes_rows=rows_bytes,
        alive_density=None if alive is None else alive / spec.D,
        workload=f"{spec.name}-shaped layer d={spec.d} D={spec.D} r={spec.r} batch={B}, {K} decode steps, "
                 f"~{spec.sparsity:.0%} activation sparsity per token",
        dtype=spec.dtype, cache_mode="cold" if len(copies) > 1 else "hot", copies=len(copies),
    )
    if not a.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline_layer(layer, synth.storage_to_f32(X_st, spec.dtype), B, a.cpu_seconds)
    return res


def run_stack(a, torch, np, binding, cost, synth):
    from paper_2603_14110_amd import stack

    assert a.batch == 1, "the stacked workload is batch 1"
    over = {"r": a.rank} if a.rank else {}
    specs = stack.stack_specs(a.layers, base="7b", **over)
    K = a.steps
    dev_layers, u_all, L0 = [], [], None
    for i, sp in enumerate(specs):
        L = synth.load_or_make(sp)
        dev_layers.append(binding.DeviceLayer.from_synth(L, flags=a.flags))
        u_all.append(L.u)
        if i == 0:
            L0 = L                      # tokens and the oracle baseline use the first layer
        del L
        print(f"[bench] layer {i + 1}/{len(specs)} ready (target sparsity {sp.sparsity:.3f})", file=sys.stderr, flush=True)
    shifts = [torch.from_numpy((2.0 * u_all[i + 1]).astype(np.float32)).cuda() for i in range(len(specs) - 1)]
    shifts.append(torch.zeros(specs[0].d, dtype=torch.float32, device="cuda"))
    st = stack.FFNStack(dev_layers, shifts, fused_glue=not a.glue_launches)
    X_st = synth.timed_tokens(L0, K)
    Xd = binding.to_device(X_st, "bf16")
    NNZ = torch.zeros((K, len(specs), 1), dtype=torch.int32, device="cuda")
    OUT = torch.zeros((K, specs[0].d), dtype=torch.bfloat16, device="cuda")

    def sparse_step(k):
        OUT[k].copy_(st.step(Xd[k], nnz=NNZ[k]))

    dense = st.as_dense()

    def dense_step(k):
        OUT[k].copy_(dense.step(Xd[k]))

    ms, all_ms = time_graph(torch, sparse_step, K, min(a.warmup, 4), a.reps, not a.no_graph)
    nnz = NNZ.cpu().numpy().reshape(K, len(specs)).astype(np.int64)
    Kd = min(K, 16)
    ms_dense, _ = time_graph(torch, dense_step, Kd, 2, 3, not a.no_graph)
    sp0 = specs[0]
    per_step = [sum(cost.bytes_sparse(sp0.d, sp0.D, sp0.r, int(n), 1, 2) for n in row) for row in nnz]
    res = dict(
        us_step=ms * 1e3 / K, us_dense=ms_dense * 1e3 / Kd, bytes_step=float(np.mean(per_step)),
        bytes_dense=len(specs) * cost.bytes_dense(sp0.d, sp0.D, 1, 2), layers=len(specs), all_ms=all_ms,
        density=(nnz / sp0.D).reshape(-1),
        workload=f"{len(specs)}-layer stack of 7b-shaped layers d={sp0.d} D={sp0.D} r={sp0.r} batch=1, {K} decode "
                 f"steps, per-layer target sparsity U(0.80,0.95), residual + RMS-norm glue, one HIP graph",
        dtype="bf16", cache_mode="cold (8.9 GB of weights)", copies=1,
    )
    if not a.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline_layer(L0, synth.storage_to_f32(X_st, "bf16"), 1, a.cpu_seconds)
        res["cpu_baseline"]["sample"] += " (first layer of the stack only)"
    return res


def measured_traffic(a):
    """HBM bytes per step from the committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE runs,
    calibrated on a plain copy), for the workload that summary covers; None otherwise."""
    if not (a.workload == "7b" and a.batch == 1 and a.rank in (0, 256) and a.flags == 0):
        return None
    path = os.path.join(ROOT, "profiles", "ffn_step_7b_pmc_traffic.txt")
    try:
        out = {}
        for line in open(path):
            if line.startswith("traffic per step"):
                out["bytes_per_step"] = float(line.split(":")[1].split()[0])
            elif line.startswith("algorithmic bytes per step"):
                out["algorithmic_bytes_same_steps"] = float(line.split(":")[1].split()[0])
            elif line.startswith("k_rows traffic per launch"):
                out["rows_bytes_per_launch"] = float(line.split(":")[1].split()[0])
            elif line.startswith("  launches of the kernel alone"):
                out["rows_algorithmic_bytes_same_steps"] = float(line.split(":")[1].split()[0])
        return out if len(out) >= 2 else None
    except OSError:
        return None


def gpu_clocks():
    """Current clocks as rocm-smi reports them right after the timed runs (they cannot be pinned here)."""
    import subprocess

    try:
        p = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=20)
        card = next(iter(json.loads(p.stdout).values()))
        return {k.split()[0]: str(v).strip("()") for k, v in card.items() if "clock speed" in k}
    except Exception as e:          # absent tool, other output format: the benchmark line does not depend on it
        return {"unavailable": type(e).__name__}


def table4(a):
    """The protocol of the paper's executor table (Sec. 5.4): FFN only, predictor excluded, the same
    fixed sparsity on all three projections, speed-up over the dense FFN on the same GPU."""
    import numpy as np
    import torch

    from paper_2603_14110_amd import binding

    shapes = {"llama2-7b": (4096, 11008), "mistral-7b": (4096, 14336), "qwen2-7b": (3584, 18944)}
    rows = []
    rng = np.random.default_rng(7)
    for name, (d, D) in shapes.items():
        g = torch.Generator(device="cuda").manual_seed(11)
        mk = lambda *sh: (torch.randn(*sh, device="cuda", generator=g) / d ** 0.5).to(torch.bfloat16)
        base = binding.DeviceLayer(mk(d, 64), mk(D, 64), torch.zeros(D, device="cuda"), mk(D, d), mk(D, d), mk(D, d))
        copies = [base] + [base.clone() for _ in range(7)]
        K = 64
        X = torch.randn(K, 1, d, device="cuda", generator=g).to(torch.bfloat16)
        Y = torch.zeros(K, 1, d, device="cuda")
        ws = base.workspace(1)
        ms_dense, _ = time_graph(torch, lambda k: binding.dense_ffn(copies[k % 8], X[k], ws=ws, out=Y[k]), K, 4, 3)
        for sp in (0.20, 0.50, 0.80, 0.90, 0.95):
            n = int(round((1.0 - sp) * D))
            IDX = torch.zeros(K, D, dtype=torch.int32, device="cuda")
            for k in range(K):
                IDX[k, :n] = torch.from_numpy(np.sort(rng.choice(D, n, replace=False)).astype(np.int32)).cuda()
            nnz = torch.tensor([n], dtype=torch.int32, device="cuda")
            ms, _ = time_graph(torch, lambda k: binding.sparse_ffn(copies[k % 8], X[k], IDX[k], nnz, ws=ws, out=Y[k]),
                               K, 4, 3)
            rows.append({"shape": name, "d": d, "D": D, "sparsity": sp, "sparse_us": ms * 1e3 / K,
                         "dense_us": ms_dense * 1e3 / K, "speedup": ms_dense / ms})
        del copies, base
        torch.cuda.empty_cache()
    print(json.dumps({"table": "FFN-only speed-up vs dense at fixed sparsity, predictor excluded, bf16, batch 1, "
                               "cold weights (8 copies)", "rows": rows}))


def calibrate(a):
    """Offline bias calibration (Alg. 2) of one layer on the GPU: statistics of T calibration tokens
    (svdp_calib_stats, MFMA contractions), then the greedy selection (svdp_calib_bias).  One JSON line."""
    import time

    import numpy as np
    import torch

    from paper_2603_14110_amd import binding, synth

    L = synth.load_or_make(synth.workload(a.workload if a.workload in ("7b", "13b", "mistral") else "7b"))
    sp = L.spec
    dev = binding.DeviceLayer.from_synth(L)
    T, eta = a.calib_tokens, a.calib_eta
    Xc = synth.make_tokens(sp, L.u, T, 1)                                         # the generator's calibration stream
    Xd = binding.to_device(Xc, sp.dtype)
    need = binding.calib_need(a.calib_sparsity, sp.D, T)
    st = torch.cuda.Stream()

    def timed(fn, reps):
        with torch.cuda.stream(st):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            for _ in range(reps):
                out = fn()
            e1.record(st)
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps, out

    ms_stats, (w, s) = timed(lambda: binding.calib_stats(dev, Xd), 5)
    ms_bias, (b, k, steps, _) = timed(lambda: binding.calib_bias(w, s, eta, need), 3)
    ms_bias_k, _ = timed(lambda: binding.calib_bias(w, s, eta, need, want_kendall=True), 3)
    # the dominant contraction: gate and up against the tokens
    flops = 2.0 * 2.0 * sp.D * T * sp.d
    total_flops = flops + 2.0 * T * sp.r * sp.d + 2.0 * 3 * sp.D * T * sp.r
    tflops = total_flops / (ms_stats * 1e-3) / 1e12
    # what the calibrated bias does on the timed tokens, against the generator's recall-based bias
    Xt = binding.to_device(synth.timed_tokens(L, 256), sp.dtype)
    w_t, s_t = binding.calib_stats(dev, Xt)
    act = (w_t > 0)
    on_new, on_old = s_t + b[:, None] > 0, s_t + dev.tensors["b"][:, None] > 0
    summ = lambda on: {"density": float(on.float().mean()), "recall_of_active": float((on & act).sum() / act.sum()),
                       "lost_damage_fraction": float((w_t * (~on)).sum() / w_t.sum())}
    # CPU oracle: the same layer and tokens (numpy contractions, then the priority-queue loop in Python)
    cpu = None
    if not a.no_cpu_baseline:
        from oracle import calib

        f = {n: L.f32(n) for n in ("W_gate", "W_up", "W_downT", "Q")}
        Xf = synth.storage_to_f32(Xc, sp.dtype)
        t0 = time.perf_counter()
        wo = calib.damage_weights(f["W_gate"], f["W_up"], f["W_downT"], Xf)
        so = calib.proxy_scores(f["Q"], L.f32("P").T, Xf)
        ref = calib.greedy_bias(wo, so, need, eta)
        dt = time.perf_counter() - t0
        cpu = {"value": dt * 1e3, "unit": "ms per layer", "cores": os.cpu_count(), "kind": "oracle",
               "sample": f"the whole layer, {T} tokens, {ref['steps']} greedy steps"}
    print(json.dumps({
        "metric": "offline_bias_calibration_ms_per_layer", "value": ms_stats + ms_bias, "unit": "ms", "n_gpus": 1,
        "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{sp.name} layer d={sp.d} D={sp.D} r={sp.r}, {T} calibration tokens, eta={eta}, "
                               f"sparsity level {a.calib_sparsity}"},
        "stats_ms": ms_stats, "bias_ms": ms_bias, "bias_with_kendall_ms": ms_bias_k, "greedy_steps": int(steps.item()),
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": 2500.0, "unit": "TFLOP/s", "frac": tflops / 2500.0,
                     "traffic": None, "kernel": "svdp_calib_stats (k_gemm_nt x3 + row norms + transpose), bf16 MFMA"},
        "on_256_decode_tokens": {"calibrated_bias": summ(on_new), "generator_bias": summ(on_old)},
        "cpu_baseline": cpu}))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no multi-GPU path exists); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2603_14110_amd import binding, cost, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    binding.lib()
    a.flags |= {"auto": 0, "vector": binding.FLAG_ENGINE_VECTOR, "matrix": binding.FLAG_ENGINE_MATRIX}[a.engine]
    if a.table4:
        table4(a)
        return
    if a.calibrate:
        calibrate(a)
        return
    r = (run_stack if a.workload == "stack" else run_layer)(a, torch, np, binding, cost, synth)
    if a.calib_copy_mb:
        n = a.calib_copy_mb << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    tr = measured_traffic(a)
    K, B, Lyr = a.steps, a.batch, r["layers"]
    us_step, us_dense = r["us_step"], r["us_dense"]
    achieved = r["bytes_step"] / (us_step * 1e-6) / 1e9
    dens = r["density"]
    if "us_rows" in r:
        # the dominant kernel by itself: k_rows, algorithmic bytes = 3 matrices x active rows x d x w per launch
        ach_rows = r["bytes_rows"] / (r["us_rows"] * 1e-6) / 1e9
        roofline = {"bound": "hbm", "achieved": ach_rows, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": ach_rows / HBM_PEAK_GBS, "traffic": (tr or {}).get("rows_bytes_per_launch"),
                    "traffic_algorithmic_bytes_same_launches": (tr or {}).get("rows_algorithmic_bytes_same_steps"),
                    "kernel": "k_rows (mask scan, gate/up/down over the active rows), launched alone K times from the "
                              "steps' mask words (svdp_active_rows), HIP events around the replayed graph",
                    "us_per_launch": r["us_rows"], "algorithmic_bytes_per_launch": r["bytes_rows"]}
    else:
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                    "kernel": "whole step (all kernels of every layer and the glue)",
                    "algorithmic_bytes_per_step": r["bytes_step"]}
    out = {
        "metric": "us_per_token_per_layer_sparse_ffn_decode_incl_predictor",
        "value": us_step / B / Lyr,
        "unit": "us/token/layer",
        "n_gpus": 1,
        "steps": K,
        "warmup": a.warmup,
        "ms_per_step": us_step / 1e3,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if r["dtype"] == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": r["workload"], "batch": B, "layers": Lyr, "weight_copies": r["copies"],
                   "cache_mode": r["cache_mode"], "flags": a.flags, "graph": not a.no_graph,
                   "engine": a.engine,
                   "storage": "bf16 weights/tokens, f32 accumulate" if r["dtype"] == "bf16" else "f32"},
        "density_mean": float(dens.mean()),
        "density_after_gate_mean": None if r.get("alive_density") is None else float(r["alive_density"].mean()),
        "density_percentiles_0_5_50_95_100": [float(np.percentile(dens, p)) for p in (0, 5, 50, 95, 100)],
        "dense_us_per_step": us_dense,
        "dense_us_per_token_per_layer": us_dense / B / Lyr,
        "speedup_vs_dense": us_dense / us_step,
        "dense_achieved_GBs": r["bytes_dense"] / (us_dense * 1e-6) / 1e9,
        "replay_ms_all": r["all_ms"],
        "roofline": roofline,
        "roofline_step": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": (tr or {}).get("bytes_per_step"),
            "traffic_algorithmic_bytes_same_steps": (tr or {}).get("algorithmic_bytes_same_steps"),
            "traffic_source": "profiles/ffn_step_7b_pmc_traffic.txt (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; 64-token run)"
                              if tr else None,
            "kernel": "whole step: all kernels svdp_ffn_step launches (k_xP, k_scores, k_rows, k_reduce_y), "
                      "timed together with HIP events around the replayed graph",
            "algorithmic_bytes_per_step": r["bytes_step"],
        },
        "paper_context": "the paper reports ratios only: up to 1.8x end-to-end decode-time reduction (RTX 3090, fp16, "
                         "vLLM) and 3.3-4.9x FFN-only speedup at 80-95 % sparsity (predictor excluded)",
    }
    if "cpu_baseline" in r:
        out["cpu_baseline"] = r["cpu_baseline"]
    out["clocks"] = gpu_clocks()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
