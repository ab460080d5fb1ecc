#!/usr/bin/env python3
"""Benchmark of the sparse decode step on one MI355X.

A "step" is one pass of the whole hot path - predictor scores, union mask, index
list, gate/up on the active rows, down projection - for one batch of decode
tokens of one layer (for --workload stack: through all layers of the stack, glue
included).

Which tokens are timed: the workload's stream of 1024 decode steps is run once,
untimed, to get every step's list length; the K timed steps are a fixed,
density-stratified subsample of it (K equal-count strata of the sorted densities,
from each the step closest to the stratum's mean, in a seeded random order), so
that a short run sees the stream's density distribution and not its first K tokens.

How they are timed: the K steps are captured in one HIP graph and replayed; a
single layer's weights rotate over several copies at distinct addresses and a 1 GiB
buffer is overwritten before every timed replay, so that a step never finds its
rows in the 256 MB last-level cache ("cold", the mode the roofline fraction is
quoted on; the stack is cold by construction).  The same steps on one copy ("hot"),
each step's own duration from time stamps between the steps of a second graph
(median, 95th percentile), the step with an empty list (the fixed cost of the four
dependent launches), the dense FFN, the machine's floor figures (graph node, value
hand-over between nodes, dependent-load latencies, streaming-read ceiling) and
the CPU oracle on this machine's host cores are reported beside it.

Prints ONE JSON line.  `value` is microseconds per token per layer (lower is
better); `roofline` is for the dominant kernel, `roofline_step` for the whole step:
algorithmic HBM bytes (summed from the measured list length of every timed step)
divided by the measured time, against the 8 TB/s peak and against the measured
streaming-read ceiling.
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
    ap.add_argument("--workload", default="7b", choices=["tiny", "7b", "13b", "mistral", "qwen", "stack"])
    ap.add_argument("--rank", type=int, default=0, help="predictor rank (0 = the workload's default)")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--layers", type=int, default=32, help="layers of --workload stack")
    ap.add_argument("--copies", type=int, default=48,
                    help="weight copies rotated through; 48 copies of a 7B-shaped layer are 13.7 GB, the footprint "
                         "of a whole 7B model, so that caches and address translation see what a decoder's layers "
                         "see (1 = hot cache)")
    ap.add_argument("--reps", type=int, default=5, help="graph replays; the median is reported")
    ap.add_argument("--flags", type=int, default=0)
    ap.add_argument("--glue-launches", action="store_true",
                    help="--workload stack: the glue between layers as launches of its own (default: inside the "
                         "next layer's first kernel)")
    ap.add_argument("--engine", default="auto", choices=["auto", "vector", "matrix"],
                    help="arithmetic units of the batch-sensitive kernels (SVDP_FLAG_ENGINE_* of the layer)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-floor", action="store_true", help="skip the machine-floor probes (graph node, load latency, ceiling)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--table4", action="store_true",
                    help="instead of the step benchmark: FFN-only speed-up at fixed sparsity on the paper's three shapes")
    ap.add_argument("--calibrate", action="store_true",
                    help="time the offline bias calibration (Alg. 2) of the 7B-shaped layer instead of the decode step")
    ap.add_argument("--whiten", action="store_true",
                    help="time the offline predictor build with data whitening (Alg. 1) of the 7B-shaped layer's gate "
                         "matrix instead of the decode step")
    ap.add_argument("--whiten-tokens", type=int, default=8192)
    ap.add_argument("--calib-tokens", type=int, default=2048)
    ap.add_argument("--calib-eta", type=int, default=16)
    ap.add_argument("--calib-sparsity", type=float, default=0.9)
    ap.add_argument("--traffic-pass", action="store_true",
                    help="for rocprofv3 --pmc: one eager pass of the sampled steps between marker launches, then a "
                         "device copy of known size (see profiles/ffn_step_7b_pmc_traffic.txt)")
    return ap.parse_args()


def time_graph(torch, fn_step, n_steps, warmup, reps, use_graph=True, before=None):
    """Median milliseconds for n_steps calls of fn_step(k) (k = 0..n_steps-1), HIP events on the
    stream the kernels are launched on.  `before` (optional) runs untimed before every timed pass."""
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
            if before is not None:
                before()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            run()
            e1.record(stream)
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
    times.sort()
    return times[len(times) // 2], times


POOL_STEPS = 1024          # decode steps of a single-layer workload's stream
SAMPLE_SEED = 20260314


def stratified_sample(np, dens, K, seed=SAMPLE_SEED):
    """K indices into `dens`: one from each of K equal-count strata of the sorted values (the one closest to
    the stratum's mean), in a seeded random order.  K >= len(dens) returns every index."""
    n = len(dens)
    order = np.argsort(dens, kind="stable")
    if K >= n:
        picks = order.copy()
    else:
        edges = (np.arange(K + 1) * n) // K
        picks = np.empty(K, dtype=np.int64)
        for i in range(K):
            stratum = order[edges[i]:edges[i + 1]]
            picks[i] = stratum[np.argmin(np.abs(dens[stratum] - dens[stratum].mean()))]
    np.random.default_rng(seed).shuffle(picks)
    return picks


def cpu_baseline_layer(layer, X, B, seconds):
    """The oracle as it stands, timed on the host cores over a bounded sample of the timed tokens: on all
    cores (OpenMP across independent outputs) and on one thread."""
    import oracle

    f = {k: layer.f32(k) for k in ("W_gate", "W_up", "W_downT", "P", "Q", "b")}
    steps = X.shape[0] // B

    def leg(budget):
        oracle.ffn_step(f, X[:B])                      # load / page in
        n, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < budget:
            k = n % steps
            oracle.ffn_step(f, X[k * B:(k + 1) * B])
            n += 1
        dt = time.perf_counter() - t0
        return dt / (n * B) * 1e6, n, dt

    cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
    oracle.set_threads(cores)
    us_all, n_all, dt_all = leg(seconds)
    oracle.set_threads(1)
    us_one, n_one, dt_one = leg(seconds / 2)
    oracle.set_threads(cores)
    return {"value": us_all, "unit": "us/token/layer", "cores": cores, "kind": "oracle",
            "sample": f"{n_all} steps of batch {B} over the timed tokens (in their timed order, wrapping), "
                      f"{dt_all:.1f} s of wall time",
            "single_thread": {"value": us_one, "unit": "us/token/layer", "cores": 1,
                              "sample": f"{n_one} steps of batch {B}, {dt_one:.1f} s of wall time"}}


def machine_floor(torch, np):
    """Fixed costs and ceilings of this machine, measured with libsvdp_probe in the same process: cost of a
    dependent kernel node in a replayed graph, of handing one value from a node to the next, latency of a
    dependent load at three footprints, and the streaming-read ceiling at three sizes."""
    from paper_2603_14110_amd import probe

    probe.lib()
    out = {}
    N = 1000
    ms, _ = time_graph(torch, lambda k: probe.null(256, 256), N, 8, 3)
    out["graph_node_us"] = ms * 1e3 / N
    cell = torch.zeros(64, dtype=torch.int32, device="cuda")
    ms, _ = time_graph(torch, lambda k: probe.handover(cell), N, 8, 3)
    out["node_with_dependent_load_store_us"] = ms * 1e3 / N
    # dependent-load latency of one lane: a ring that sits in one L2 (1 MiB, walked once before), one that sits
    # in the memory-side cache (64 MiB, streamed through once before, so that the 4 MiB L2 keeps little of it),
    # one that sits in neither (2 GiB, untouched since it was written, pages not yet translated)
    ticks = torch.zeros(2, dtype=torch.int64, device="cuda")
    sink0 = torch.zeros(1, dtype=torch.int32, device="cuda")
    lat = {}
    for name, nbytes, hops, warm in (("L2_1MiB", 1 << 20, 2000, "walk"), ("LLC_64MiB", 64 << 20, 60, "stream"),
                                     ("HBM_2GiB", 2 << 30, 1000, "none")):
        n = nbytes // 4
        # every hop lands on another line (and, for the large rings, another 2 MiB page)
        stride = 4099 if nbytes <= (1 << 20) else (1031 * 1024) // 4 + 33 if nbytes <= (64 << 20) else (2053 * 1024) // 4 + 33
        ring = ((torch.arange(n, dtype=torch.int64, device="cuda") + stride) % n).to(torch.int32)
        if warm == "walk":
            probe.chase(ring, hops, ticks)
        elif warm == "stream":
            probe.stream_read(ring, nbytes, 1024, sink0)
        else:
            torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(3)     # pushes the ring out of the caches
        torch.cuda.synchronize()
        probe.chase(ring, hops, ticks)
        torch.cuda.synchronize()
        lat[name] = float(ticks[0].item()) * 10.0 / hops
        del ring
    out["dependent_load_ns"] = lat
    buf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    buf.fill_(1)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    ceil = {}
    for name, nbytes in (("32MB", 32 << 20), ("256MB", 256 << 20), ("2GB", 2 << 30)):
        nl = min((2 << 30) // nbytes, 32)
        views = [buf[i * nbytes:(i + 1) * nbytes] for i in range(nl)]     # a fresh region per launch
        ms, _ = time_graph(torch, lambda k: probe.stream_read(views[k], nbytes, 1024, sink), nl, 2, 3)
        ceil[name] = nbytes / (ms * 1e-3 / nl) / 1e9
    out["stream_read_GBs"] = ceil
    del buf
    torch.cuda.empty_cache()
    return out


def run_layer(a, torch, np, binding, cost, synth):
    from paper_2603_14110_amd import probe

    over = {"r": a.rank} if a.rank else {}
    spec = synth.workload(a.workload, **over)
    B, K = a.batch, a.steps
    layer = synth.load_or_make(spec)
    w = 2 if spec.dtype == "bf16" else 4
    base = binding.DeviceLayer.from_synth(layer, flags=a.flags)
    copies = [base] + [base.clone() for _ in range(max(a.copies, 1) - 1)]
    ws = base.workspace(B)

    # ---- the stream and the timed subsample of it
    pool = max(POOL_STEPS, K)
    Xpool_st = synth.timed_tokens(layer, pool * B)
    Xpool = binding.to_device(Xpool_st, spec.dtype).view(pool, B, spec.d)
    nnz_pool = torch.zeros((pool, 1), dtype=torch.int32, device="cuda")
    ypool = torch.zeros((B, spec.d), dtype=torch.float32, device="cuda")
    for k in range(pool):
        binding.ffn_step(base, Xpool[k], ws=ws, out=ypool, nnz=nnz_pool[k])
    dens_pool = nnz_pool.cpu().numpy().reshape(-1).astype(np.float64) / spec.D
    sel = stratified_sample(np, dens_pool, K)
    Xd = Xpool[torch.from_numpy(sel).cuda()].contiguous()
    X_st = Xpool_st.reshape(pool, B, spec.d)[sel].reshape(K * B, spec.d)
    del Xpool, nnz_pool

    Y = torch.zeros((K, B, spec.d), dtype=torch.float32, device="cuda")
    NNZ = torch.zeros((K, 1), dtype=torch.int32, device="cuda")
    MASK = torch.zeros((K, spec.D // 64), dtype=torch.int64, device="cuda")
    # untimed, before every timed replay: 1 GiB of other data is READ through the caches, so that nothing of the
    # layer stays in them and they hold no dirty lines whose write-back would ride on the timed steps
    probe.lib()
    flush_buf = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
    flush_sink = torch.zeros(1, dtype=torch.int32, device="cuda")

    def flush():
        probe.stream_read(flush_buf, 1 << 30, 2048, flush_sink)

    def sparse_step(k):
        binding.ffn_step(copies[k % len(copies)], Xd[k], ws=ws, out=Y[k], nnz=NNZ[k], mask=MASK[k])

    def hot_step(k):
        binding.ffn_step(base, Xd[k], ws=ws, out=Y[k])

    def rows_only(k):          # the dominant kernel by itself, on the mask words the steps produced
        binding.active_rows(copies[k % len(copies)], Xd[k], MASK[k], ws=ws, first_kernel_only=True)

    engine_bits = a.flags & (binding.FLAG_ENGINE_VECTOR | binding.FLAG_ENGINE_MATRIX)
    plain = [c.with_flags(engine_bits) for c in copies]     # the dense baseline never takes the pipeline flags

    def dense_step(k):
        binding.dense_ffn(plain[k % len(plain)], Xd[k], ws=ws, out=Y[k])

    graph = not a.no_graph
    ms, all_ms = time_graph(torch, sparse_step, K, a.warmup, a.reps, graph, before=flush)
    nnz = NNZ.cpu().numpy().reshape(-1).astype(np.int64)
    ms_hot, _ = time_graph(torch, hot_step, K, a.warmup, max(3, a.reps // 2), graph)
    ms_rows, _ = time_graph(torch, rows_only, K, a.warmup, max(3, a.reps // 2), graph, before=flush)
    Kd = min(K, 128)
    ms_dense, _ = time_graph(torch, dense_step, Kd, min(a.warmup, 8), max(3, a.reps // 2), graph, before=flush)

    # ---- the same steps with an empty list: what four dependent launches cost when no row is touched
    t = base.tensors
    none_on = binding.DeviceLayer(t["P"], t["Q"], torch.full_like(t["b"], -3.0e38), t["W_gate"], t["W_up"],
                                  t["W_downT"], a.flags)
    empties = [none_on] + [none_on.clone() for _ in range(min(len(copies), 4) - 1)]
    ms_empty, _ = time_graph(torch, lambda k: binding.ffn_step(empties[k % len(empties)], Xd[k], ws=ws, out=Y[k]), K,
                             a.warmup, 3, graph, before=flush)
    del empties, none_on

    # ---- each step's own duration: time stamps between the steps of a second graph
    per_step = None
    if graph:
        stamps = torch.zeros(K + 1, dtype=torch.int64, device="cuda")
        pair = torch.zeros(257, dtype=torch.int64, device="cuda")

        def stamped(k):
            if k == 0:
                probe.stamp(stamps[0:1])
            sparse_step(k)
            probe.stamp(stamps[k + 1:k + 2])

        time_graph(torch, stamped, K, a.warmup, 2, True, before=flush)
        dt = np.diff(stamps.cpu().numpy().astype(np.int64)) * 0.01          # 100 MHz counter -> us
        time_graph(torch, lambda k: probe.stamp(pair[k:k + 1]), 257, 4, 2, True)
        node = float(np.median(np.diff(pair.cpu().numpy().astype(np.int64)))) * 0.01
        own = dt - node                                                    # minus the stamp's own node
        per_step = {"median_us": float(np.median(own)), "p95_us": float(np.percentile(own, 95)),
                    "mean_us": float(own.mean()), "min_us": float(own.min()), "max_us": float(own.max()),
                    "stamp_node_us": node,
                    "how": "time stamps of the GPU's 100 MHz counter between the steps of a replayed graph, one "
                           "stamp node's own cost subtracted"}

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
    dens = nnz / spec.D
    res = dict(
        us_step=ms * 1e3 / K, us_hot=ms_hot * 1e3 / K, us_empty=ms_empty * 1e3 / K, us_dense=ms_dense * 1e3 / Kd,
        bytes_step=bytes_mean, bytes_dense=cost.bytes_dense(spec.d, spec.D, B, w), layers=1, all_ms=all_ms,
        density=dens, density_pool=dens_pool, us_rows=ms_rows * 1e3 / K, bytes_rows=rows_bytes,
        alive_density=None if alive is None else alive / spec.D, per_step=per_step,
        workload=f"{spec.name}-shaped layer d={spec.d} D={spec.D} r={spec.r} batch={B}: {K} decode steps, a "
                 f"density-stratified sample of the stream's {pool}; measured {'union ' if B > 1 else ''}list density "
                 f"{dens.mean():.1%} (stream {dens_pool.mean():.1%}) = {1.0 - dens.mean():.1%} sparsity of the "
                 f"predicted mask (generator target ~{spec.sparsity:.0%} per token)",
        dtype=spec.dtype, cache_mode="cold" if len(copies) > 1 else "hot", copies=len(copies), sample_seed=SAMPLE_SEED,
    )
    del flush_buf
    torch.cuda.empty_cache()
    if not a.no_floor:
        res["floor"] = machine_floor(torch, np)
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


TRAFFIC_PROFILE_MISTRAL_B8 = "profiles/ffn_step_mistral_b8_pmc_traffic.txt"
TRAFFIC_PROFILE = os.path.join("profiles", "ffn_step_7b_pmc_traffic.txt")


def measured_traffic(a):
    """HBM bytes per step and per row-kernel launch from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs of `bench.py --traffic-pass`, calibrated on a plain copy of known size) - but only when
    that summary holds an entry for exactly this run's timed sample (workload, number of steps, sampling seed);
    otherwise None, and the line carries no traffic figure."""
    if (a.flags & 3) != 0 or a.engine != "auto" or a.rank not in (0, 256):
        return None
    if a.workload == "7b" and a.batch == 1:
        profile = TRAFFIC_PROFILE
    elif a.workload == "mistral" and a.batch == 8:
        profile = TRAFFIC_PROFILE_MISTRAL_B8
    else:
        return None
    try:
        for line in open(os.path.join(ROOT, profile)):
            if line.startswith("entry "):
                e = dict(kv.split("=") for kv in line.split()[1:])
                if int(e["steps"]) == a.steps and int(e["sample_seed"]) == SAMPLE_SEED:
                    out = {k: float(v) for k, v in e.items()}
                    out["source"] = profile
                    return out
    except (OSError, ValueError, KeyError):
        pass
    return None


def traffic_pass(a, torch, np, binding, cost, synth):
    """For rocprofv3 --pmc: exactly one eager pass of the K sampled steps on cold weight copies, then the row kernel
    alone on the same steps, then the dense FFN, each region between marker launches (an empty kernel with a
    telling grid size), then a device copy of known size that calibrates the byte counters.  Prints the steps'
    list lengths so that the summary can state the algorithmic bytes of the same steps."""
    from paper_2603_14110_amd import probe

    probe.lib()
    over = {"r": a.rank} if a.rank else {}
    spec = synth.workload(a.workload, **over)
    layer = synth.load_or_make(spec)
    B = a.batch
    base = binding.DeviceLayer.from_synth(layer, flags=a.flags)
    copies = [base] + [base.clone() for _ in range(max(a.copies, 1) - 1)]
    ws = base.workspace(B)
    pool, K = max(POOL_STEPS, a.steps), a.steps
    Xpool = binding.to_device(synth.timed_tokens(layer, pool * B), spec.dtype).view(pool, B, spec.d)
    nnz_pool = torch.zeros((pool, 1), dtype=torch.int32, device="cuda")
    y = torch.zeros((B, spec.d), dtype=torch.float32, device="cuda")
    for k in range(pool):
        binding.ffn_step(base, Xpool[k], ws=ws, out=y, nnz=nnz_pool[k])
    dens_pool = nnz_pool.cpu().numpy().reshape(-1).astype(np.float64) / spec.D
    sel = stratified_sample(np, dens_pool, K)
    Xd = Xpool[torch.from_numpy(sel).cuda()].contiguous()
    NNZ = torch.zeros((K, 1), dtype=torch.int32, device="cuda")
    MASK = torch.zeros((K, spec.D // 64), dtype=torch.int64, device="cuda")
    flush_buf = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
    flush_sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()

    def region(marker_blocks, fn, n):
        probe.stream_read(flush_buf, 1 << 30, 2048, flush_sink)
        probe.null(marker_blocks, 64)
        for k in range(n):
            fn(k)
        probe.null(marker_blocks, 64)
        torch.cuda.synchronize()

    region(7, lambda k: binding.ffn_step(copies[k % len(copies)], Xd[k], ws=ws, out=y, nnz=NNZ[k], mask=MASK[k]), K)
    region(11, lambda k: binding.active_rows(copies[k % len(copies)], Xd[k], MASK[k], ws=ws, first_kernel_only=True), K)
    Kd = min(K, 16)
    region(13, lambda k: binding.dense_ffn(copies[k % len(copies)], Xd[k], ws=ws, out=y), Kd)
    src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    probe.null(17, 64)
    dst.copy_(src)
    probe.null(17, 64)
    torch.cuda.synchronize()
    nnz = NNZ.cpu().numpy().reshape(-1).astype(int)
    w = 2 if spec.dtype == "bf16" else 4
    print(json.dumps({"traffic_pass": True, "workload": a.workload, "batch": B, "steps": K, "sample_seed": SAMPLE_SEED,
                      "dense_steps": Kd, "copy_bytes": 256 << 20, "d": spec.d, "D": spec.D, "r": spec.r,
                      "nnz": nnz.tolist(),
                      "algorithmic_bytes_per_step": float(np.mean([cost.bytes_sparse(spec.d, spec.D, spec.r, int(n), B, w)
                                                                   for n in nnz])),
                      "algorithmic_bytes_rows_per_launch": float(np.mean(cost.bytes_rows(spec.d, nnz, w))),
                      "algorithmic_bytes_dense": cost.bytes_dense(spec.d, spec.D, B, w)}))


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


def whiten(a):
    """Offline predictor build with data whitening (Alg. 1) of one layer's gate matrix on the GPU
    (svdp_whiten_factors: fp64 MFMA contractions, blocked Cholesky factor, block-Jacobi eigen-decomposition).
    One JSON line."""
    import numpy as np
    import torch

    from paper_2603_14110_amd import binding, synth

    L = synth.load_or_make(synth.workload(a.workload if a.workload in ("7b", "13b", "mistral", "qwen") else "7b"))
    sp = L.spec
    r, T = (a.rank or sp.r), a.whiten_tokens
    Wg = binding.to_device(L.W_gate, sp.dtype)
    # calibration tokens: the generator's stream 1 mixed through a fixed anisotropic map, so that whitening matters
    rng = np.random.default_rng([sp.seed, 7])
    Xc = synth.storage_to_f32(synth.make_tokens(sp, L.u, T, 1), sp.dtype).astype(np.float64)
    Xc = Xc * (0.9995 ** np.arange(sp.d))[rng.permutation(sp.d)][None, :]
    X_st = synth.to_storage(Xc, sp.dtype)
    Xd = binding.to_device(X_st, sp.dtype)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    P, Q, sigma, sweeps = binding.whiten_factors(Wg, Xd, r)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3
    # what Alg. 1 minimises, evaluated on the GPU in fp64 with plain torch ops (a check, not part of the path)
    W64 = Wg.double()
    X64 = Xd.double()
    err = torch.linalg.norm((W64 - Q.double() @ P.double().T) @ X64.T).item()
    ref = torch.linalg.norm(W64 @ X64.T).item()
    flops = 2.0 * (sp.d * sp.d * T + 2.0 * sp.D * sp.d * sp.d + sp.D * sp.d * r + sp.d * sp.d * r)
    # block Jacobi: per round every 64 x 64 tile of the matrix takes two 64^3 products and every tile of the
    # eigenvector rows one; d/32 - 1 rounds per sweep; the Cholesky factor d^3 / 3
    tiles = (sp.d // 64) ** 2
    jacobi_flops = sweeps[1] * (sp.d // 32 - 1) * tiles * 3 * 2.0 * 64 ** 3
    all_flops = flops + jacobi_flops + sp.d ** 3 / 3.0
    peak = 78.6
    cpu = None
    if not a.no_cpu_baseline:
        from oracle import calib

        Wf = L.f32("W_gate").astype(np.float64)
        Xf = synth.storage_to_f32(X_st, sp.dtype).astype(np.float64)
        t0 = time.perf_counter()
        A, B = calib.whitened_factors(Wf, Xf, r)
        dt = time.perf_counter() - t0
        err_or = float(np.linalg.norm((Wf - A @ B) @ Xf.T))
        cpu = {"value": dt * 1e3, "unit": "ms per layer", "cores": os.cpu_count(), "kind": "oracle",
               "sample": f"the whole layer (LAPACK Cholesky, SVD of the {sp.D} x {sp.d} whitened matrix, triangular solve)",
               "error_on_the_tokens": err_or, "gpu_error_relative_to_it": err / err_or}
    print(json.dumps({
        "metric": "offline_whitened_factorisation_ms_per_layer", "value": ms, "unit": "ms", "n_gpus": 1,
        "higher_is_better": False, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{sp.name} gate matrix d={sp.d} D={sp.D}, rank {r}, {T} calibration tokens"},
        "jacobi_sweeps": list(sweeps), "sigma_first_last": [float(sigma[0]), float(sigma[-1])],
        "error_on_the_tokens": err, "error_relative_to_W_X": err / ref,
        "contraction_gflop": flops / 1e9, "jacobi_gflop": jacobi_flops / 1e9,
        "roofline": {"bound": "mfma", "achieved": all_flops / (ms * 1e-3) / 1e12, "peak": peak, "unit": "TFLOP/s",
                     "frac": all_flops / (ms * 1e-3) / 1e12 / peak, "traffic": None,
                     "kernel": "the whole call (fp64 matrix-core flops of the contractions, the Cholesky factor and the "
                               "block-Jacobi tile updates over the wall time, host synchronisations included)"},
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
    if a.whiten:
        whiten(a)
        return
    if a.traffic_pass:
        traffic_pass(a, torch, np, binding, cost, synth)
        return
    r = (run_stack if a.workload == "stack" else run_layer)(a, torch, np, binding, cost, synth)

    tr = measured_traffic(a)
    K, B, Lyr = a.steps, a.batch, r["layers"]
    us_step, us_dense = r["us_step"], r["us_dense"]
    achieved = r["bytes_step"] / (us_step * 1e-6) / 1e9
    dens = r["density"]
    floor = r.get("floor")
    ceiling = None if floor is None else floor["stream_read_GBs"]["256MB"]
    of_ceiling = lambda gbs: None if ceiling is None else gbs / ceiling
    if "us_rows" in r:
        # the dominant kernel by itself: the row kernel, algorithmic bytes = 3 matrices x active rows x d x w per launch
        ach_rows = r["bytes_rows"] / (r["us_rows"] * 1e-6) / 1e9
        roofline = {"bound": "hbm", "achieved": ach_rows, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": ach_rows / HBM_PEAK_GBS,
                    "traffic": (tr or {}).get("rows_traffic_per_launch"),
                    "traffic_algorithmic_bytes_same_launches": (tr or {}).get("rows_algorithmic_per_launch"),
                    "frac_of_measured_ceiling": of_ceiling(ach_rows),
                    "kernel": "k_rows (mask scan, gate/up/down over the active rows; for batches on the matrix cores the "
                              "pair k_gate_up_mfma + k_down_slices), launched alone K times from the steps' mask words "
                              "(svdp_active_rows), HIP events around the replayed graph",
                    "us_per_launch": r["us_rows"], "algorithmic_bytes_per_launch": r["bytes_rows"]}
    else:
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                    "kernel": "whole step (all kernels of every layer and the glue)",
                    "algorithmic_bytes_per_step": r["bytes_step"]}
    dense_gbs = r["bytes_dense"] / (us_dense * 1e-6) / 1e9
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
                   "engine": a.engine, "sample_seed": r.get("sample_seed"),
                   "storage": "bf16 weights/tokens, f32 accumulate" if r["dtype"] == "bf16" else "f32"},
        "density_mean": float(dens.mean()),
        "density_mean_of_stream": None if r.get("density_pool") is None else float(r["density_pool"].mean()),
        "density_after_gate_mean": None if r.get("alive_density") is None else float(r["alive_density"].mean()),
        "density_percentiles_0_5_50_95_100": [float(np.percentile(dens, p)) for p in (0, 5, 50, 95, 100)],
        "cold_us_per_step": us_step,
        "hot_us_per_step": r.get("us_hot"),
        "empty_list_step_us": r.get("us_empty"),
        "per_step_us": r.get("per_step"),
        "dense_us_per_step": us_dense,
        "dense_us_per_token_per_layer": us_dense / B / Lyr,
        "speedup_vs_dense": us_dense / us_step,
        "dense_achieved_GBs": dense_gbs,
        "dense_frac_of_measured_ceiling": of_ceiling(dense_gbs),
        "replay_ms_all": r["all_ms"],
        "roofline": roofline,
        "roofline_step": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": (tr or {}).get("step_traffic"),
            "traffic_algorithmic_bytes_same_steps": (tr or {}).get("step_algorithmic"),
            "traffic_source": (tr["source"] + " (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE of `bench.py --traffic-pass` "
                               "on this run's timed sample)") if tr else None,
            "frac_of_measured_ceiling": of_ceiling(achieved),
            "kernel": "whole step: all kernels svdp_ffn_step launches (k_xP, k_scores, k_rows or k_gate_up_mfma + "
                      "k_down_slices, k_reduce_y), timed together with HIP events around the replayed graph",
            "algorithmic_bytes_per_step": r["bytes_step"],
        },
        "machine_floor": floor,
        "paper_context": "the paper reports ratios only: up to 1.8x end-to-end decode-time reduction (RTX 3090, fp16, "
                         "vLLM) and 3.3-4.9x FFN-only speedup at 80-95 % sparsity (predictor excluded)",
    }
    if "cpu_baseline" in r:
        out["cpu_baseline"] = r["cpu_baseline"]
    out["clocks"] = gpu_clocks()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
