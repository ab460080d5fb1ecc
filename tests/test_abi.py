"""CPU checks of the C-ABI boundary: the library loads, exports every symbol the
header declares, and its host-only logic (workspace sizing, argument validation,
status strings) behaves.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def svdp():
    from paper_2603_14110_amd import binding, build

    if not os.path.exists(binding.LIB_PATH):
        build.build_lib()
    return binding


def _declared():
    text = open(os.path.join(ROOT, "include", "svdp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(svdp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(svdp):
    L = svdp.lib()
    names = _declared()
    assert set(names) == set(svdp.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_probe_library_exports_what_its_header_declares():
    """libsvdp_probe (the benchmark's measurement helpers): loads, and exports exactly the header's symbols."""
    import subprocess

    from paper_2603_14110_amd import build, probe

    if not os.path.exists(probe.LIB_PATH):
        build.build_probe()
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "svdp_probe.h")).read(), flags=re.S)
    declared = sorted(set(re.findall(r"\b(svdp_probe_[a-z_]+)\s*\(", text)))
    assert declared == sorted(probe.EXPORTS)
    L = probe.lib()
    for n in declared:
        assert getattr(L, n) is not None
    out = subprocess.run(["nm", "-D", "--defined-only", probe.LIB_PATH], capture_output=True, text=True, check=True).stdout
    assert sorted(set(re.findall(r"\b(svdp_probe_[a-z_0-9]+)\b", out))) == declared
    # host-side validation: nothing is launched for bad arguments
    assert L.svdp_probe_null(0, 64, None) == 1 and L.svdp_probe_null(1, 2048, None) == 1
    assert L.svdp_probe_stamp(None, None) == 1 and L.svdp_probe_handover(None, None) == 1
    assert L.svdp_probe_stream_read(0x1000, 24, 4, 0x1000, None) == 1          # not a multiple of 16 bytes
    assert L.svdp_probe_chase(None, 4, 4, 0x1000, None) == 1


def test_bench_sample_is_stratified_and_seeded():
    """The timed subsample of bench.py: fixed for a given K, without repeats, and its mean density follows the
    stream's within half a percentage point from 20 steps up, on a skewed density distribution."""
    import numpy as np

    import bench

    rng = np.random.default_rng(5)
    dens = np.clip(rng.gamma(0.45, 0.22, 1024), 0.0, 0.9)          # median well under the mean, a long tail
    for K in (5, 20, 64, 200, 1024, 2000):
        s1, s2 = bench.stratified_sample(np, dens, K), bench.stratified_sample(np, dens, K)
        assert np.array_equal(s1, s2) and len(set(s1.tolist())) == min(K, 1024) == len(s1)
        if K >= 20:
            assert abs(dens[s1].mean() - dens.mean()) < 0.005
    first20 = dens[:20].mean()
    assert abs(dens[bench.stratified_sample(np, dens, 20)].mean() - dens.mean()) <= abs(first20 - dens.mean()) + 0.005


def test_bench_attaches_measured_traffic_only_to_the_sample_it_was_measured_on():
    """bench.py takes roofline.traffic from the committed counter summaries, and only for the workload, number of
    steps and sampling seed a summary has an entry for (the driver's 20-step run and the default run among them)."""
    import types

    import bench

    def args(**kw):
        base = dict(workload="7b", batch=1, rank=0, flags=0, engine="auto", steps=20)
        base.update(kw)
        return types.SimpleNamespace(**base)

    for a in (args(), args(steps=1024), args(workload="mistral", batch=8, steps=256)):
        e = bench.measured_traffic(a)
        assert e is not None and e["steps"] == a.steps and e["sample_seed"] == bench.SAMPLE_SEED
        assert e["step_traffic"] >= e["step_algorithmic"] > 0
        assert e["rows_traffic_per_launch"] >= e["rows_algorithmic_per_launch"] > 0
        assert e["step_traffic"] < 1.5 * e["step_algorithmic"]
    for a in (args(steps=21), args(workload="13b"), args(flags=2), args(engine="vector"), args(rank=128),
              args(workload="mistral", batch=4, steps=256)):
        assert bench.measured_traffic(a) is None


def test_status_strings_and_version(svdp):
    L = svdp.lib()
    seen = {L.svdp_status_string(i).decode() for i in range(5)}
    assert len(seen) == 5 and "ok" in seen
    assert L.svdp_status_string(99) is not None
    assert re.match(r"^\d+\.\d+$", svdp.version())


def _layer(svdp, d=4096, D=11008, r=256, dt=1, ptr=0x1000):
    return svdp.svdp_layer(d, D, r, dt, ptr, ptr, ptr, ptr, ptr, ptr, 0)


def test_workspace_bytes(svdp):
    L = svdp.lib()
    l = _layer(svdp)
    w1 = L.svdp_workspace_bytes(ctypes.byref(l), 1)
    w8 = L.svdp_workspace_bytes(ctypes.byref(l), 8)
    assert 0 < w1 < w8 < (1 << 30)
    assert w1 % 256 == 0
    # at least the mask words and the partial y's of the row blocks
    assert w1 >= 11008 // 8 + 256 * 4096 * 4
    assert L.svdp_workspace_bytes(ctypes.byref(l), 0) == 0
    assert L.svdp_workspace_bytes(ctypes.byref(l), 9) == 0
    assert L.svdp_workspace_bytes(ctypes.byref(_layer(svdp, D=11000)), 1) == 0     # D % 64
    assert L.svdp_workspace_bytes(ctypes.byref(_layer(svdp, d=4100)), 1) == 0      # d % 8 (bf16)
    assert L.svdp_workspace_bytes(ctypes.byref(_layer(svdp, d=4100, dt=0)), 1) > 0  # d % 4 ok for fp32
    assert L.svdp_workspace_bytes(ctypes.byref(_layer(svdp, dt=7)), 1) == 0
    assert L.svdp_workspace_bytes(None, 1) == 0


def test_validation_rejects_before_any_launch(svdp):
    """Bad arguments return an error code on the host; nothing reaches a device."""
    L = svdp.lib()
    l = _layer(svdp)
    ws = 1 << 28
    INVALID, UNSUPPORTED, WORKSPACE = 1, 2, 3
    assert L.svdp_predict(ctypes.byref(l), None, 1, 0x1000, 0x1000, ws, None) == INVALID
    assert L.svdp_predict(ctypes.byref(l), 0x1000, 0, 0x1000, 0x1000, ws, None) == INVALID
    assert L.svdp_predict(ctypes.byref(l), 0x1000, 9, 0x1000, 0x1000, ws, None) == INVALID
    assert L.svdp_predict(ctypes.byref(l), 0x1000, 1, 0x1000, None, ws, None) == WORKSPACE
    assert L.svdp_predict(ctypes.byref(l), 0x1000, 1, 0x1000, 0x1000, 16, None) == WORKSPACE
    assert L.svdp_predict(ctypes.byref(l), 0x1000, 1, 0x1000, 0x1010, ws, None) == WORKSPACE   # misaligned ws
    assert L.svdp_dense_ffn(ctypes.byref(_layer(svdp, D=100)), 0x1000, 1, 0x1000, 0x1000, ws, None) == UNSUPPORTED
    assert L.svdp_dense_ffn(ctypes.byref(_layer(svdp, ptr=0x1004)), 0x1000, 1, 0x1000, 0x1000, ws, None) == INVALID
    assert L.svdp_sparse_ffn(ctypes.byref(l), 0x1000, 1, None, 0x1000, 0x1000, 0x1000, ws, None) == INVALID
    assert L.svdp_ffn_step(ctypes.byref(l), 0x1000, 1, None, None, None, None, 0x1000, ws, None) == INVALID
    bad = _layer(svdp)
    bad.flags = 16                                        # an unknown flag bit
    assert L.svdp_ffn_step(ctypes.byref(bad), 0x1000, 1, 0x1000, None, None, None, 0x1000, ws, None) == INVALID
    bad.flags = svdp.FLAG_ENGINE_VECTOR | svdp.FLAG_ENGINE_MATRIX       # both engines at once
    assert L.svdp_ffn_step(ctypes.byref(bad), 0x1000, 1, 0x1000, None, None, None, 0x1000, ws, None) == INVALID
    assert L.svdp_workspace_bytes(ctypes.byref(bad), 1) == 0
    # a batch of tokens that does not fit a compute unit's local memory next to the row kernel's scratch is
    # refused before anything is enqueued, and the size query says so too
    big = _layer(svdp, d=16384, D=4096, r=64, dt=0)
    assert L.svdp_workspace_bytes(ctypes.byref(big), 8) == 0
    assert L.svdp_workspace_bytes(ctypes.byref(big), 1) > 0
    assert L.svdp_ffn_step(ctypes.byref(big), 0x1000, 8, 0x1000, None, None, None, 0x1000, 1 << 40, None) == UNSUPPORTED
    assert L.svdp_dense_ffn(ctypes.byref(big), 0x1000, 8, 0x1000, 0x1000, 1 << 40, None) == UNSUPPORTED
    assert L.svdp_compact(None, 1, 64, 0x1000, 0x1000, 0x1000, None, 0, None) == INVALID
    assert L.svdp_compact(0x1000, 1, 100, 0x1000, 0x1000, 0x1000, None, 0, None) == UNSUPPORTED
    assert L.svdp_stack_glue(None, 0x1000, 0x1000, 64, 0, 1e-6, 0x1000, None) == INVALID
    assert L.svdp_active_rows(ctypes.byref(l), 0x1000, 1, None, None, 0x1000, ws, None) == INVALID
    assert L.svdp_active_rows(ctypes.byref(l), 0x1000, 1, 0x1000, 0x1004, 0x1000, ws, None) == INVALID
    assert L.svdp_active_rows(ctypes.byref(l), 0x1000, 1, 0x1000, None, 0x1000, 64, None) == WORKSPACE


def test_library_has_no_process_wide_switches(svdp):
    """Modes and engines travel in svdp_layer.flags: no setter (or any other call that changes later calls)
    is exported, by the header or by the shared object."""
    import subprocess

    names = _declared()
    assert not [n for n in names if "_set_" in n or n.endswith("_timeouts")]
    out = subprocess.run(["nm", "-D", "--defined-only", svdp.LIB_PATH], capture_output=True, text=True, check=True).stdout
    exported = sorted(set(re.findall(r"\b(svdp_[a-z_0-9]+)\b", out)))
    assert exported == names, (exported, names)


def test_static_scratch_entry_point_validates_on_the_host(svdp):
    """svdp_ffn_step_static: same argument checks as svdp_ffn_step, and a layer or batch whose scratch need
    exceeds the library's static array is refused (before any device is touched)."""
    L = svdp.lib()
    INVALID, UNSUPPORTED, WORKSPACE = 1, 2, 3
    l = _layer(svdp)
    assert L.svdp_workspace_bytes(ctypes.byref(l), 1) <= svdp.STATIC_SCRATCH_BYTES < L.svdp_workspace_bytes(ctypes.byref(l), 2)
    assert L.svdp_ffn_step_static(ctypes.byref(l), 0x1000, 2, 0x1000, None, None, None, None) == WORKSPACE
    assert L.svdp_ffn_step_static(ctypes.byref(l), 0x1000, 8, 0x1000, None, None, None, None) == WORKSPACE
    assert L.svdp_ffn_step_static(ctypes.byref(l), None, 1, 0x1000, None, None, None, None) == INVALID
    assert L.svdp_ffn_step_static(ctypes.byref(l), 0x1000, 0, 0x1000, None, None, None, None) == INVALID
    assert L.svdp_ffn_step_static(ctypes.byref(_layer(svdp, D=100)), 0x1000, 1, 0x1000, None, None, None, None) == UNSUPPORTED
    text = open(os.path.join(ROOT, "include", "svdp.h")).read()
    m = re.search(r"#define SVDP_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", text)
    assert int(m.group(1)) << int(m.group(2)) == svdp.STATIC_SCRATCH_BYTES


def test_calib_need_is_the_oracles_rule(svdp):
    """svdp_calib_need against the oracle's required_drops on a grid incl. products that are not exact in
    binary (0.7 * 10, 0.1 * 3 ...), the clamps and the invalid cases."""
    import math
    from fractions import Fraction

    from oracle import calib

    L = svdp.lib()
    for D, T in ((1, 1), (10, 1), (3, 1), (7, 13), (11008, 2048), (64, 4096), (1000, 1000)):
        for sp in (0.0, 0.1, 0.3, 0.5, 0.7, 0.85, 0.9, 0.95, 0.999, 1.0, 1.5, -0.2, 1 / 3, 2 / 3, 1e-12):
            assert L.svdp_calib_need(sp, D, T) == calib.required_drops(sp, D, T), (sp, D, T)
    assert L.svdp_calib_need(0.5, 0, 4) == -1 and L.svdp_calib_need(float("nan"), 4, 4) == -1


def test_whitening_entry_points_validate_on_the_host(svdp):
    L = svdp.lib()
    a = 0x1000
    INVALID, UNSUPPORTED, WORKSPACE = 1, 2, 3
    n = L.svdp_whiten_workspace_bytes(4096, 11008, 8192, 256)
    # fp64 copies of W, W S and its transpose, the tokens, two ping-pong pairs of d x d matrices, S^T and E
    assert n % 256 == 0 and n >= 8 * (3 * 11008 * 4096 + 4096 * 8192 + 6 * 4096 * 4096)
    for bad in ((4000, 11008, 8192, 256), (4096, 0, 8192, 256), (4096, 11008, 4095, 256), (4096, 11008, 8192, 0),
                (4096, 11008, 8192, 5000), (32, 64, 64, 8)):
        assert L.svdp_whiten_workspace_bytes(*bad) == 0, bad
    args = lambda **o: [o.get("W", a), o.get("X", a), o.get("d", 128), 256, o.get("T", 512), o.get("r", 8), o.get("dt", 1),
                        o.get("P", a), a, None, None, o.get("ws", a), o.get("n", 1 << 30), None]
    assert L.svdp_whiten_factors(*args(W=None)) == INVALID
    assert L.svdp_whiten_factors(*args(P=None)) == INVALID
    assert L.svdp_whiten_factors(*args(dt=5)) == UNSUPPORTED
    assert L.svdp_whiten_factors(*args(d=96)) == UNSUPPORTED
    assert L.svdp_whiten_factors(*args(T=100)) == UNSUPPORTED
    assert L.svdp_whiten_factors(*args(ws=None)) == WORKSPACE
    assert L.svdp_whiten_factors(*args(ws=0x1010)) == WORKSPACE
    assert L.svdp_whiten_factors(*args(n=1024)) == WORKSPACE


def test_calibration_entry_points_validate_on_the_host(svdp):
    L = svdp.lib()
    INVALID, UNSUPPORTED, WORKSPACE = 1, 2, 3
    wb = L.svdp_calib_workspace_bytes(11008, 2048, 16)
    # running maxima, dropped counts and thresholds per step of every neuron
    assert wb % 256 == 0 and wb >= 11008 * (128 * 4 + 2 * 129 * 4 + 4)
    assert L.svdp_calib_workspace_bytes(11008, 4096, 1) > wb
    for bad in ((0, 16, 1), (4, 0, 1), (4, 4097, 1), (4, 16, 0)):
        assert L.svdp_calib_workspace_bytes(*bad) == 0
    a = 0x1000
    assert L.svdp_calib_bias(None, a, 4, 8, 1, 3, a, None, None, None, a, 1 << 20, None) == INVALID
    assert L.svdp_calib_bias(a, a, 4, 8, 1, -1, a, None, None, None, a, 1 << 20, None) == INVALID
    assert L.svdp_calib_bias(a, a, 4, 8, 0, 3, a, None, None, None, a, 1 << 20, None) == INVALID
    assert L.svdp_calib_bias(a, a, 4, 5000, 1, 3, a, None, None, None, a, 1 << 30, None) == UNSUPPORTED
    assert L.svdp_calib_bias(a, a, 4, 8, 1, 3, a, None, None, None, None, 1 << 20, None) == WORKSPACE
    assert L.svdp_calib_bias(a, a, 4, 8, 1, 3, a, None, None, None, a, 16, None) == WORKSPACE
    l = _layer(svdp)
    ws = L.svdp_calib_stats_workspace_bytes(ctypes.byref(l), 2048)
    assert ws % 256 == 0 and ws >= 256 * 4096 * 2 + 11008 * 4 + 2048 * 3 * 256 * 2
    assert L.svdp_calib_stats_workspace_bytes(ctypes.byref(_layer(svdp, dt=0)), 2048) == 0      # bf16 only
    assert L.svdp_calib_stats_workspace_bytes(ctypes.byref(l), 0) == 0
    assert L.svdp_calib_stats(ctypes.byref(l), None, 8, a, a, a, ws, None) == INVALID
    assert L.svdp_calib_stats(ctypes.byref(_layer(svdp, dt=0, d=4096)), a, 8, a, a, a, 1 << 30, None) == UNSUPPORTED
    assert L.svdp_calib_stats(ctypes.byref(l), a, 8, a, a, a, 64, None) == WORKSPACE


def test_binding_fails_loudly_without_library(svdp, monkeypatch):
    monkeypatch.setattr(svdp, "_lib", None)
    monkeypatch.setattr(svdp, "LIB_PATH", "/nonexistent/libsvdp.so")
    with pytest.raises(svdp.SvdpError):
        svdp.lib()


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: `bench.py --gpus N` with N > 1 says so and exits without touching a device."""
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""
