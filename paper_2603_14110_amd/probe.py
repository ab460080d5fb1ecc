"""ctypes binding over ``libsvdp_probe.so`` (declared in ``include/svdp_probe.h``): measurement helpers for
``bench.py`` - cost of a dependent kernel node, time stamps between graph nodes, latency of a dependent
load, streaming-read ceiling.  Not part of the decode path.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import torch  # imported before the library so both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsvdp_probe.so")
EXPORTS = ["svdp_probe_null", "svdp_probe_stamp", "svdp_probe_handover", "svdp_probe_stream_read", "svdp_probe_chase"]

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.svdp_probe_null.argtypes = [i32, i32, vp]
        L.svdp_probe_stamp.argtypes = [vp, vp]
        L.svdp_probe_handover.argtypes = [vp, vp]
        L.svdp_probe_stream_read.argtypes = [vp, ctypes.c_size_t, i32, vp, vp]
        L.svdp_probe_chase.argtypes = [vp, ctypes.c_uint32, i32, vp, vp]
        for n in EXPORTS:
            getattr(L, n).restype = i32
        _lib = L
    return _lib


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ok(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"{what}: status {rc}")


def null(blocks: int = 256, threads: int = 256) -> None:
    _ok(lib().svdp_probe_null(blocks, threads, _stream()), "svdp_probe_null")


def stamp(slot: torch.Tensor) -> None:
    """slot: one int64 element on the device (a view into a larger tensor is fine)."""
    _ok(lib().svdp_probe_stamp(slot.data_ptr(), _stream()), "svdp_probe_stamp")


def handover(cell: torch.Tensor) -> None:
    _ok(lib().svdp_probe_handover(cell.data_ptr(), _stream()), "svdp_probe_handover")


def stream_read(src: torch.Tensor, nbytes: int, blocks: int, sink: torch.Tensor) -> None:
    _ok(lib().svdp_probe_stream_read(src.data_ptr(), nbytes, blocks, sink.data_ptr(), _stream()),
        "svdp_probe_stream_read")


def chase(ring: torch.Tensor, hops: int, ticks: torch.Tensor) -> None:
    _ok(lib().svdp_probe_chase(ring.data_ptr(), ring.numel(), hops, ticks.data_ptr(), _stream()), "svdp_probe_chase")
