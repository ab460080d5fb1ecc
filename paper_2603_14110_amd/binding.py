"""Thin ctypes binding over ``libsvdp.so`` (declared in ``include/svdp.h``).

Argument marshalling only: torch supplies device memory and the current HIP
stream, every step of the path runs in the library's kernels.  There is no CPU
or eager fallback: if the library has not been built, ``lib()`` raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np
import torch  # imported before the library so both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsvdp.so")

SVDP_F32, SVDP_BF16 = 0, 1
FLAG_DRELU, FLAG_REVALIDATE, FLAG_ENGINE_VECTOR, FLAG_ENGINE_MATRIX = 1, 2, 4, 8
MAX_BATCH = 8
STATIC_SCRATCH_BYTES = 8 << 20

EXPORTS = [
    "svdp_workspace_bytes", "svdp_predict", "svdp_compact", "svdp_sparse_ffn", "svdp_dense_ffn",
    "svdp_ffn_step", "svdp_ffn_step_static", "svdp_stack_glue", "svdp_status_string", "svdp_version",
    "svdp_active_rows", "svdp_calib_workspace_bytes", "svdp_calib_need", "svdp_calib_bias",
    "svdp_calib_stats_workspace_bytes", "svdp_calib_stats", "svdp_ffn_step_glued",
    "svdp_whiten_workspace_bytes", "svdp_whiten_factors",
]


class SvdpError(RuntimeError):
    pass


class svdp_layer(ctypes.Structure):
    _fields_ = [
        ("d", ctypes.c_int32), ("D", ctypes.c_int32), ("r", ctypes.c_int32), ("wdtype", ctypes.c_int32),
        ("P", ctypes.c_void_p), ("Q", ctypes.c_void_p), ("b", ctypes.c_void_p),
        ("W_gate", ctypes.c_void_p), ("W_up", ctypes.c_void_p), ("W_downT", ctypes.c_void_p),
        ("flags", ctypes.c_uint32),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """Load the built library; raises SvdpError when it is missing (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise SvdpError(f"{LIB_PATH} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lp = ctypes.POINTER(svdp_layer)
    L.svdp_workspace_bytes.argtypes = [lp, i32]
    L.svdp_workspace_bytes.restype = sz
    L.svdp_predict.argtypes = [lp, vp, i32, vp, vp, sz, vp]
    L.svdp_compact.argtypes = [vp, i32, i32, vp, vp, vp, vp, sz, vp]
    L.svdp_sparse_ffn.argtypes = [lp, vp, i32, vp, vp, vp, vp, sz, vp]
    L.svdp_dense_ffn.argtypes = [lp, vp, i32, vp, vp, sz, vp]
    L.svdp_ffn_step.argtypes = [lp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
    L.svdp_ffn_step_static.argtypes = [lp, vp, i32, vp, vp, vp, vp, vp]
    L.svdp_ffn_step_static.restype = ctypes.c_int
    L.svdp_stack_glue.argtypes = [vp, vp, vp, i32, i32, ctypes.c_float, vp, vp]
    L.svdp_active_rows.argtypes = [lp, vp, i32, vp, vp, vp, sz, vp]
    L.svdp_active_rows.restype = ctypes.c_int
    for n in ("svdp_predict", "svdp_compact", "svdp_sparse_ffn", "svdp_dense_ffn", "svdp_ffn_step",
              "svdp_stack_glue"):
        getattr(L, n).restype = ctypes.c_int
    L.svdp_status_string.argtypes = [ctypes.c_int]
    L.svdp_status_string.restype = ctypes.c_char_p
    L.svdp_version.argtypes = []
    L.svdp_version.restype = ctypes.c_char_p
    L.svdp_calib_workspace_bytes.argtypes = [i32, i32, i32]
    L.svdp_calib_workspace_bytes.restype = ctypes.c_size_t
    L.svdp_calib_need.argtypes = [ctypes.c_double, i32, i32]
    L.svdp_calib_need.restype = ctypes.c_int64
    L.svdp_calib_bias.argtypes = [vp, vp, i32, i32, i32, ctypes.c_int64, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.svdp_calib_bias.restype = ctypes.c_int
    L.svdp_calib_stats_workspace_bytes.argtypes = [lp, i32]
    L.svdp_calib_stats_workspace_bytes.restype = ctypes.c_size_t
    L.svdp_calib_stats.argtypes = [lp, vp, i32, vp, vp, vp, ctypes.c_size_t, vp]
    L.svdp_calib_stats.restype = ctypes.c_int
    L.svdp_whiten_workspace_bytes.argtypes = [i32, i32, i32, i32]
    L.svdp_whiten_workspace_bytes.restype = ctypes.c_size_t
    L.svdp_whiten_factors.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, ctypes.POINTER(ctypes.c_float),
                                      ctypes.POINTER(ctypes.c_int32), vp, ctypes.c_size_t, vp]
    L.svdp_whiten_factors.restype = ctypes.c_int
    L.svdp_ffn_step_glued.argtypes = [lp, vp, vp, vp, ctypes.c_float, vp, i32, vp, vp, vp, vp, vp, sz, vp]
    L.svdp_ffn_step_glued.restype = ctypes.c_int
    _lib = L
    return L


def _check(st: int, what: str) -> None:
    if st != 0:
        raise SvdpError(f"{what}: {lib().svdp_status_string(st).decode()} (status {st})")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not (t.is_cuda and t.is_contiguous()):
        raise SvdpError("expected a contiguous device tensor")
    return t.data_ptr()


def to_device(a: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """Storage array from ``synth`` (float32, or uint16 bf16 bits) -> device tensor."""
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


class DeviceLayer:
    """Device-resident layer: owns the tensors and the C struct that points at them."""

    def __init__(self, P, Q, b, W_gate, W_up, W_downT, flags: int = 0):
        self.tensors = dict(P=P, Q=Q, b=b, W_gate=W_gate, W_up=W_up, W_downT=W_downT)
        wd = W_gate.dtype
        if wd not in (torch.float32, torch.bfloat16):
            raise SvdpError(f"unsupported weight dtype {wd}")
        for k, t in self.tensors.items():
            if not (t.is_cuda and t.is_contiguous()):
                raise SvdpError(f"{k}: expected a contiguous device tensor")
            if k != "b" and t.dtype != wd:
                raise SvdpError(f"{k}: dtype {t.dtype} differs from W_gate's {wd}")
        if b.dtype != torch.float32:
            raise SvdpError("b must be float32")
        self.D, self.d = W_gate.shape
        self.r = P.shape[1]
        assert P.shape == (self.d, self.r) and Q.shape == (self.D, self.r) and b.shape == (self.D,)
        assert W_up.shape == (self.D, self.d) and W_downT.shape == (self.D, self.d)
        self.dtype = wd
        self.c = svdp_layer(self.d, self.D, self.r, SVDP_BF16 if wd == torch.bfloat16 else SVDP_F32,
                            P.data_ptr(), Q.data_ptr(), b.data_ptr(), W_gate.data_ptr(), W_up.data_ptr(),
                            W_downT.data_ptr(), flags)
        self._ws = {}

    @classmethod
    def from_synth(cls, layer, flags: int = 0, device="cuda") -> "DeviceLayer":
        dt = layer.spec.dtype
        g = lambda name: to_device(getattr(layer, name), dt, device)
        return cls(g("P"), g("Q"), torch.from_numpy(layer.b).to(device), g("W_gate"), g("W_up"), g("W_downT"), flags)

    def clone(self) -> "DeviceLayer":
        """A copy at fresh device addresses (used to defeat cache residency when timing)."""
        t = {k: v.clone() for k, v in self.tensors.items()}
        return DeviceLayer(t["P"], t["Q"], t["b"], t["W_gate"], t["W_up"], t["W_downT"], self.c.flags)

    def with_flags(self, flags: int) -> "DeviceLayer":
        """The same tensors under other SVDP_FLAG_* bits (pipeline variant, engine selection)."""
        t = self.tensors
        return DeviceLayer(t["P"], t["Q"], t["b"], t["W_gate"], t["W_up"], t["W_downT"], flags)

    def workspace(self, max_batch: int = 1) -> torch.Tensor:
        key = int(max_batch)
        if key not in self._ws:
            n = workspace_bytes(self, max_batch)
            self._ws[key] = torch.empty(n, dtype=torch.uint8, device=self.tensors["P"].device)
        return self._ws[key]


def workspace_bytes(layer: DeviceLayer, max_batch: int) -> int:
    n = lib().svdp_workspace_bytes(ctypes.byref(layer.c), int(max_batch))
    if n == 0:
        raise SvdpError("svdp_workspace_bytes: unsupported layer or batch")
    return int(n)


def _x2(layer: DeviceLayer, x: torch.Tensor) -> Tuple[torch.Tensor, int]:
    if x.dim() == 1:
        x = x[None, :]
    if x.dtype != layer.dtype or x.shape[1] != layer.d:
        raise SvdpError(f"x: expected [B][{layer.d}] of {layer.dtype}, got {tuple(x.shape)} {x.dtype}")
    return x, x.shape[0]


def predict(layer: DeviceLayer, x: torch.Tensor, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    x, B = _x2(layer, x)
    ws = layer.workspace(B) if ws is None else ws
    s = torch.empty((B, layer.D), dtype=torch.float32, device=x.device)
    _check(lib().svdp_predict(ctypes.byref(layer.c), _ptr(x), B, _ptr(s), _ptr(ws), ws.numel(), _stream()),
           "svdp_predict")
    return s


def compact(s: torch.Tensor):
    """Returns (mask int64 [D/64], idx int32 [D], nnz int32 [1]) device tensors."""
    if s.dim() == 1:
        s = s[None, :]
    B, D = s.shape
    mask = torch.empty(max(D // 64, 1), dtype=torch.int64, device=s.device)
    idx = torch.full((D,), -1, dtype=torch.int32, device=s.device)
    nnz = torch.empty(1, dtype=torch.int32, device=s.device)
    _check(lib().svdp_compact(_ptr(s), B, D, _ptr(mask), _ptr(idx), _ptr(nnz), None, 0, _stream()), "svdp_compact")
    return mask, idx, nnz


def sparse_ffn(layer: DeviceLayer, x: torch.Tensor, idx: torch.Tensor, nnz: torch.Tensor,
               ws: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    x, B = _x2(layer, x)
    ws = layer.workspace(B) if ws is None else ws
    y = torch.empty((B, layer.d), dtype=torch.float32, device=x.device) if out is None else out
    _check(lib().svdp_sparse_ffn(ctypes.byref(layer.c), _ptr(x), B, _ptr(idx), _ptr(nnz), _ptr(y), _ptr(ws),
                                 ws.numel(), _stream()), "svdp_sparse_ffn")
    return y


def dense_ffn(layer: DeviceLayer, x: torch.Tensor, ws: Optional[torch.Tensor] = None,
              out: Optional[torch.Tensor] = None) -> torch.Tensor:
    x, B = _x2(layer, x)
    ws = layer.workspace(B) if ws is None else ws
    y = torch.empty((B, layer.d), dtype=torch.float32, device=x.device) if out is None else out
    _check(lib().svdp_dense_ffn(ctypes.byref(layer.c), _ptr(x), B, _ptr(y), _ptr(ws), ws.numel(), _stream()),
           "svdp_dense_ffn")
    return y


def ffn_step(layer: DeviceLayer, x: torch.Tensor, ws: Optional[torch.Tensor] = None,
             out: Optional[torch.Tensor] = None, mask: Optional[torch.Tensor] = None,
             idx: Optional[torch.Tensor] = None, nnz: Optional[torch.Tensor] = None) -> torch.Tensor:
    x, B = _x2(layer, x)
    ws = layer.workspace(B) if ws is None else ws
    y = torch.empty((B, layer.d), dtype=torch.float32, device=x.device) if out is None else out
    _check(lib().svdp_ffn_step(ctypes.byref(layer.c), _ptr(x), B, _ptr(y), _ptr(mask), _ptr(idx), _ptr(nnz),
                               _ptr(ws), ws.numel(), _stream()), "svdp_ffn_step")
    return y


def ffn_step_static(layer: DeviceLayer, x: torch.Tensor, out: Optional[torch.Tensor] = None,
                    mask: Optional[torch.Tensor] = None, idx: Optional[torch.Tensor] = None,
                    nnz: Optional[torch.Tensor] = None) -> torch.Tensor:
    """svdp_ffn_step with the scratch taken from the library's own static device array (no workspace argument)."""
    x, B = _x2(layer, x)
    y = torch.empty((B, layer.d), dtype=torch.float32, device=x.device) if out is None else out
    _check(lib().svdp_ffn_step_static(ctypes.byref(layer.c), _ptr(x), B, _ptr(y), _ptr(mask), _ptr(idx), _ptr(nnz),
                                      _stream()), "svdp_ffn_step_static")
    return y


def ffn_step_glued(layer: DeviceLayer, x_prev: torch.Tensor, y_prev: torch.Tensor, shift: torch.Tensor,
                   x_out: torch.Tensor, eps: float = 1e-6, ws: Optional[torch.Tensor] = None,
                   out: Optional[torch.Tensor] = None, mask: Optional[torch.Tensor] = None,
                   idx: Optional[torch.Tensor] = None, nnz: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The step on x = RMSNorm(x_prev + y_prev) + shift (written to x_out), glue and step in the same launches."""
    x_prev, B = _x2(layer, x_prev)
    assert y_prev.numel() == B * layer.d and x_out.numel() == B * layer.d and shift.numel() == layer.d
    assert x_out.dtype == x_prev.dtype and y_prev.dtype == torch.float32 and shift.dtype == torch.float32
    ws = layer.workspace(B) if ws is None else ws
    y = torch.empty((B, layer.d), dtype=torch.float32, device=x_prev.device) if out is None else out
    _check(lib().svdp_ffn_step_glued(ctypes.byref(layer.c), _ptr(x_prev), _ptr(y_prev), _ptr(shift), float(eps),
                                     _ptr(x_out), B, _ptr(y), _ptr(mask), _ptr(idx), _ptr(nnz), _ptr(ws), ws.numel(),
                                     _stream()), "svdp_ffn_step_glued")
    return y


def active_rows(layer: DeviceLayer, x: torch.Tensor, mask: torch.Tensor, ws: Optional[torch.Tensor] = None,
                out: Optional[torch.Tensor] = None, first_kernel_only: bool = False) -> Optional[torch.Tensor]:
    """The sparse FFN from given mask words (no predictor).  With first_kernel_only the dominant kernel is
    enqueued alone (its results stay in the workspace, nothing is returned): for timing it by itself."""
    x, B = _x2(layer, x)
    ws = layer.workspace(B) if ws is None else ws
    y = None
    if not first_kernel_only:
        y = torch.empty((B, layer.d), dtype=torch.float32, device=x.device) if out is None else out
    _check(lib().svdp_active_rows(ctypes.byref(layer.c), _ptr(x), B, _ptr(mask), _ptr(y), _ptr(ws), ws.numel(),
                                  _stream()), "svdp_active_rows")
    return y


def stack_glue(x: torch.Tensor, y: torch.Tensor, shift: torch.Tensor, eps: float = 1e-6,
               out: Optional[torch.Tensor] = None) -> torch.Tensor:
    d = x.numel()
    out = torch.empty_like(x) if out is None else out
    dt = SVDP_BF16 if x.dtype == torch.bfloat16 else SVDP_F32
    _check(lib().svdp_stack_glue(_ptr(x), _ptr(y), _ptr(shift), d, dt, float(eps), _ptr(out), _stream()),
           "svdp_stack_glue")
    return out


def calib_stats(layer: "DeviceLayer", X: torch.Tensor):
    """Damage weights and proxy scores of T calibration tokens X [T][d]: two device tensors [D][T] fp32."""
    assert X.dim() == 2 and X.is_cuda and X.is_contiguous()
    T = X.shape[0]
    D = layer.c.D
    nbytes = lib().svdp_calib_stats_workspace_bytes(ctypes.byref(layer.c), T)
    if nbytes == 0:
        raise SvdpError("svdp_calib_stats: unsupported layer (bf16 storage only) or T < 1")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=X.device)
    w = torch.empty((D, T), dtype=torch.float32, device=X.device)
    s = torch.empty((D, T), dtype=torch.float32, device=X.device)
    _check(lib().svdp_calib_stats(ctypes.byref(layer.c), _ptr(X), T, _ptr(w), _ptr(s), _ptr(ws), ws.numel(),
                                  _stream()), "svdp_calib_stats")
    return w, s


def calib_need(sparsity: float, D: int, T: int) -> int:
    """Number of (neuron, sample) pairs Alg. 2's loop has to reach for a sparsity level (computed by the library)."""
    n = int(lib().svdp_calib_need(float(sparsity), int(D), int(T)))
    if n < 0:
        raise SvdpError(f"svdp_calib_need: invalid arguments sparsity={sparsity} D={D} T={T}")
    return n


def calib_bias(w: torch.Tensor, s: torch.Tensor, eta: int, need: int, want_kendall: bool = False):
    """Greedy bias calibration on device tensors w, s of shape [D][T] (fp32).
    Returns (b [D] fp32, k [D] int32, steps [1] int32, kendall [D] fp32 or None), all on the device."""
    assert w.shape == s.shape and w.dim() == 2 and w.dtype == torch.float32 and s.dtype == torch.float32
    D, T = w.shape
    nbytes = lib().svdp_calib_workspace_bytes(D, T, int(eta))
    if nbytes == 0:
        raise SvdpError(f"svdp_calib_bias: unsupported sizes D={D} T={T} eta={eta}")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    b = torch.empty(D, dtype=torch.float32, device=w.device)
    k = torch.empty(D, dtype=torch.int32, device=w.device)
    steps = torch.empty(1, dtype=torch.int32, device=w.device)
    kend = torch.empty(D, dtype=torch.float32, device=w.device) if want_kendall else None
    _check(lib().svdp_calib_bias(_ptr(w), _ptr(s), D, T, int(eta), int(need), _ptr(b), _ptr(k), _ptr(steps),
                                 _ptr(kend), _ptr(ws), ws.numel(), _stream()), "svdp_calib_bias")
    return b, k, steps, kend


def whiten_factors(W_gate: torch.Tensor, X: torch.Tensor, r: int):
    """Predictor factors with data whitening (Alg. 1) for W_gate [D][d] and calibration tokens X [T][d] (device,
    both float32 or both bfloat16).  Returns (P [d][r] fp32, Q [D][r] fp32, sigma [r] numpy, sweeps (2 ints))."""
    assert W_gate.dim() == 2 and X.dim() == 2 and W_gate.dtype == X.dtype and W_gate.shape[1] == X.shape[1]
    assert W_gate.is_cuda and X.is_cuda and W_gate.is_contiguous() and X.is_contiguous()
    D, d = W_gate.shape
    T = X.shape[0]
    dt = SVDP_BF16 if W_gate.dtype == torch.bfloat16 else SVDP_F32
    nbytes = lib().svdp_whiten_workspace_bytes(d, D, T, int(r))
    if nbytes == 0:
        raise SvdpError(f"svdp_whiten_factors: unsupported sizes d={d} D={D} T={T} r={r}")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=X.device)
    P = torch.empty((d, r), dtype=torch.float32, device=X.device)
    Q = torch.empty((D, r), dtype=torch.float32, device=X.device)
    sigma = (ctypes.c_float * int(r))()
    sweeps = (ctypes.c_int32 * 2)()
    _check(lib().svdp_whiten_factors(_ptr(W_gate), _ptr(X), d, D, T, int(r), dt, _ptr(P), _ptr(Q), sigma, sweeps,
                                     _ptr(ws), ws.numel(), _stream()), "svdp_whiten_factors")
    return P, Q, np.array(sigma[:], dtype=np.float32), (int(sweeps[0]), int(sweeps[1]))


def version() -> str:
    return lib().svdp_version().decode()
