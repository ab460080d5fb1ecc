"""A stack of FFN layers with the benchmark's glue between them.

Not part of the paper's method: the stacked benchmark carries the residual as
x + y with RMS normalisation and re-centres it on the next layer's token
direction, x_{l+1} = RMSNorm(x_l + y_l) + 2 u_{l+1} (no gain, eps = 1e-6), rounded
to the activation dtype.  The last layer's output is normalised with a zero
shift.  Every call goes through the C-ABI library; nothing here computes.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from . import binding, synth


def stack_specs(n_layers: int, base: str = "7b", seed0: int = 4000, lo: float = 0.80, hi: float = 0.95, **over):
    """Per-layer specs: own seed, target sparsity drawn uniformly from [lo, hi]."""
    rng = np.random.default_rng([seed0, 99])
    targets = rng.uniform(lo, hi, size=n_layers)
    return [synth.workload(base, seed=seed0 + l, sparsity=float(round(targets[l], 4)), **over) for l in range(n_layers)]


class FFNStack:
    """Device-resident stack; `step` runs every layer of one decode step on the current stream."""

    def __init__(self, layers: List[binding.DeviceLayer], shifts: List[torch.Tensor], dense: bool = False,
                 fused_glue: bool = True):
        assert len(shifts) == len(layers)
        self.layers, self.shifts, self.dense = layers, shifts, dense
        # sparse stack: the glue between two layers runs inside the next layer's first kernel
        # (svdp_ffn_step_glued) instead of as a launch of its own; same bits either way
        self.fused_glue = fused_glue
        dev = layers[0].tensors["P"].device
        self.d, self.dtype = layers[0].d, layers[0].dtype
        self.ws = layers[0].workspace(1)
        self.x = [torch.zeros(self.d, dtype=self.dtype, device=dev) for _ in range(len(layers) + 1)]
        self.y = torch.zeros((1, self.d), dtype=torch.float32, device=dev)
        self.nnz = torch.zeros((len(layers), 1), dtype=torch.int32, device=dev)

    @classmethod
    def from_synth(cls, synth_layers, dense: bool = False, fused_glue: bool = True):
        dev_layers = [binding.DeviceLayer.from_synth(L) for L in synth_layers]
        shifts = [torch.from_numpy((2.0 * L.u).astype(np.float32)).cuda() for L in synth_layers[1:]]
        shifts.append(torch.zeros(synth_layers[0].spec.d, dtype=torch.float32, device="cuda"))
        return cls(dev_layers, shifts, dense, fused_glue)

    def as_dense(self) -> "FFNStack":
        return FFNStack(self.layers, self.shifts, dense=True)

    def with_glue_launches(self) -> "FFNStack":
        return FFNStack(self.layers, self.shifts, dense=self.dense, fused_glue=False)

    def step(self, x0: torch.Tensor, nnz: Optional[torch.Tensor] = None) -> torch.Tensor:
        """x0: [d] in the activation dtype.  nnz: optional int32 [n_layers][1] receiving the
        list length of every layer.  Returns the stack output (a persistent buffer)."""
        nnz = self.nnz if nnz is None else nnz
        self.x[0].copy_(x0)
        fused = self.fused_glue and not self.dense
        for l, layer in enumerate(self.layers):
            if self.dense:
                binding.dense_ffn(layer, self.x[l], ws=self.ws, out=self.y)
            elif fused and l > 0:
                binding.ffn_step_glued(layer, self.x[l - 1], self.y, self.shifts[l - 1], self.x[l], ws=self.ws,
                                       out=self.y, nnz=nnz[l])
            else:
                binding.ffn_step(layer, self.x[l], ws=self.ws, out=self.y, nnz=nnz[l])
            if not fused or l == len(self.layers) - 1:
                binding.stack_glue(self.x[l], self.y, self.shifts[l], out=self.x[l + 1])
        return self.x[-1]
