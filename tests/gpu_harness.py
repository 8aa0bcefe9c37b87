"""Shared plumbing of the GPU parity tests: build device tensors for a tensor
set, call the HIP path through the C ABI, bring results back as numpy."""
from __future__ import annotations

import numpy as np
import torch

from paper_2411_19870_amd import binding as B
from paper_2411_19870_amd import synth

DEV = "cuda:0"


def np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


class Case:
    """Device state of one tensor set: gradients, momentum, parameters, payload buffers."""

    def __init__(self, specs, s, k, W=1, grad_dtype=torch.float32, param_dtype=torch.float32, seed=0,
                 grad="gauss", grad_std=1e-2, mom_std=1e-3, param_std=0.02):
        self.specs, self.s, self.k, self.W = list(specs), s, k, W
        self.seed, self.grad_kind, self.grad_std, self.grad_dtype = seed, grad, grad_std, grad_dtype
        self.g, self.m, self.x, self.idx, self.val = [], [], [], [], []
        for ti, sp in enumerate(self.specs):
            self.g.append(self._draw_grad(sp, ti, 0))
            if mom_std == 0:
                self.m.append(torch.zeros(sp.shape, dtype=torch.float32, device=DEV))
            else:
                self.m.append(synth.gaussian(sp, mom_std, seed, ti, 0, "mom").to(DEV))
            self.x.append(synth.gaussian(sp, param_std, seed, ti, 0, "param", dtype=param_dtype).to(DEV))
            nch = sp.nchunks(s)
            self.idx.append(torch.zeros((W, nch, k), dtype=torch.int32, device=DEV))
            self.val.append(torch.zeros((W, nch, k), dtype=torch.float32, device=DEV))
        self.args = B.TensorList([B.TensorArgs(g, m, x, i, v) for g, m, x, i, v in
                                  zip(self.g, self.m, self.x, self.idx, self.val)])

    def _draw_grad(self, sp, ti, step):
        if self.grad_kind == "gauss":
            return synth.gaussian(sp, self.grad_std, self.seed, ti, step, "grad", dtype=self.grad_dtype).to(DEV)
        if self.grad_kind == "student":
            return synth.student_t3(sp, self.grad_std, self.seed, ti, step, "grad", dtype=self.grad_dtype).to(DEV)
        if self.grad_kind == "zero":
            return torch.zeros(sp.shape, dtype=self.grad_dtype, device=DEV)
        raise KeyError(self.grad_kind)

    def new_grads(self, step):
        for ti, sp in enumerate(self.specs):
            self.g[ti].copy_(self._draw_grad(sp, ti, step))

    def fill_payloads(self, val_std=1e-3, exact=True):
        f = synth.payload_exact if exact else synth.payload_fast
        for ti, sp in enumerate(self.specs):
            i, v = f(sp, self.s, self.k, self.W, val_std, self.seed, ti, device="cpu")
            self.idx[ti].copy_(i)
            self.val[ti].copy_(v)

    def snapshot(self):
        return {"g": [np64(t) for t in self.g], "m": [np64(t) for t in self.m], "x": [np64(t) for t in self.x],
                "idx": [t.cpu().numpy().copy() for t in self.idx], "val": [t.cpu().numpy().copy() for t in self.val]}
