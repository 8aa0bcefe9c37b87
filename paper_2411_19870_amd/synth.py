"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the HIP path and the CPU oracle with the *same* data and
holds none of the method's arithmetic: it only lists tensor shapes and draws
random numbers.  The shapes stand in for the momentum / gradient tensors of the
300M- and 1B-parameter decoder-only transformers of the paper's experimental
setup (Sec. 3 "Experimental Setup": chunk size s = 64, beta = 0.999), whose
training data and weights are not available here.

Seed rule: every tensor draws from its own generator seeded with
    seed * 1000003 + tensor_index * 101 + step   (+ a fixed salt per role).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import torch

_SALT = {"grad": 0, "mom": 7_000_003, "param": 13_000_007, "pay_idx": 19_000_013, "pay_val": 23_000_029}


@dataclass(frozen=True)
class TensorSpec:
    name: str
    rows: int
    cols: int            # 0 -> 1-D tensor of `rows` elements

    @property
    def shape(self) -> Tuple[int, ...]:
        return (self.rows,) if self.cols == 0 else (self.rows, self.cols)

    @property
    def numel(self) -> int:
        return self.rows if self.cols == 0 else self.rows * self.cols

    def nchunks(self, s: int) -> int:
        return self.rows // s if self.cols == 0 else (self.rows // s) * (self.cols // s)

    def chunk_elems(self, s: int) -> int:
        return s if self.cols == 0 else s * s


def _transformer_set(d: int, layers: int, ffn: int, vocab: int, norm_name: str) -> List[TensorSpec]:
    out = [TensorSpec("embedding", vocab, d)]
    for l in range(layers):
        out += [
            TensorSpec(f"l{l}.wqkv", d, 3 * d),
            TensorSpec(f"l{l}.wo", d, d),
            TensorSpec(f"l{l}.ffn_up", d, ffn),
            TensorSpec(f"l{l}.ffn_down", ffn, d),
            TensorSpec(f"l{l}.{norm_name}1", d, 0),
            TensorSpec(f"l{l}.{norm_name}2", d, 0),
        ]
    return out


def tensor_set(name: str) -> List[TensorSpec]:
    """Named tensor sets.

    "single"  : one 1024 x 1024 matrix
    "300m"    : d=1024, 24 layers, FFN 4096, two LayerNorm vectors per layer, embedding 50304 x 1024
    "1b"      : d=2048, 16 layers, FFN 8192, two RMSNorm vectors per layer, embedding 50304 x 2048
    "tiny"    : a few small tensors with ragged block counts, for element-wise parity tests
    """
    if name == "single":
        return [TensorSpec("w", 1024, 1024)]
    if name == "300m":
        return _transformer_set(1024, 24, 4096, 50304, "ln")
    if name == "1b":
        return _transformer_set(2048, 16, 8192, 50304, "rms")
    if name == "tiny":
        return [TensorSpec("a", 384, 640), TensorSpec("v0", 1152, 0), TensorSpec("b", 128, 128),
                TensorSpec("c", 640, 128), TensorSpec("v1", 128, 0)]
    raise KeyError(name)


def _gen(seed: int, tensor_index: int, step: int, role: str, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000003 + tensor_index * 101 + step + _SALT[role])
    return g


def gaussian(spec: TensorSpec, std: float, seed: int, tensor_index: int, step: int, role: str,
             dtype=torch.float32, device="cpu") -> torch.Tensor:
    g = _gen(seed, tensor_index, step, role, device)
    t = torch.randn(spec.shape, generator=g, device=device, dtype=torch.float32) * std
    return t.to(dtype)


def projection_draws(s: int, step: int) -> torch.Tensor:
    """s x s float32 draws from N(0, 1) seeded with the step number: the raw material of the random
    projection matrix of the paper's ablation (every worker draws the same matrix at a given step).
    Orthonormalising them is the method's business, not this module's."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(step))
    return torch.randn((s, s), generator=g, dtype=torch.float32)


def student_t3(spec: TensorSpec, scale: float, seed: int, tensor_index: int, step: int, role: str,
               dtype=torch.float32, device="cpu") -> torch.Tensor:
    """Student-t with 3 degrees of freedom, times `scale` (heavy tails; rounding
    the result to bfloat16 produces many exactly equal magnitudes)."""
    g = _gen(seed, tensor_index, step, role, device)
    z = torch.randn((4,) + spec.shape, generator=g, device=device, dtype=torch.float32)
    chi2 = (z[1:] * z[1:]).sum(0)
    t = z[0] / torch.sqrt(chi2 / 3.0) * scale
    return t.to(dtype)


def payload_exact(spec: TensorSpec, s: int, k: int, W: int, val_std: float, seed: int, tensor_index: int,
                  device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """W workers' payloads for one tensor: int32 idx [W, nchunks, k], k indices
    uniform without replacement in [0, M) per (worker, chunk), and float32 val
    ~ N(0, val_std^2).  Draws a full random key per slot, so only for small cases."""
    nch, M = spec.nchunks(s), spec.chunk_elems(s)
    gi = _gen(seed, tensor_index, 0, "pay_idx", device)
    gv = _gen(seed, tensor_index, 0, "pay_val", device)
    keys = torch.rand((W, nch, M), generator=gi, device=device)
    idx = keys.topk(k, dim=-1).indices.to(torch.int32)
    val = torch.randn((W, nch, k), generator=gv, device=device, dtype=torch.float32) * val_std
    return idx.contiguous(), val.contiguous()


def payload_fast(spec: TensorSpec, s: int, k: int, W: int, val_std: float, seed: int, tensor_index: int,
                 device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """Same distribution family as `payload_exact` at full size: the k indices of
    a (worker, chunk) are the first k images of a keyed bijection of [0, M)
    (M a power of two), hence distinct; cost is O(W * nchunks * k)."""
    nch, M = spec.nchunks(s), spec.chunk_elems(s)
    bits = M.bit_length() - 1
    assert (1 << bits) == M and k <= M
    gi = _gen(seed, tensor_index, 0, "pay_idx", device)
    gv = _gen(seed, tensor_index, 0, "pay_val", device)
    key = torch.randint(0, 1 << 30, (4, W, nch, 1), generator=gi, device=device, dtype=torch.int64)
    x = torch.arange(k, device=device, dtype=torch.int64).view(1, 1, k).expand(W, nch, k)
    mask = M - 1
    h = max(bits // 2, 1)
    x = (x * (2 * key[0] + 1) + key[1]) & mask
    x = x ^ (x >> h)
    x = (x * (2 * key[2] + 1) + key[3]) & mask
    x = x ^ (x >> h)
    idx = x.to(torch.int32).contiguous()
    val = torch.randn((W, nch, k), generator=gv, device=device, dtype=torch.float32) * val_std
    return idx, val.contiguous()
