"""Tools of the full-size parity tests: which chunks to check, gathering them on the GPU, and
running the float64 oracle on them in a pool of worker processes.

The sample of a tensor holds every chunk of an order-1 tensor and, for an order-2 tensor, its first and
last chunk, the chunks at which a wavefront or workgroup of the persistent kernels hands over to its next
work item (global work items j*n - 1 and j*n for the grid strides n the kernels use), and seeded random
chunks up to the requested fraction.  The worker processes import numpy and the oracle only; they never
touch the GPU.
"""
from __future__ import annotations

import math
import multiprocessing
import os
from concurrent.futures import ProcessPoolExecutor
from typing import Dict, List

import numpy as np
import torch

from tests import compare as C

GRID_STRIDES = (256, 2048)      # workgroups per grid (s = 128) and wavefronts per grid (s = 64, 32) on 256 CUs
ELEMS_PER_JOB = 1 << 21


def pool_size() -> int:
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def _worker_init():
    # one BLAS thread per worker: the pool already uses every core
    try:
        import threadpoolctl
        global _blas_limit
        _blas_limit = threadpoolctl.threadpool_limits(limits=1)
    except Exception:
        pass


def make_pool() -> ProcessPoolExecutor:
    # "spawn": the workers start from a fresh interpreter instead of a copy of a process that holds the GPU
    return ProcessPoolExecutor(max_workers=pool_size(), mp_context=multiprocessing.get_context("spawn"),
                               initializer=_worker_init)


# ---------------------------------------------------------------------------------------------------
# sampling
# ---------------------------------------------------------------------------------------------------
def _handover_items(total: int) -> List[int]:
    out = []
    for n in GRID_STRIDES:
        last = (total - 1) // n
        for j in sorted({1, 2, 3, last}):
            out += [j * n - 1, j * n, j * n + 1]
    return [i for i in out if 0 <= i < total]


def pick_chunks(specs, s: int, frac: float, seed: int) -> Dict[int, np.ndarray]:
    """{tensor index: sorted local chunk ids}."""
    rng = np.random.default_rng(seed)
    picks: Dict[int, set] = {}
    two = [(ti, sp) for ti, sp in enumerate(specs) if sp.cols != 0]
    for ti, sp in enumerate(specs):
        n = sp.nchunks(s)
        if sp.cols == 0:
            picks[ti] = set(range(n))
            continue
        want = min(n, max(2, math.ceil(frac * n)))
        picks[ti] = {0, n - 1} | set(rng.choice(n, size=want, replace=False).tolist())
    # hand-over points, in the numbering of the kernels' work items: chunks in list order (s = 64, 128),
    # 64 x 64 tiles of 2 x 2 chunks in list order (s = 32)
    unit = 64 if s == 32 else s
    first = 0
    offsets = []
    for ti, sp in two:
        offsets.append(first)
        first += (sp.rows // unit) * (sp.cols // unit)
    for item in _handover_items(first):
        j = max(i for i, o in enumerate(offsets) if o <= item)
        ti, sp = two[j]
        local = item - offsets[j]
        if s != 32:
            picks[ti].add(local)
        else:
            r, c = divmod(local, sp.cols // 64)
            cc = sp.cols // 32
            picks[ti] |= {(2 * r + a) * cc + 2 * c + b for a in (0, 1) for b in (0, 1)}
    return {ti: np.array(sorted(v), dtype=np.int64) for ti, v in picks.items()}


# ---------------------------------------------------------------------------------------------------
# gathering on the GPU
# ---------------------------------------------------------------------------------------------------
def gather_blocks(t: torch.Tensor, sp, s: int, chunks: np.ndarray) -> np.ndarray:
    """The chunks `chunks` of tensor t as a numpy array [n, s] or [n, s, s]; float32 stays float32, bfloat16
    comes back as its 16-bit codes (uint16)."""
    ci = torch.as_tensor(chunks, device=t.device)
    if sp.cols == 0:
        b = t.view(sp.rows // s, s)[ci]
    else:
        c1 = sp.cols // s
        b = t.view(sp.rows // s, s, c1, s)[ci // c1, :, ci % c1, :]
    b = b.contiguous()
    if b.dtype == torch.bfloat16:
        return b.view(torch.int16).cpu().numpy().view(np.uint16)
    return b.cpu().numpy()


def to_f64(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:                       # bfloat16 codes
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _stack(blocks: np.ndarray) -> np.ndarray:
    """[n, s] -> vector of n chunks; [n, s, s] -> (n*s) x s matrix whose chunk c is block c."""
    a = to_f64(blocks)
    return a.reshape(-1) if a.ndim == 2 else a.reshape(-1, a.shape[2])


# ---------------------------------------------------------------------------------------------------
# jobs (run in the worker processes)
# ---------------------------------------------------------------------------------------------------
def encode_job(m0, g0, beta, s, k, idx, val, m1, tag, P=None):
    try:
        st = C.check_encode(_stack(m0), _stack(g0), beta, s, k, idx, val, _stack(m1), P=P)
    except AssertionError as e:
        raise AssertionError(f"{tag}: {e}") from None
    return st


def decode_job(x0, idx, val, lr, wd, s, pdt, x1, tag, P=None):
    try:
        st = C.check_decode(_stack(x0), idx, val, lr, wd, s, pdt, _stack(x1).astype(np.float32), P=P)
    except AssertionError as e:
        raise AssertionError(f"{tag}: {e}") from None
    return st


def split(n_chunks: int, chunk_elems: int):
    per = max(1, ELEMS_PER_JOB // chunk_elems)
    return [(a, min(n_chunks, a + per)) for a in range(0, n_chunks, per)]


class Tally:
    """Sums the statistics the jobs return."""

    def __init__(self):
        self.futures = []
        self.stats: Dict[str, float] = {}

    def add(self, fut):
        self.futures.append(fut)

    def drain(self, keep: int = 0):
        while len(self.futures) > keep:
            st = self.futures.pop(0).result()
            for key, v in st.items():
                if key.startswith("max_"):
                    self.stats[key] = max(self.stats.get(key, 0.0), v)
                else:
                    self.stats[key] = self.stats.get(key, 0) + v
        return self.stats
