"""Parity at the benchmark's full size and launch configuration: the 1B-like tensor
set (bf16 gradients, fp32 momentum, bf16 parameters, s = 64, k = 32, W = 64), checked
on sampled chunks the oracle computes one by one, plus properties that hold at any size."""
import numpy as np
import pytest
import torch

from paper_2411_19870_amd import binding as B
from paper_2411_19870_amd import synth
from tests import compare as C

pytestmark = pytest.mark.gpu

S, K, W = 64, 32, 64
BETA, LR = 0.999, 1e-3
DEV = "cuda:0"


def block(t: torch.Tensor, sp, c: int) -> np.ndarray:
    if sp.cols == 0:
        return t[c * S:(c + 1) * S].to("cpu", torch.float64).numpy()
    cc = sp.cols // S
    k0, k1 = divmod(c, cc)
    return t[k0 * S:(k0 + 1) * S, k1 * S:(k1 + 1) * S].to("cpu", torch.float64).numpy()


@pytest.fixture(scope="module")
def big():
    assert torch.cuda.is_available()
    specs = synth.tensor_set("1b")
    tensors = []
    for ti, sp in enumerate(specs):
        g = synth.gaussian(sp, 1e-2, 0, ti, 0, "grad", dtype=torch.bfloat16, device=DEV)
        m = synth.gaussian(sp, 1e-3, 0, ti, 0, "mom", device=DEV)
        x = synth.gaussian(sp, 0.02, 0, ti, 0, "param", dtype=torch.bfloat16, device=DEV)
        idx, val = synth.payload_fast(sp, S, K, W, 1e-3, 0, ti, device=DEV)
        tensors.append(B.TensorArgs(g, m, x, idx, val))
    ctx = B.Context()
    yield specs, tensors, B.TensorList(tensors), ctx
    ctx.close()


def sample_chunks(specs, per_tensor, seed):
    rng = np.random.default_rng(seed)
    out = []
    for ti, sp in enumerate(specs):
        n = sp.nchunks(S)
        picks = {0, n - 1} | set(rng.integers(0, n, size=per_tensor).tolist())
        out += [(ti, c) for c in sorted(picks)]
    return out


def test_full_size_encode_then_decode(big):
    specs, tensors, tl, ctx = big
    picks = sample_chunks(specs, 2, 0)
    pre = {(ti, c): (block(tensors[ti].mom, specs[ti], c), block(tensors[ti].grad, specs[ti], c)) for ti, c in picks}
    energy_mid = [float((BETA * t.mom.double() + t.grad.double()).pow(2).sum()) for t in tensors[:8]]
    ctx.demo_encode(tl, BETA, S, K)
    torch.cuda.synchronize()
    swaps = 0
    worst_v = worst_m = 0.0
    for ti, c in picks:
        m0, g0 = pre[(ti, c)]
        st = C.check_encode(m0, g0, BETA, S, K, tensors[ti].idx[0, c].cpu().numpy(),
                            tensors[ti].val[0, c].cpu().numpy(), block(tensors[ti].mom, specs[ti], c))
        swaps += st["tie_swaps"]
        worst_v, worst_m = max(worst_v, st["max_rel_err_val"]), max(worst_m, st["max_rel_err_mom"])
    print(f"encode: {len(picks)} sampled chunks, tie swaps {swaps}, worst rel err val {worst_v:.2e} mom {worst_m:.2e}")
    # any-size properties: indices in range and distinct per chunk; energy split
    # ||beta m + g||^2 = ||val||^2 + ||m_new||^2 (orthonormal transform)
    for ti, t in enumerate(tensors):
        M = specs[ti].chunk_elems(S)
        i0 = t.idx[0]
        assert int(i0.min()) >= 0 and int(i0.max()) < M
        srt = i0.sort(dim=1).values
        assert bool((srt[:, 1:] != srt[:, :-1]).all())
    for ti, t in enumerate(tensors[:8]):
        e_after = float(t.val[0].double().pow(2).sum() + t.mom.double().pow(2).sum())
        assert abs(e_after - energy_mid[ti]) <= 1e-5 * energy_mid[ti]

    # ---- decode of W = 64 payloads (slot 0 is the encode output above)
    pre_x = {(ti, c): block(tensors[ti].param, specs[ti], c) for ti, c in picks}
    ctx.demo_decode(tl, W, LR, 0.0, S, K)
    torch.cuda.synchronize()
    in_band = 0
    for ti, c in picks:
        sp = specs[ti]
        idx = tensors[ti].idx[:, c:c + 1].cpu().numpy()
        val = tensors[ti].val[:, c:c + 1].cpu().numpy()
        st = C.check_decode(pre_x[(ti, c)], idx, val, LR, 0.0, S, "bf16", block(tensors[ti].param, sp, c).astype(np.float32))
        in_band += st["in_band"]
    print(f"decode: {len(picks)} sampled chunks, parameters inside the sign-noise band: {in_band}")


# ---- stress sweep at full size: heavy-tailed bf16 gradients (exact magnitude ties), momentum carried over
#      10 steps of encode + decode of the worker's own payload, sampled chunks checked every step ---------------
def _block(t: torch.Tensor, sp, c: int, s: int) -> np.ndarray:
    if sp.cols == 0:
        return t[c * s:(c + 1) * s].to("cpu", torch.float64).numpy()
    k0, k1 = divmod(c, sp.cols // s)
    return t[k0 * s:(k0 + 1) * s, k1 * s:(k1 + 1) * s].to("cpu", torch.float64).numpy()


@pytest.mark.parametrize("s,k", [(32, 8), (128, 32), (64, 1)])
def test_full_size_ten_carried_steps(s, k):
    specs = synth.tensor_set("1b")
    tensors = []
    for ti, sp in enumerate(specs):
        g = torch.empty(sp.shape, dtype=torch.bfloat16, device=DEV)
        m = torch.zeros(sp.shape, dtype=torch.float32, device=DEV)
        x = synth.gaussian(sp, 0.02, 1, ti, 0, "param", dtype=torch.bfloat16, device=DEV)
        nch = sp.nchunks(s)
        tensors.append(B.TensorArgs(g, m, x, torch.zeros((1, nch, k), dtype=torch.int32, device=DEV),
                                    torch.zeros((1, nch, k), dtype=torch.float32, device=DEV)))
    tl = B.TensorList(tensors)
    ctx = B.Context()
    rng = np.random.default_rng(s)
    swaps = in_band = checked = 0
    for step in range(10):
        for ti, sp in enumerate(specs):
            tensors[ti].grad.copy_(synth.student_t3(sp, 1e-2, 1, ti, step, "grad", dtype=torch.bfloat16, device=DEV))
        picks = [(ti, int(c)) for ti, sp in enumerate(specs) if (ti + step) % 5 == 0
                 for c in {0, sp.nchunks(s) - 1, int(rng.integers(0, sp.nchunks(s)))}]
        pre = {(ti, c): (_block(tensors[ti].mom, specs[ti], c, s), _block(tensors[ti].grad, specs[ti], c, s),
                         _block(tensors[ti].param, specs[ti], c, s)) for ti, c in picks}
        ctx.demo_step(tl, BETA, LR, 0.0, s, k)
        torch.cuda.synchronize()
        for ti, c in picks:
            m0, g0, x0 = pre[(ti, c)]
            idx = tensors[ti].idx[0, c].cpu().numpy()
            val = tensors[ti].val[0, c].cpu().numpy()
            st = C.check_encode(m0, g0, BETA, s, k, idx, val, _block(tensors[ti].mom, specs[ti], c, s))
            swaps += st["tie_swaps"]
            sd = C.check_decode(x0, idx[None, None], val[None, None], LR, 0.0, s, "bf16",
                                _block(tensors[ti].param, specs[ti], c, s).astype(np.float32))
            in_band += sd["in_band"]
            checked += 1
    ctx.close()
    print(f"s={s} k={k}: {checked} chunk-steps checked, tie swaps {swaps}, parameters inside the sign-noise band {in_band}")
