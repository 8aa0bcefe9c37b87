"""Seeded random operating points through the C ABI against the float64 oracle: chunk size, budget, worker
count, tensor shapes (ragged chunk grids, order-1 tensors, shapes the s = 32 tile kernels cannot take), dtypes per
tensor, update rule and aggregate are drawn together, so that the kernel selection logic (payload access modes,
streaming, dtype groups, fallbacks) is exercised in combinations the hand-picked cases do not list."""
import os

import numpy as np
import pytest
import torch

from paper_2411_19870_amd import binding as B
from paper_2411_19870_amd import synth
from tests import compare as C
from tests.gpu_harness import Case

pytestmark = pytest.mark.gpu

PHI = {"sign": B.DEMO_PHI_SIGN, "identity": B.DEMO_PHI_IDENTITY}
AGG = {"sum": B.DEMO_AGG_SUM, "mean": B.DEMO_AGG_MEAN, "count": B.DEMO_AGG_COUNT}


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available()
    c = B.Context()
    yield c
    c.close()


def draw(seed):
    rng = np.random.default_rng(1000 + seed)
    s = int(rng.choice([32, 64, 128]))
    k = int(rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 20, 32, 33, 48, 64, 65, 100, 256]))
    vectors = rng.random() < 0.7
    if vectors or k > 64 and rng.random() < 0.5:
        k = min(k, s)                               # order-1 tensors: k <= s
    vectors = vectors and k <= s
    # worker counts around the limits of the register-resident payload (W k = 512 / 2048 / 4096) and beyond
    W = int(rng.choice([1, 2, 3, 7, 8, 16, 17, 31, 64, 65, 100, 128, 200, 255, 700]))
    if W * k > 20000:
        W = max(1, 20000 // k)
    specs = []
    for i in range(int(rng.integers(1, 5))):
        unit = s if (s != 32 or rng.random() < 0.3) else 64
        specs.append(synth.TensorSpec(f"t{i}", unit * int(rng.integers(1, 4)), unit * int(rng.integers(1, 4))))
    if vectors:
        specs.append(synth.TensorSpec("v", s * int(rng.integers(1, 5)), 0))
    dts = [(bool(rng.integers(0, 2)), bool(rng.integers(0, 2))) for _ in specs]
    if rng.random() < 0.5:                          # one dtype for the whole list, as a training run has it
        dts = [dts[0]] * len(specs)
    phi = str(rng.choice(["sign", "sign", "identity"]))
    agg = str(rng.choice(["sum", "sum", "mean", "count"]))
    if W > 255:                                     # the count aggregate is defined up to 255 workers; past about
        agg, phi = "sum", "sign"                    # 1000 workers the fixed-point quantum only suits the sign
    return dict(s=s, k=k, W=W, specs=specs, dts=dts, phi=phi, agg=agg, wd=float(rng.choice([0.0, 0.1])),
                alpha=float(rng.choice([1.0, 1.0, 0.2, 0.0])), beta=float(rng.choice([0.999, 0.9])),
                gscale=float(rng.choice([1.0, 1.0, 0.1])), grad=str(rng.choice(["gauss", "gauss", "student"])),
                unaligned=bool(rng.random() < 0.2), seed=seed)


# DEMO_RANDOM_CASES=N draws more of them
@pytest.mark.parametrize("seed", range(int(os.environ.get("DEMO_RANDOM_CASES", "60"))))
def test_random_operating_point(ctx, seed):
    cfg = draw(seed)
    s, k, W, specs = cfg["s"], cfg["k"], cfg["W"], cfg["specs"]
    print({key: (val if key != "specs" else [sp.shape for sp in val]) for key, val in cfg.items()}, flush=True)
    ctx.demo_set_variant(0 if seed % 3 == 2 else 1)   # every third point on the generic kernels
    case = Case(specs, s, k, W=W, seed=300 + seed, grad=cfg["grad"])
    if cfg["unaligned"]:    # payload arrays as views one element into a padded buffer: 4-byte alignment only
        for ti in range(len(specs)):
            bi = torch.zeros(case.idx[ti].numel() + 4, dtype=torch.int32, device=case.idx[ti].device)
            bv = torch.zeros(case.val[ti].numel() + 4, dtype=torch.float32, device=case.val[ti].device)
            case.idx[ti] = bi[1:1 + case.idx[ti].numel()].view(case.idx[ti].shape)
            case.val[ti] = bv[1:1 + case.val[ti].numel()].view(case.val[ti].shape)
    for ti, (gb, xb) in enumerate(cfg["dts"]):
        if gb:
            case.g[ti] = case.g[ti].to(torch.bfloat16)
        if xb:
            case.x[ti] = case.x[ti].to(torch.bfloat16)
    case.args = B.TensorList([B.TensorArgs(g, m, x, i, v) for g, m, x, i, v in zip(case.g, case.m, case.x, case.idx, case.val)])
    lr = 1e-3
    hp = B.demo_hparams_default(beta=cfg["beta"], lr=lr, weight_decay=cfg["wd"], alpha=cfg["alpha"],
                                grad_scale=cfg["gscale"], phi=PHI[cfg["phi"]], aggregate=AGG[cfg["agg"]])
    before = case.snapshot()
    ctx.demo_encode_ex(case.args, hp, s, k)
    torch.cuda.synchronize()
    after = case.snapshot()
    for ti in range(len(specs)):
        C.check_encode(before["m"][ti], before["g"][ti], cfg["beta"], s, k, after["idx"][ti][0], after["val"][ti][0],
                       after["m"][ti], alpha32=cfg["alpha"], grad_scale32=cfg["gscale"])
    # exact uniform index sets while the draw stays small, the keyed bijection beyond
    heavy = W * max(sp.nchunks(s) * sp.chunk_elems(s) for sp in specs) > 4_000_000
    case.fill_payloads(exact=not heavy)
    before = case.snapshot()
    ctx.demo_decode_ex(case.args, W, hp, s, k)
    torch.cuda.synchronize()
    after = case.snapshot()
    for ti in range(len(specs)):
        pd = "bf16" if case.x[ti].dtype == torch.bfloat16 else "f32"
        C.check_decode(before["x"][ti], before["idx"][ti][:W], before["val"][ti][:W], lr, cfg["wd"], s, pd,
                       after["x"][ti], phi=cfg["phi"], aggregate_mode=cfg["agg"])
    ctx.demo_set_variant(1)
