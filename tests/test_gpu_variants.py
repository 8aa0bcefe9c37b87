"""GPU parity of the method's other operating points (the _ex entry points): subtraction
coefficient alpha, weighted momentum, identity phi, mean and count-normalised aggregates."""
import numpy as np
import pytest
import torch

from paper_2411_19870_amd import binding as B
from paper_2411_19870_amd import synth
from tests import compare as C
from tests.gpu_harness import Case

pytestmark = pytest.mark.gpu

BETA, LR = 0.9, 1e-3
PHI = {"sign": B.DEMO_PHI_SIGN, "identity": B.DEMO_PHI_IDENTITY}
AGG = {"sum": B.DEMO_AGG_SUM, "mean": B.DEMO_AGG_MEAN, "count": B.DEMO_AGG_COUNT}


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available()
    c = B.Context()
    yield c
    c.close()


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("s,k", [(32, 8), (64, 32), (128, 8)])
@pytest.mark.parametrize("alpha,gscale", [(0.2, 1.0), (0.0, 1.0), (1.0, 1.0 - BETA), (0.5, 0.25)])
@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
def test_encode_alpha_and_weighted_momentum(ctx, variant, s, k, alpha, gscale, gdt):
    ctx.demo_set_variant(variant)
    case = Case(synth.tensor_set("tiny"), s, k, grad_dtype=gdt, seed=31)
    hp = B.demo_hparams_default(beta=BETA, alpha=alpha, grad_scale=gscale)
    before = case.snapshot()
    ctx.demo_encode_ex(case.args, hp, s, k)
    torch.cuda.synchronize()
    after = case.snapshot()
    for ti in range(len(case.specs)):
        st = C.check_encode(before["m"][ti], before["g"][ti], BETA, s, k, after["idx"][ti][0], after["val"][ti][0],
                            after["m"][ti], alpha32=alpha, grad_scale32=gscale)
        assert st["chunks"] == case.specs[ti].nchunks(s)


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("s,k,W", [(32, 8, 4), (64, 32, 8), (64, 8, 1), (128, 32, 3)])
@pytest.mark.parametrize("phi,agg", [("identity", "sum"), ("identity", "mean"), ("sign", "mean"),
                                     ("sign", "count"), ("identity", "count")])
@pytest.mark.parametrize("pdt", [torch.float32, torch.bfloat16])
def test_decode_phi_and_aggregates(ctx, variant, s, k, W, phi, agg, pdt):
    ctx.demo_set_variant(variant)
    case = Case(synth.tensor_set("tiny"), s, k, W=W, param_dtype=pdt, seed=32)
    case.fill_payloads()
    wd = 0.1
    hp = B.demo_hparams_default(lr=LR, weight_decay=wd, phi=PHI[phi], aggregate=AGG[agg])
    before = case.snapshot()
    ctx.demo_decode_ex(case.args, W, hp, s, k)
    torch.cuda.synchronize()
    after = case.snapshot()
    pd = "bf16" if pdt == torch.bfloat16 else "f32"
    for ti in range(len(case.specs)):
        C.check_decode(before["x"][ti], before["idx"][ti][:W], before["val"][ti][:W], LR, wd, s, pd, after["x"][ti],
                       phi=phi, aggregate_mode=agg)


# ---- phi = identity with many workers: the fixed-point aggregate keeps the update within its bound up to the
#      documented worker limit; beyond it the call is refused instead of returning a coarser update ------------
@pytest.mark.parametrize("s,k", [(64, 4), (32, 4), (128, 8)])
@pytest.mark.parametrize("agg", ["sum", "mean"])
def test_identity_phi_at_the_worker_limit(ctx, s, k, agg):
    ctx.demo_set_variant(1)
    W = B.DEMO_MAX_W_IDENTITY
    specs = [synth.TensorSpec("a", 2 * s, 3 * s), synth.TensorSpec("v", 2 * s, 0)]
    case = Case(specs, s, k, W=W, param_dtype=torch.float32, seed=34)
    case.fill_payloads()
    hp = B.demo_hparams_default(lr=LR, phi=B.DEMO_PHI_IDENTITY, aggregate=AGG[agg])
    before = case.snapshot()
    ctx.demo_decode_ex(case.args, W, hp, s, k)
    torch.cuda.synchronize()
    after = case.snapshot()
    worst = 0.0
    for ti in range(len(case.specs)):
        st = C.check_decode(before["x"][ti], before["idx"][ti], before["val"][ti], LR, 0.0, s, "f32", after["x"][ti],
                            phi="identity", aggregate_mode=agg)
        worst = max(worst, st["max_err_over_lr_Rmax"])
    print(f"identity, W = {W}, s = {s}, {agg}: worst error {worst:.2e} of lr * max|R| (bound 1e-5 plus one ulp)")
    big = Case(specs, s, k, W=W + 1, param_dtype=torch.float32, seed=34)
    with pytest.raises(B.DemoError) as e:
        ctx.demo_decode_ex(big.args, W + 1, hp, s, k)
    assert e.value.status == B.DEMO_ERR_UNSUPPORTED
    # the sign update takes any number of workers
    ctx.demo_decode(big.args, W + 1, LR, 0.0, s, k)
    torch.cuda.synchronize()


def test_count_aggregate_with_repeated_senders(ctx):
    # every worker sends the same k indices: the count-normalised average is the mean of the values,
    # and coefficients nobody sent stay zero (0/0 = 0)
    s, k, W = 64, 8, 7
    case = Case(synth.tensor_set("tiny"), s, k, W=W, seed=33)
    case.fill_payloads()
    for ti in range(len(case.specs)):
        case.idx[ti][1:] = case.idx[ti][0:1]
    hp = B.demo_hparams_default(lr=LR, phi=B.DEMO_PHI_IDENTITY, aggregate=B.DEMO_AGG_COUNT)
    before = case.snapshot()
    ctx.demo_decode_ex(case.args, W, hp, s, k)
    torch.cuda.synchronize()
    after = case.snapshot()
    for ti in range(len(case.specs)):
        C.check_decode(before["x"][ti], before["idx"][ti], before["val"][ti], LR, 0.0, s, "f32", after["x"][ti],
                       phi="identity", aggregate_mode="count")


@pytest.mark.parametrize("s,k,W", [(64, 32, 64), (64, 6, 20), (64, 7, 9), (64, 8, 4), (64, 32, 255), (64, 64, 32),
                                   (32, 32, 16), (32, 5, 30), (32, 8, 3), (32, 32, 17),
                                   (128, 32, 128), (128, 7, 40), (128, 1, 255), (128, 32, 129)])
@pytest.mark.parametrize("phi", ["sign", "identity"])
@pytest.mark.parametrize("pdt", [torch.float32, torch.bfloat16])
def test_count_aggregate_with_many_collisions(ctx, s, k, W, phi, pdt):
    # every worker draws its k distinct indices from the same 2k positions of the chunk: each of them is named by
    # about W/2 workers.  Covers every payload access mode of the fast kernels and the sizes they hand on.
    ctx.demo_set_variant(1)
    case = Case(synth.tensor_set("tiny"), s, k, W=W, param_dtype=pdt, seed=36)
    case.fill_payloads()
    gen = torch.Generator(device="cpu").manual_seed(36)
    for ti, sp in enumerate(case.specs):
        M = s if sp.cols == 0 else s * s
        R = min(2 * k, M)
        stride = M // R
        nch = sp.nchunks(s)
        pick = torch.rand(W, nch, R, generator=gen).argsort(dim=-1)[..., :k] * stride
        case.idx[ti][:W].copy_(pick.to(torch.int32))
    hp = B.demo_hparams_default(lr=LR, weight_decay=0.05, phi=PHI[phi], aggregate=B.DEMO_AGG_COUNT)
    before = case.snapshot()
    ctx.demo_decode_ex(case.args, W, hp, s, k)
    torch.cuda.synchronize()
    after = case.snapshot()
    pd = "bf16" if pdt == torch.bfloat16 else "f32"
    for ti in range(len(case.specs)):
        C.check_decode(before["x"][ti], before["idx"][ti][:W], before["val"][ti][:W], LR, 0.05, s, pd, after["x"][ti],
                       phi=phi, aggregate_mode="count")


@pytest.mark.parametrize("s,k,W", [(64, 32, 200), (64, 8, 300), (32, 32, 64), (32, 8, 255), (128, 32, 255), (128, 64, 200)])
@pytest.mark.parametrize("grow", [1.0, -1.0])
@pytest.mark.parametrize("pdt", [torch.float32, torch.bfloat16])
def test_streamed_payload_with_changing_magnitudes(ctx, s, k, W, grow, pdt):
    # more pairs per chunk than the decode kernels hold in registers: the payload is streamed in rounds, and
    # the magnitudes grow (or shrink) by a factor 2^12 from the first worker to the last, so that round after
    # round the block exponent of the running sums rises (or never does).  phi = identity: the values count.
    ctx.demo_set_variant(1)
    specs = [synth.TensorSpec("a", 2 * s, 3 * s), synth.TensorSpec("v", 2 * s, 0)]
    case = Case(specs, s, k, W=W, param_dtype=pdt, seed=37)
    case.fill_payloads()
    w = torch.arange(W, dtype=torch.float32, device=case.val[0].device)
    factor = torch.exp2(grow * 12.0 * w / (W - 1)).reshape(W, 1, 1)
    for ti in range(len(case.specs)):
        case.val[ti][:W] *= factor
    hp = B.demo_hparams_default(lr=LR, weight_decay=0.0, phi=B.DEMO_PHI_IDENTITY)
    before = case.snapshot()
    ctx.demo_decode_ex(case.args, W, hp, s, k)
    torch.cuda.synchronize()
    after = case.snapshot()
    pd = "bf16" if pdt == torch.bfloat16 else "f32"
    for ti in range(len(case.specs)):
        C.check_decode(before["x"][ti], before["idx"][ti][:W], before["val"][ti][:W], LR, 0.0, s, pd, after["x"][ti],
                       phi="identity")


@pytest.mark.parametrize("variant", [0, 1])
def test_default_hparams_match_plain_calls_bit_for_bit(ctx, variant):
    ctx.demo_set_variant(variant)
    s, k = 64, 32
    a = Case(synth.tensor_set("tiny"), s, k, grad_dtype=torch.bfloat16, param_dtype=torch.bfloat16, seed=34)
    b = Case(synth.tensor_set("tiny"), s, k, grad_dtype=torch.bfloat16, param_dtype=torch.bfloat16, seed=34)
    ctx.demo_step(a.args, 0.999, LR, 0.01, s, k)
    ctx.demo_step_ex(b.args, B.demo_hparams_default(0.999, LR, 0.01), s, k)
    torch.cuda.synchronize()
    sa, sb = a.snapshot(), b.snapshot()
    for key in ("m", "x", "idx", "val"):
        for ta, tb in zip(sa[key], sb[key]):
            assert np.array_equal(ta, tb)


def test_step_ex_is_encode_ex_then_decode_ex(ctx):
    s, k = 64, 16
    hp = B.demo_hparams_default(0.9, LR, 0.05, alpha=0.2, grad_scale=0.1, phi=B.DEMO_PHI_IDENTITY)
    a = Case(synth.tensor_set("tiny"), s, k, seed=35)
    b = Case(synth.tensor_set("tiny"), s, k, seed=35)
    ctx.demo_step_ex(a.args, hp, s, k)
    ctx.demo_encode_ex(b.args, hp, s, k)
    ctx.demo_decode_ex(b.args, 1, hp, s, k)
    torch.cuda.synchronize()
    sa, sb = a.snapshot(), b.snapshot()
    for key in ("m", "x", "idx", "val"):
        for ta, tb in zip(sa[key], sb[key]):
            assert np.array_equal(ta, tb)


def test_hparams_are_validated(ctx):
    case = Case(synth.tensor_set("tiny"), 64, 8, W=2, seed=36)
    for bad in (dict(phi=7), dict(aggregate=-1), dict(reserved=1), dict(lr=float("nan"))):
        with pytest.raises(B.DemoError) as e:
            ctx.demo_decode_ex(case.args, 2, B.demo_hparams_default(**{**dict(lr=LR), **bad}), 64, 8)
        assert e.value.status == B.DEMO_ERR_ARG
    with pytest.raises(B.DemoError):
        ctx.demo_encode_ex(case.args, B.demo_hparams_default(beta=0.9, alpha=float("inf")), 64, 8)


# ---- other projection matrices (ablation "Choice of Linear Projections") ---------------------------------
def _projection(s, kind, step):
    """(argument for demo_set_basis, the oracle's matrix)"""
    from oracle import demo_oracle as O
    if kind == "identity":
        return None, np.eye(s)
    a = synth.projection_draws(s, step)
    return a, O.gram_schmidt(a.double().numpy())


@pytest.mark.parametrize("s,k", [(32, 8), (64, 32), (128, 8)])
@pytest.mark.parametrize("kind", ["identity", "gram_schmidt"])
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_other_projection_matrices(ctx, s, k, kind, dt):
    W = 3
    case = Case(synth.tensor_set("tiny"), s, k, W=W, grad_dtype=dt, param_dtype=dt, seed=37)
    a, P = _projection(s, kind, step=5)
    code = B.DEMO_BASIS_IDENTITY if kind == "identity" else B.DEMO_BASIS_GRAM_SCHMIDT
    try:
        ctx.demo_set_basis(s, code, a)
        before = case.snapshot()
        ctx.demo_encode(case.args, 0.9, s, k)
        torch.cuda.synchronize()
        after = case.snapshot()
        for ti in range(len(case.specs)):
            C.check_encode(before["m"][ti], before["g"][ti], 0.9, s, k, after["idx"][ti][0], after["val"][ti][0],
                           after["m"][ti], P=P)
        case.fill_payloads()
        before = case.snapshot()
        ctx.demo_decode(case.args, W, LR, 0.0, s, k)
        torch.cuda.synchronize()
        after = case.snapshot()
        pd = "bf16" if dt == torch.bfloat16 else "f32"
        for ti in range(len(case.specs)):
            C.check_decode(before["x"][ti], before["idx"][ti], before["val"][ti], LR, 0.0, s, pd, after["x"][ti], P=P)
    finally:
        ctx.demo_set_basis(s, B.DEMO_BASIS_DCT)


# ---- s = 64 with another matrix runs on the full-product instances of the wavefront kernels: budgets, worker counts,
#      both payload access modes, the identity update and the other scalars, against the same oracle ---------------
@pytest.mark.parametrize("W,k", [(1, 32), (8, 32), (64, 32), (5, 7), (3, 1), (16, 64), (100, 20), (2, 33)])
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("phi", ["sign", "identity"])
def test_random_projection_on_the_wavefront_kernels(ctx, W, k, dt, phi):
    s = 64
    ctx.demo_set_variant(1)
    specs = [synth.TensorSpec("a", 384, 640), synth.TensorSpec("v0", 256, 0), synth.TensorSpec("b", 2048, 1536)]
    case = Case(specs, s, k, W=W, grad_dtype=dt, param_dtype=dt, seed=41)
    a, P = _projection(s, "gram_schmidt", step=W + k)
    pd = "bf16" if dt == torch.bfloat16 else "f32"
    try:
        ctx.demo_set_basis(s, B.DEMO_BASIS_GRAM_SCHMIDT, a)
        hp = B.demo_hparams_default(0.9, LR, 0.05, alpha=0.5, grad_scale=0.25, phi=PHI[phi],
                                    aggregate=B.DEMO_AGG_MEAN if phi == "identity" else B.DEMO_AGG_SUM)
        before = case.snapshot()
        ctx.demo_encode_ex(case.args, hp, s, k)
        torch.cuda.synchronize()
        after = case.snapshot()
        for ti in range(len(case.specs)):
            C.check_encode(before["m"][ti], before["g"][ti], 0.9, s, k, after["idx"][ti][0], after["val"][ti][0],
                           after["m"][ti], alpha32=0.5, grad_scale32=0.25, P=P)
        case.fill_payloads(exact=False)
        before = case.snapshot()
        ctx.demo_decode_ex(case.args, W, hp, s, k)
        torch.cuda.synchronize()
        after = case.snapshot()
        for ti in range(len(case.specs)):
            C.check_decode(before["x"][ti], before["idx"][ti], before["val"][ti], LR, 0.05, s, pd, after["x"][ti],
                           phi=phi, aggregate_mode="mean" if phi == "identity" else "sum", P=P)
    finally:
        ctx.demo_set_basis(s, B.DEMO_BASIS_DCT)


@pytest.mark.parametrize("kind", ["dct", "identity", "gram_schmidt"])
@pytest.mark.parametrize("exp2", [-80, 60])
def test_encode_is_scale_free_over_the_exponent_range(ctx, kind, exp2):
    # gradients and momentum scaled by 2^-80 and 2^60: every bound of the comparison is relative to the chunk's largest
    # magnitude, so nothing may depend on the absolute scale.  With another matrix than the DCT the s = 64 products run
    # on the float16 matrix pipe: the tile is scaled by a power of two taken from its largest magnitude and every
    # operand carried as two float16 parts (22 significant bits); with the identity matrix the coefficients are the
    # momentum values themselves to that precision.
    s, k = 64, 32
    ctx.demo_set_variant(1)
    scale = 2.0 ** exp2
    specs = [synth.TensorSpec("a", 256, 384), synth.TensorSpec("v0", 256, 0)]
    case = Case(specs, s, k, seed=43, grad_std=1e-2 * scale, mom_std=1e-3 * scale)
    P = None
    try:
        if kind == "identity":
            ctx.demo_set_basis(s, B.DEMO_BASIS_IDENTITY)
            P = np.eye(s)
        elif kind == "gram_schmidt":
            a, P = _projection(s, kind, step=11)
            ctx.demo_set_basis(s, B.DEMO_BASIS_GRAM_SCHMIDT, a)
        before = case.snapshot()
        ctx.demo_encode(case.args, 0.9, s, k)
        torch.cuda.synchronize()
        after = case.snapshot()
        for ti in range(len(case.specs)):
            st = C.check_encode(before["m"][ti], before["g"][ti], 0.9, s, k, after["idx"][ti][0], after["val"][ti][0],
                                after["m"][ti], P=P)
            assert st["chunks"] == case.specs[ti].nchunks(s)
        if kind == "identity":
            # Q = momentum after the update: the k payload values of a chunk are elements of beta m + g as float32
            m0, g0 = before["m"][0].astype(np.float32), before["g"][0].astype(np.float32)
            upd = (np.float32(0.9) * m0.astype(np.float64) + g0.astype(np.float64)).astype(np.float32)
            blocks = upd.reshape(256 // s, s, 384 // s, s).transpose(0, 2, 1, 3).reshape(-1, s * s)
            idx, val = after["idx"][0][0], after["val"][0][0]
            want = np.take_along_axis(blocks, idx.astype(np.int64), axis=1).astype(np.float64)
            assert np.all(np.abs(val.astype(np.float64) - want) <= np.abs(want) * 2.0 ** -21)
    finally:
        ctx.demo_set_basis(s, B.DEMO_BASIS_DCT)


def test_new_matrix_every_step_then_back_to_dct(ctx):
    # the paper's random projection: a fresh matrix per step, seeded with the step number
    s, k = 64, 16
    case = Case(synth.tensor_set("tiny"), s, k, seed=38)
    ref = Case(synth.tensor_set("tiny"), s, k, seed=38)
    try:
        for step in range(3):
            a, P = _projection(s, "gram_schmidt", step)
            ctx.demo_set_basis(s, B.DEMO_BASIS_GRAM_SCHMIDT, a)
            case.new_grads(step)
            before = case.snapshot()
            ctx.demo_encode(case.args, 0.9, s, k)
            torch.cuda.synchronize()
            after = case.snapshot()
            for ti in range(len(case.specs)):
                C.check_encode(before["m"][ti], before["g"][ti], 0.9, s, k, after["idx"][ti][0],
                               after["val"][ti][0], after["m"][ti], P=P)
    finally:
        ctx.demo_set_basis(s, B.DEMO_BASIS_DCT)
    # back on the DCT the wavefront kernels are in use again and give what a fresh context gives
    fresh = B.Context()
    a2 = Case(synth.tensor_set("tiny"), s, k, seed=39)
    ctx.demo_encode(a2.args, 0.9, s, k)
    fresh.demo_encode(ref.args, 0.9, s, k)   # `ref` holds seed 38: only its own consistency matters below
    b2 = Case(synth.tensor_set("tiny"), s, k, seed=39)
    fresh.demo_encode(b2.args, 0.9, s, k)
    torch.cuda.synchronize()
    sa, sb = a2.snapshot(), b2.snapshot()
    for key in ("m", "idx", "val"):
        for ta, tb in zip(sa[key], sb[key]):
            assert np.array_equal(ta, tb)
    fresh.close()


def test_set_basis_rejects_dependent_rows(ctx):
    a = synth.projection_draws(32, 0)
    a[7] = a[3] * 2.0
    with pytest.raises(B.DemoError) as e:
        ctx.demo_set_basis(32, B.DEMO_BASIS_GRAM_SCHMIDT, a)
    assert e.value.status == B.DEMO_ERR_ARG


@pytest.mark.parametrize("s,k,W", [(64, 32, 8), (32, 8, 4), (128, 32, 3)])
def test_identity_phi_with_zero_step_leaves_parameters_untouched(ctx, s, k, W):
    # lr = 0 with phi = identity: x' = x - 0 * (R + wd x) must give x back bit for bit, on freshly allocated float32
    # tensors and in the first launches of a context.  (Regression: the data registers of a 16-byte buffer store
    # were overwritten by the instruction right behind it; a few elements per launch then held R instead of x.)
    for rep in range(4):
        c = B.Context()
        c.demo_set_variant(1)
        case = Case(synth.tensor_set("tiny"), s, k, W=W, param_dtype=torch.float32, seed=40 + rep)
        case.fill_payloads()
        before = [x.clone() for x in case.x]
        hp = B.demo_hparams_default(lr=0.0, weight_decay=0.0, phi=PHI["identity"], aggregate=AGG["sum"])
        c.demo_decode_ex(case.args, W, hp, s, k)
        torch.cuda.synchronize()
        for b, a in zip(before, case.x):
            assert torch.equal(a, b)
        c.close()


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("s,k", [(64, 32), (32, 8), (128, 32)])
@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
def test_encode_with_nothing_to_add_or_subtract_leaves_momentum_untouched(variant, s, k, gdt):
    # beta = 1, g = 0, alpha = 0: m' = 1 m + 0 - 0 R must give the momentum back bit for bit, on freshly allocated
    # tensors and in the first launches of a context.  The encode kernels' twin of the test above: a momentum store
    # whose data registers were overwritten by the instruction behind it would leave some other row's value here.
    for rep in range(3):
        c = B.Context()
        c.demo_set_variant(variant)
        case = Case(synth.tensor_set("tiny"), s, k, grad_dtype=gdt, grad="zero", seed=50 + rep)
        before = [m.clone() for m in case.m]
        c.demo_encode_ex(case.args, B.demo_hparams_default(beta=1.0, alpha=0.0), s, k)
        torch.cuda.synchronize()
        for ti, (b, a) in enumerate(zip(before, case.m)):
            assert torch.equal(a, b), case.specs[ti].name
            assert bool((case.val[ti][0].abs().amax(dim=1) > 0).all())   # the payload is still the top-k of m
        c.close()
