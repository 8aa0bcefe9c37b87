"""Parity of the s = 128 workgroup-per-chunk kernels with the float64 oracle: more chunks than workgroups
(persistent loop, prefetch across tensor boundaries), the candidate-list overflow that hands a chunk to the
exact kernel, all-zero chunks, budgets up to the kernel's limit and beyond it, payload sizes up to the
register capacity of the decode kernel and beyond it, very different payload scales from chunk to chunk."""
import numpy as np
import pytest
import torch

from paper_2411_19870_amd import binding as B
from paper_2411_19870_amd import synth
from tests.gpu_harness import Case, DEV
from tests.test_gpu_parity import run_encode_check, run_decode_check, BETA, LR

pytestmark = pytest.mark.gpu

S = 128


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available()
    c = B.Context()
    c.demo_set_variant(1)
    yield c
    c.close()


@pytest.mark.parametrize("gdt,pdt", [(torch.float32, torch.float32), (torch.bfloat16, torch.bfloat16)])
def test_more_chunks_than_workgroups(ctx, gdt, pdt):
    # 288 + 15 + 40 chunks on 256 workgroups: some workgroups take a second chunk, of another tensor
    specs = [synth.TensorSpec("a", 1536, 3072), synth.TensorSpec("b", 640, 384), synth.TensorSpec("v", 256, 0),
             synth.TensorSpec("c", 1024, 640)]
    case = Case(specs, S, 32, W=2, grad_dtype=gdt, param_dtype=pdt, seed=21)
    st = run_encode_check(ctx, case)
    assert sum(x["chunks"] for x in st) == 288 + 15 + 2 + 40
    run_decode_check(ctx, case, W=1)
    case.fill_payloads()
    run_decode_check(ctx, case, W=2, wd=0.05)


@pytest.mark.parametrize("k", [1, 5, 64, 65])
def test_budgets_up_to_and_past_the_kernel_limit(ctx, k):
    specs = [synth.TensorSpec("a", 384, 256), synth.TensorSpec("b", 128, 128)]
    case = Case(specs, S, k, grad="student", grad_dtype=torch.bfloat16, seed=30 + k)
    run_encode_check(ctx, case)
    run_decode_check(ctx, case, W=1)


@pytest.mark.parametrize("nequal", [40, 600, 5000])
def test_many_near_equal_magnitudes(ctx, nequal):
    # chunks built as the inverse DCT of `nequal` coefficients of magnitude exactly 1 (and one clear winner):
    # past 512 candidates at the threshold the kernel queues the chunk for the exact kernel
    import scipy.fft
    rng = np.random.default_rng(nequal)
    specs = [synth.TensorSpec("a", 256, 384)]
    case = Case(specs, S, 32, grad="zero", mom_std=0, seed=11)
    blocks = np.zeros((2, 3, S, S))
    for a in range(2):
        for b in range(3):
            q = np.zeros(S * S)
            q[rng.permutation(S * S)[:nequal]] = rng.choice([-1.0, 1.0], size=nequal)
            q[rng.integers(0, S * S)] = 3.0
            blocks[a, b] = scipy.fft.idctn(q.reshape(S, S), type=2, norm="ortho")
    blocks[1, 1] = rng.normal(size=(S, S))      # an ordinary chunk among them
    case.g[0].copy_(torch.from_numpy(blocks.transpose(0, 2, 1, 3).reshape(256, 384)).float())
    st = run_encode_check(ctx, case, beta=0.0)[0]
    print("near-equal magnitudes", nequal, st)


def test_all_zero_and_constant_chunks(ctx):
    specs = [synth.TensorSpec("a", 256, 256)]
    case = Case(specs, S, 4, grad="zero", mom_std=0, seed=4)
    case.g[0][:128, :128] = 0.5                 # one DC coefficient, every other exactly or nearly zero
    case.g[0][128:, 128:] = synth.gaussian(synth.TensorSpec("q", 128, 128), 1e-2, 1, 0, 0, "grad").to(DEV)
    m_before = case.m[0].clone()
    ctx.demo_encode(case.args, BETA, S, 4)
    torch.cuda.synchronize()
    assert case.idx[0][0, 0, 0] == 0 and abs(float(case.val[0][0, 0, 0]) - 0.5 * 128) < 1e-4
    # the two all-zero chunks: the k lowest indices, zero values, momentum stays zero
    for c in (1, 2):
        assert case.idx[0][0, c].tolist() == [0, 1, 2, 3] and (case.val[0][0, c] == 0).all()
    assert (case.m[0][:128, 128:] == 0).all() and (case.m[0][128:, :128] == 0).all()
    # the oracle on the same tensor without the constant chunk (whose runners-up are rounding noise)
    case2 = Case(specs, S, 4, grad="zero", mom_std=0, seed=4)
    case2.g[0].copy_(case.g[0])
    case2.g[0][:128, :128] = 0
    case2.m[0].copy_(m_before)
    run_encode_check(ctx, case2)


@pytest.mark.parametrize("W,k", [(128, 32), (129, 32), (64, 64), (255, 16), (1, 1), (33, 7), (255, 32), (200, 30), (90, 6)])
@pytest.mark.parametrize("pdt", [torch.float32, torch.bfloat16])
def test_decode_payload_sizes(ctx, W, k, pdt):
    # W k = 4096 is the register capacity of the workgroup kernel; past it the payload is streamed in rounds
    # (k a multiple of 4) or the generic kernel runs
    specs = [synth.TensorSpec("a", 256, 384), synth.TensorSpec("v", 256, 0)]
    case = Case(specs, S, k, W=W, param_dtype=pdt, seed=200 + W)
    case.fill_payloads()
    st = run_decode_check(ctx, case, W=W, wd=0.01)
    assert sum(x["elements"] for x in st) == sum(sp.numel for sp in specs)


def test_decode_chunks_with_very_different_scales(ctx):
    specs = [synth.TensorSpec("a", 256, 256)]
    W, k = 4, 16
    case = Case(specs, S, k, W=W, seed=7)
    case.fill_payloads()
    case.val[0][:, 1, :] *= 1e12
    case.val[0][:, 2, :] *= 1e-12
    run_decode_check(ctx, case, W=W)


def test_generic_and_workgroup_kernels_agree_on_the_payload(ctx):
    # same inputs through both kernel families: identical index sets (ties aside, none here) and values to rounding
    specs = [synth.TensorSpec("a", 384, 512)]
    a = Case(specs, S, 32, grad_dtype=torch.bfloat16, seed=3)
    b = Case(specs, S, 32, grad_dtype=torch.bfloat16, seed=3)
    ctx.demo_set_variant(1)
    ctx.demo_encode(a.args, BETA, S, 32)
    ctx.demo_set_variant(0)
    ctx.demo_encode(b.args, BETA, S, 32)
    ctx.demo_set_variant(1)
    torch.cuda.synchronize()
    assert torch.equal(a.idx[0].sort(dim=-1).values, b.idx[0].sort(dim=-1).values)
    assert torch.allclose(a.val[0].abs().sum(), b.val[0].abs().sum(), rtol=1e-5)
    assert torch.allclose(a.m[0], b.m[0], rtol=0, atol=1e-6)


# ---- few pairs per chunk (W k <= 64): the kernel without a coefficient tile -------------------------------------------
@pytest.mark.parametrize("W,k", [(1, 32), (1, 64), (2, 32), (64, 1), (7, 9), (3, 1), (1, 5)])
@pytest.mark.parametrize("pdt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("phi,agg", [("sign", "sum"), ("identity", "mean")])
def test_few_pairs_decode(ctx, W, k, pdt, phi, agg):
    from tests import compare as C
    # 288 + 6 chunks on 256 workgroups (second chunks, of another tensor), an order-1 tensor in between
    specs = [synth.TensorSpec("a", 1536, 3072), synth.TensorSpec("v", 256, 0), synth.TensorSpec("b", 384, 256)]
    case = Case(specs, S, k, W=W, param_dtype=pdt, seed=500 + W + k)
    case.fill_payloads()
    # workers that name the same coefficient add up; indices out of range contribute nothing
    if W > 1:
        case.idx[0][1, :, 0] = case.idx[0][0, :, 0]
        case.idx[2][W - 1, 3, 0] = case.idx[2][0, 3, 0]
    case.idx[0][0, 5, k - 1] = 16384
    case.idx[2][0, 1, 0] = -7
    hp = B.demo_hparams_default(lr=LR, weight_decay=0.05, phi=B.DEMO_PHI_IDENTITY if phi == "identity" else B.DEMO_PHI_SIGN,
                                aggregate=B.DEMO_AGG_MEAN if agg == "mean" else B.DEMO_AGG_SUM)
    before = case.snapshot()
    ctx.demo_decode_ex(case.args, W, hp, S, k)
    torch.cuda.synchronize()
    after = case.snapshot()
    pd = "bf16" if pdt == torch.bfloat16 else "f32"
    for ti in range(len(specs)):
        C.check_decode(before["x"][ti], before["idx"][ti][:W], before["val"][ti][:W], LR, 0.05, S, pd, after["x"][ti],
                       phi=phi, aggregate_mode=agg)


# ---- the products run on the float16 matrix pipe at a scale taken from the chunk: nothing may depend on the
#      absolute scale of the data, and patterns that line up with one basis row must stay inside the float16 range ----
@pytest.mark.parametrize("exp2", [-100, -80, 60, 100])
@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
def test_encode_is_scale_free_over_the_exponent_range(ctx, exp2, gdt):
    scale = 2.0 ** exp2
    specs = [synth.TensorSpec("a", 384, 256)]
    case = Case(specs, S, 32, seed=61, grad_dtype=gdt, grad_std=1e-2 * scale, mom_std=1e-3 * scale)
    st = run_encode_check(ctx, case, beta=0.9)[0]
    assert st["chunks"] == 6


def test_encode_of_patterns_that_line_up_with_a_basis_row(ctx):
    # every chunk is the inverse transform of eight planted coefficients with magnitudes 1, 1/2, ..., 1/128 times an
    # amplitude: a tile of bounded elements whose energy sits in a few basis rows has the largest coefficients such a
    # tile can have (constant and checkerboard tiles: s times the element size), and the smallest planted one lies
    # seven binary orders below the largest
    import scipy.fft
    specs = [synth.TensorSpec("a", 256, 384)]
    case = Case(specs, S, 8, seed=62, mom_std=0, grad="zero")
    rng = np.random.default_rng(62)
    planted = [[(0, 0), (127, 127)], [(127, 127), (0, 0)], [(17, 90), (90, 17)], [(0, 127), (64, 64)],
               [(1, 1), (126, 2)], [(63, 65), (127, 0)]]
    q = np.zeros((2, 3, S, S))
    for c, heads in enumerate(planted):
        pos = list(heads)
        while len(pos) < 8:
            p = (int(rng.integers(0, S)), int(rng.integers(0, S)))
            if p not in pos:
                pos.append(p)
        for j, (u, v) in enumerate(pos):
            q[c // 3, c % 3, u, v] = (1.0 if j % 2 == 0 else -1.0) * 2.0 ** -j * (3.0 if c % 2 == 0 else 1e-3)
    g = scipy.fft.idctn(q, type=2, norm="ortho", axes=(2, 3)).transpose(0, 2, 1, 3).reshape(256, 384)
    case.g[0].copy_(torch.from_numpy(g).float())
    st = run_encode_check(ctx, case, beta=0.0)[0]
    assert st["chunks"] == 6 and st["sets_identical"] == 6
    run_decode_check(ctx, case, W=1)


def test_decode_when_every_worker_names_the_same_coefficients(ctx):
    # W equal pairs per coefficient: the sums reach W times the largest value, the top of the block fixed point and of
    # the float16 range the products are scaled to
    W, k = 64, 32
    specs = [synth.TensorSpec("a", 256, 256), synth.TensorSpec("v", 128, 0)]
    case = Case(specs, S, k, W=W, param_dtype=torch.bfloat16, seed=63)
    case.fill_payloads()
    for ti in range(len(specs)):
        case.idx[ti][:] = case.idx[ti][0:1]
        case.val[ti][:] = case.val[ti][0:1].abs()
    run_decode_check(ctx, case, W=W)
