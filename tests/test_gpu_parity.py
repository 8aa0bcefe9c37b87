"""Element-by-element parity of the HIP path (through the C ABI) with the float64
oracle on seeded inputs small enough for the oracle to finish in seconds, spanning
several chunks per tensor, ragged chunk grids, both dtypes and the edge cases."""
import numpy as np
import pytest
import torch

from paper_2411_19870_amd import binding as B
from paper_2411_19870_amd import synth
from tests import compare as C
from tests.gpu_harness import Case, np64, DEV

pytestmark = pytest.mark.gpu

BETA, LR = 0.999, 1e-3


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available()
    c = B.Context()
    yield c
    c.close()


def run_encode_check(ctx, case, beta=BETA):
    before = case.snapshot()
    ctx.demo_encode(case.args, beta, case.s, case.k)
    torch.cuda.synchronize()
    after = case.snapshot()
    stats = []
    for ti in range(len(case.specs)):
        st = C.check_encode(before["m"][ti], before["g"][ti], beta, case.s, case.k,
                            after["idx"][ti][0], after["val"][ti][0], after["m"][ti])
        stats.append(st)
        assert np.array_equal(after["g"][ti], before["g"][ti])          # encode leaves g and x alone
        assert np.array_equal(after["x"][ti], before["x"][ti])
    return stats


def run_decode_check(ctx, case, W, lr=LR, wd=0.0):
    before = case.snapshot()
    ctx.demo_decode(case.args, W, lr, wd, case.s, case.k)
    torch.cuda.synchronize()
    after = case.snapshot()
    pd = "bf16" if case.x[0].dtype == torch.bfloat16 else "f32"
    stats = []
    for ti in range(len(case.specs)):
        st = C.check_decode(before["x"][ti], before["idx"][ti][:W], before["val"][ti][:W], lr, wd, case.s, pd,
                            after["x"][ti])
        stats.append(st)
        assert np.array_equal(after["m"][ti], before["m"][ti])          # decode leaves m and the payload alone
        assert np.array_equal(after["idx"][ti], before["idx"][ti])
    return stats


# ---- config 1: single fp32 1024 x 1024, s = 64, k = 32, W = 1 ------------------------------
@pytest.mark.parametrize("variant", [0, 1])
def test_config1_single_matrix(ctx, variant):
    ctx.demo_set_variant(variant)
    case = Case(synth.tensor_set("single"), 64, 32, seed=0)
    st = run_encode_check(ctx, case)[0]
    print("config1 encode", st)
    assert st["chunks"] == 256
    st = run_decode_check(ctx, case, W=1)[0]
    print("config1 decode", st)
    ctx.demo_set_variant(1)


# ---- tiny ragged set: all chunk sizes, budgets, dtypes ---------------------------------------
@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("s", [32, 64, 128])
@pytest.mark.parametrize("k", [1, 8, 32])
@pytest.mark.parametrize("gdt,pdt", [(torch.float32, torch.float32), (torch.bfloat16, torch.bfloat16)])
def test_tiny_set_encode_decode(ctx, variant, s, k, gdt, pdt):
    ctx.demo_set_variant(variant)
    case = Case(synth.tensor_set("tiny"), s, k, W=3, grad_dtype=gdt, param_dtype=pdt, seed=s + k)
    run_encode_check(ctx, case)
    # decode of the own payload (W = 1), then of three workers' payloads with weight decay
    run_decode_check(ctx, case, W=1)
    case.fill_payloads()
    run_decode_check(ctx, case, W=3, wd=0.1)
    ctx.demo_set_variant(1)


@pytest.mark.parametrize("variant", [0, 1])
def test_step_equals_encode_then_decode(ctx, variant):
    ctx.demo_set_variant(variant)
    a = Case(synth.tensor_set("tiny"), 64, 8, grad_dtype=torch.bfloat16, param_dtype=torch.bfloat16, seed=5)
    b = Case(synth.tensor_set("tiny"), 64, 8, grad_dtype=torch.bfloat16, param_dtype=torch.bfloat16, seed=5)
    ctx.demo_step(a.args, BETA, LR, 0.01, 64, 8)
    ctx.demo_encode(b.args, BETA, 64, 8)
    ctx.demo_decode(b.args, 1, LR, 0.01, 64, 8)
    torch.cuda.synchronize()
    for ti in range(len(a.specs)):
        assert torch.equal(a.m[ti], b.m[ti]) and torch.equal(a.x[ti], b.x[ti])
        assert torch.equal(a.idx[ti], b.idx[ti]) and torch.equal(a.val[ti], b.val[ti])
    ctx.demo_set_variant(1)


# ---- many workers with collisions (decode-heavy shape, small) ----------------------------------
@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("s,W", [(64, 64), (32, 16), (128, 8)])
def test_decode_many_workers(ctx, variant, s, W):
    ctx.demo_set_variant(variant)
    specs = [synth.TensorSpec("a", 2 * s, 3 * s), synth.TensorSpec("v", 4 * s, 0)]
    case = Case(specs, s, 32, W=W, param_dtype=torch.bfloat16, seed=W)
    case.fill_payloads()
    st = run_decode_check(ctx, case, W=W)
    print("decode W", W, st)
    ctx.demo_set_variant(1)


def test_decode_is_run_to_run_deterministic(ctx):
    specs = [synth.TensorSpec("a", 128, 256)]
    outs = []
    for rep in range(3):
        case = Case(specs, 64, 32, W=64, param_dtype=torch.float32, seed=1)
        case.fill_payloads()
        ctx.demo_decode(case.args, 64, LR, 0.0, 64, 32)
        torch.cuda.synchronize()
        outs.append(case.x[0].clone())
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


def test_decode_ignores_out_of_range_indices(ctx):
    specs = [synth.TensorSpec("a", 64, 64), synth.TensorSpec("v", 64, 0)]
    case = Case(specs, 64, 8, W=2, seed=2)
    case.fill_payloads()
    case.idx[0][1, 0, 0] = 4096
    case.idx[0][1, 0, 1] = -5
    case.idx[1][0, 0, 0] = 64
    run_decode_check(ctx, case, W=2)


# ---- degenerate inputs -----------------------------------------------------------------------------
@pytest.mark.parametrize("variant", [0, 1])
def test_all_zero_chunks(ctx, variant):
    # zero gradient and zero momentum: every magnitude ties at 0 -> lowest indices, zero values,
    # momentum stays zero; decode of that payload has sgn = 0 and only applies weight decay
    ctx.demo_set_variant(variant)
    case = Case(synth.tensor_set("tiny"), 64, 8, grad="zero", mom_std=0, seed=3)
    run_encode_check(ctx, case)
    for ti in range(len(case.specs)):
        assert torch.equal(case.idx[ti][0], torch.arange(8, dtype=torch.int32, device=DEV).expand_as(case.idx[ti][0]))
        assert not case.val[ti].any() and not case.m[ti].any()
    x0 = [t.clone() for t in case.x]
    run_decode_check(ctx, case, W=1, wd=0.5)
    for ti in range(len(case.specs)):
        expect = torch.addcmul(x0[ti], x0[ti], torch.tensor(-LR * 0.5, device=DEV))
        assert torch.allclose(case.x[ti], expect, rtol=1e-6, atol=0)
    ctx.demo_set_variant(1)


@pytest.mark.parametrize("variant", [0, 1])
def test_exact_ties_take_lowest_indices(ctx, variant):
    # a chunk whose only non-zero is a constant block: one DC coefficient, all others exactly 0
    ctx.demo_set_variant(variant)
    sp = [synth.TensorSpec("a", 64, 128), synth.TensorSpec("v", 128, 0)]
    case = Case(sp, 64, 4, grad="zero", mom_std=0, seed=4)
    case.g[0].fill_(0.5)
    case.g[1].fill_(-0.25)
    ctx.demo_encode(case.args, BETA, 64, 4)
    torch.cuda.synchronize()
    # the DC coefficient first, then ties among (numerically tiny) others: only check the head and legitimacy
    assert (case.idx[0][0, :, 0] == 0).all() and (case.idx[1][0, :, 0] == 0).all()
    assert torch.allclose(case.val[0][0, :, 0], torch.full((2,), 0.5 * 64, device=DEV), rtol=1e-6)
    assert torch.allclose(case.val[1][0, :, 0], torch.full((2,), -0.25 * 8, device=DEV), rtol=1e-6)
    ctx.demo_set_variant(1)


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("nequal", [40, 300, 2000])
def test_many_near_equal_magnitudes(ctx, variant, nequal):
    # chunks built as the inverse DCT of `nequal` coefficients of magnitude exactly 1: after the
    # forward transform they agree to rounding noise, far more candidates than k sit at the threshold
    # (the wavefront kernel hands such chunks to the exact workgroup kernel)
    import scipy.fft
    ctx.demo_set_variant(variant)
    rng = np.random.default_rng(nequal)
    sp = [synth.TensorSpec("a", 128, 192)]
    case = Case(sp, 64, 32, grad="zero", mom_std=0, seed=11)
    blocks = np.zeros((2, 3, 64, 64))
    for a in range(2):
        for b in range(3):
            q = np.zeros(4096)
            pos = rng.permutation(4096)[:nequal]
            q[pos] = rng.choice([-1.0, 1.0], size=nequal)
            q[rng.integers(0, 4096)] = 3.0                      # one clear winner
            blocks[a, b] = scipy.fft.idctn(q.reshape(64, 64), type=2, norm="ortho")
    g = blocks.transpose(0, 2, 1, 3).reshape(128, 192)
    case.g[0].copy_(torch.from_numpy(g).float())
    st = run_encode_check(ctx, case, beta=0.0)[0]
    print("near-equal magnitudes", nequal, st)
    ctx.demo_set_variant(1)


@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("s", [32, 64, 128])
def test_spectrum_confined_to_a_few_rows_and_columns(ctx, s, gdt):
    # every chunk's spectrum lives on a 16 x 16 grid of frequency pairs (low ones and a few odd high
    # ones), the rest is rounding noise five orders below: whatever way a kernel spreads coefficients
    # over lanes, the large ones sit in a small part of them, so a threshold taken from per-lane
    # maxima is far below the k-th magnitude and the candidate list is long
    import scipy.fft
    rng = np.random.default_rng(s)
    u = np.array([0, 1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, s // 2 + 1, s // 2 + 3, s // 2 + 5, s // 2 + 7])
    sp = [synth.TensorSpec("a", 4 * s, 6 * s)]
    case = Case(sp, s, 32, grad="zero", mom_std=0, grad_dtype=gdt, seed=12)
    q = np.zeros((4, 6, s, s))
    q[:, :, u[:, None], u[None, :]] = rng.standard_normal((4, 6, 16, 16))
    g = 1e-2 * scipy.fft.idctn(q, type=2, norm="ortho", axes=(2, 3)).transpose(0, 2, 1, 3).reshape(4 * s, 6 * s)
    case.g[0].copy_(torch.from_numpy(g).to(gdt))
    st = run_encode_check(ctx, case, beta=0.0)[0]
    print("confined spectrum", s, gdt, st)
    assert st["sets_identical"] + st["tie_swaps"] == st["chunks"] == 24


@pytest.mark.parametrize("s", [32, 64, 128])
def test_k_equals_M_exact_recovery_1d(ctx, s):
    # k = M on order-1 chunks: the payload is the whole spectrum, the residual momentum vanishes
    # (appendix remark on isometric transformations) and decode of the payload returns sgn(m_mid)
    sp = [synth.TensorSpec("v", 8 * s, 0)]
    case = Case(sp, s, s, seed=6)
    before = case.snapshot()
    run_encode_check(ctx, case)
    m_mid = np.float32(BETA).astype(np.float64) * before["m"][0] + before["g"][0]
    assert np.abs(np64(case.m[0])).max() <= 1e-5 * np.abs(m_mid).max()
    assert sorted(case.idx[0][0, 0].tolist()) == list(range(s))
    run_decode_check(ctx, case, W=1)


# ---- momentum carried over consecutive steps (teacher forced) ---------------------------------------
@pytest.mark.parametrize("s", [32, 64, 128])
@pytest.mark.parametrize("k", [1, 8, 32])
def test_ten_steps_student_t_bf16(ctx, s, k):
    specs = [synth.TensorSpec("a", 256, 384), synth.TensorSpec("v", 512, 0)]
    case = Case(specs, s, k, grad="student", grad_dtype=torch.bfloat16, param_dtype=torch.bfloat16, mom_std=0, seed=7)
    swaps = 0
    for step in range(10):
        case.new_grads(step)
        sts = run_encode_check(ctx, case)          # oracle restarts from the GPU's momentum each step
        swaps += sum(st["tie_swaps"] for st in sts)
        run_decode_check(ctx, case, W=1)
    print(f"s={s} k={k}: tie swaps over 10 steps: {swaps}")


# ---- resume: 10 steps == 5 steps, reload state, 5 steps ----------------------------------------------
def test_resume_is_bit_exact(ctx):
    specs = synth.tensor_set("tiny")

    def run(split):
        case = Case(specs, 64, 8, grad_dtype=torch.bfloat16, param_dtype=torch.bfloat16, mom_std=0, seed=8)
        for step in range(10):
            if split and step == 5:
                saved = ([t.cpu() for t in case.m], [t.cpu() for t in case.x])
                case = Case(specs, 64, 8, grad_dtype=torch.bfloat16, param_dtype=torch.bfloat16, mom_std=0, seed=8)
                for ti in range(len(specs)):
                    case.m[ti].copy_(saved[0][ti])
                    case.x[ti].copy_(saved[1][ti])
            case.new_grads(step)
            ctx.demo_step(case.args, BETA, LR, 0.0, 64, 8)
        torch.cuda.synchronize()
        return case

    a, b = run(False), run(True)
    for ti in range(len(specs)):
        assert torch.equal(a.m[ti], b.m[ti]) and torch.equal(a.x[ti], b.x[ti])


def test_timing_hooks(ctx):
    case = Case(synth.tensor_set("tiny"), 64, 8, seed=9)
    ctx.demo_set_timing(True)
    ctx.demo_encode(case.args, BETA, 64, 8)
    ctx.demo_decode(case.args, 1, LR, 0.0, 64, 8)
    for which in range(4):
        assert ctx.demo_last_kernel_ms(which) > 0
    ctx.demo_set_timing(False)


# ---- s = 32 decode: wavefront-per-tile kernel (tile-aligned shapes, W*k <= 512) and the fallback ---------------
@pytest.mark.parametrize("W,k", [(16, 32), (1, 32), (5, 7), (64, 8), (3, 1), (8, 32), (17, 32),
                                 # more than 512 pairs per chunk: streamed in rounds (k a multiple of 4), else generic
                                 (64, 32), (255, 8), (40, 20), (33, 16), (100, 7), (200, 32)])
@pytest.mark.parametrize("pdt", [torch.float32, torch.bfloat16])
def test_s32_decode_tile_kernel(ctx, W, k, pdt):
    ctx.demo_set_variant(1)
    specs = [synth.TensorSpec("a", 192, 320), synth.TensorSpec("b", 64, 64), synth.TensorSpec("v", 96, 0),
             synth.TensorSpec("c", 128, 1088)]
    case = Case(specs, 32, k, W=W, param_dtype=pdt, seed=100 + W)
    case.fill_payloads()
    st = run_decode_check(ctx, case, W=W, wd=0.01)
    assert sum(x["elements"] for x in st) == sum(sp.numel for sp in specs)
    ctx.demo_set_variant(1)


def test_s32_decode_chunks_with_very_different_scales(ctx):
    # the four chunks of a tile keep separate fixed-point scales: one chunk's payload is 1e12 times larger
    ctx.demo_set_variant(1)
    specs = [synth.TensorSpec("a", 128, 128)]
    W, k = 4, 16
    case = Case(specs, 32, k, W=W, seed=7)
    case.fill_payloads()
    case.val[0][:, 5, :] *= 1e12        # chunk 5 = tile (0, 0)... of the 4 x 4 chunk grid: row 1, column 1
    case.val[0][:, 6, :] *= 1e-12
    run_decode_check(ctx, case, W=W)


def test_s32_decode_unaligned_shape_takes_the_generic_kernel(ctx):
    ctx.demo_set_variant(1)
    specs = [synth.TensorSpec("a", 96, 160)]
    case = Case(specs, 32, 8, W=4, seed=9)
    case.fill_payloads()
    run_decode_check(ctx, case, W=4)


def test_s32_list_with_and_without_64_multiples(ctx):
    # 96 x 160 cannot be cut into 64 x 64 tiles: it runs apart from the tensors that can
    ctx.demo_set_variant(1)
    specs = [synth.TensorSpec("a", 128, 192), synth.TensorSpec("b", 96, 160), synth.TensorSpec("c", 64, 256),
             synth.TensorSpec("d", 32, 32), synth.TensorSpec("v", 96, 0)]
    case = Case(specs, 32, 8, W=4, grad_dtype=torch.bfloat16, param_dtype=torch.bfloat16, seed=10)
    run_encode_check(ctx, case)
    run_decode_check(ctx, case, W=1)
    case.fill_payloads()
    run_decode_check(ctx, case, W=4, wd=0.1)


# ---- budgets between 32 and 64 on the wavefront kernels: the threshold bound comes from two maxima per lane, the
#      candidate list is longer than the wavefront and is ranked in blocks of 64 -------------------------------------
@pytest.mark.parametrize("s,k", [(64, 33), (64, 48), (64, 56), (64, 64), (32, 33), (32, 48), (32, 64), (128, 64)])
@pytest.mark.parametrize("grad", ["gauss", "student"])
def test_budgets_above_32_on_the_fast_kernels(ctx, s, k, grad):
    ctx.demo_set_variant(1)
    case = Case([synth.TensorSpec("a", 512, 768)], s, k, W=1, seed=1000 + k, grad=grad,
                grad_dtype=torch.bfloat16 if grad == "student" else torch.float32)
    for st in run_encode_check(ctx, case):
        assert st["chunks"] == case.specs[0].nchunks(s)
    run_decode_check(ctx, case, W=1)


# ---- large sparsity budgets and many workers (generic kernels; k = 64 is the last budget of the s = 64 wavefront kernel)
@pytest.mark.parametrize("s,k", [(64, 64), (64, 65), (64, 256), (32, 200), (128, 256)])
def test_large_k(ctx, s, k):
    ctx.demo_set_variant(1)
    specs = [synth.TensorSpec("a", 2 * s, 3 * s), synth.TensorSpec("v", 8 * s, 0)]
    kk = [k, min(k, s)]
    for sp, kq in zip(specs, kk):     # the order-1 tensor allows k <= s only: one call per tensor
        case = Case([sp], s, kq, W=2, seed=k)
        run_encode_check(ctx, case)
        case.fill_payloads()
        run_decode_check(ctx, case, W=2)


@pytest.mark.parametrize("s,W,k", [(64, 200, 8), (64, 33, 64), (32, 255, 4), (128, 100, 32)])
def test_many_workers_beyond_the_register_payload(ctx, s, W, k):
    ctx.demo_set_variant(1)
    specs = [synth.TensorSpec("a", 2 * s, 2 * s), synth.TensorSpec("v", 2 * s, 0)]
    case = Case(specs, s, k, W=W, param_dtype=torch.bfloat16, seed=W)
    case.fill_payloads()
    run_decode_check(ctx, case, W=W)


# ---- the calls are plain kernel launches once a tensor list has been seen: they can be captured in a HIP graph
def test_step_can_be_captured_and_replayed(ctx):
    ctx.demo_set_variant(1)
    s, k = 64, 32
    a = Case(synth.tensor_set("tiny"), s, k, grad_dtype=torch.bfloat16, param_dtype=torch.bfloat16, seed=50)
    b = Case(synth.tensor_set("tiny"), s, k, grad_dtype=torch.bfloat16, param_dtype=torch.bfloat16, seed=50)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx.demo_step(a.args, BETA, LR, 0.01, s, k, side)      # first sight of the list: descriptor upload
        side.synchronize()
    for t_a, t_b in zip(a.m + a.x, b.m + b.x):                   # back to the common start
        t_a.copy_(t_b)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ctx.demo_step(a.args, BETA, LR, 0.01, s, k, torch.cuda.current_stream())
    for step in range(3):
        a.new_grads(step + 1)
        b.new_grads(step + 1)
        torch.cuda.synchronize()
        graph.replay()
        ctx.demo_step(b.args, BETA, LR, 0.01, s, k)            # eager, between the replays
        torch.cuda.synchronize()
        sa, sb = a.snapshot(), b.snapshot()
        for key in ("m", "x", "idx", "val"):
            for ta, tb in zip(sa[key], sb[key]):
                assert np.array_equal(ta, tb), (step, key)


# ---- payload arrays that are only 4-byte aligned (views into a larger buffer) take the narrower loads -----------
@pytest.mark.parametrize("s,W,k", [(64, 64, 32), (64, 8, 32), (32, 16, 32), (64, 100, 8), (64, 130, 12), (32, 100, 4)])
def test_payload_arrays_with_4_byte_alignment(ctx, s, W, k):
    ctx.demo_set_variant(1)
    specs = [synth.TensorSpec("a", 192, 128), synth.TensorSpec("v", 256, 0)]
    base = Case(specs, s, k, W=W, param_dtype=torch.bfloat16, grad_dtype=torch.bfloat16, seed=60)
    # rebuild the argument list with idx / val as views that start one element into a padded buffer
    idx2, val2 = [], []
    for i, v in zip(base.idx, base.val):
        bi = torch.zeros(i.numel() + 4, dtype=torch.int32, device=i.device)
        bv = torch.zeros(v.numel() + 4, dtype=torch.float32, device=v.device)
        idx2.append(bi[1:1 + i.numel()].view(i.shape))
        val2.append(bv[1:1 + v.numel()].view(v.shape))
        assert idx2[-1].data_ptr() % 16 == 4
    base.idx, base.val = idx2, val2
    base.args = B.TensorList([B.TensorArgs(g, m, x, i, v) for g, m, x, i, v in zip(base.g, base.m, base.x, base.idx, base.val)])
    run_encode_check(ctx, base)
    base.fill_payloads()
    run_decode_check(ctx, base, W=W)


# ---- tensors of different dtypes in one call: one launch per (gradient dtype, parameter dtype) group --------------
@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("s", [32, 64, 128])
def test_mixed_dtypes_in_one_list(ctx, s, variant):
    ctx.demo_set_variant(variant)
    specs = [synth.TensorSpec("a", 256, 384), synth.TensorSpec("b", 384, 128), synth.TensorSpec("v", 256, 0),
             synth.TensorSpec("c", 128, 256), synth.TensorSpec("d", 256, 256), synth.TensorSpec("w", 128, 0)]
    k, W = 8, 3
    case = Case(specs, s, k, W=W, seed=61)
    # four dtype combinations among the order-2 tensors, interleaved in the list; one bf16 vector
    for ti, (gb, xb) in {1: (True, True), 3: (True, False), 4: (False, True), 5: (True, True)}.items():
        if gb:
            case.g[ti] = case.g[ti].to(torch.bfloat16)
        if xb:
            case.x[ti] = case.x[ti].to(torch.bfloat16)
    case.args = B.TensorList([B.TensorArgs(g, m, x, i, v) for g, m, x, i, v in zip(case.g, case.m, case.x, case.idx, case.val)])
    before = case.snapshot()
    ctx.demo_encode(case.args, BETA, s, k)
    torch.cuda.synchronize()
    after = case.snapshot()
    for ti in range(len(specs)):
        C.check_encode(before["m"][ti], before["g"][ti], BETA, s, k, after["idx"][ti][0], after["val"][ti][0], after["m"][ti])
    case.fill_payloads()
    before = case.snapshot()
    ctx.demo_decode(case.args, W, LR, 0.0, s, k)
    torch.cuda.synchronize()
    after = case.snapshot()
    for ti in range(len(specs)):
        pd = "bf16" if case.x[ti].dtype == torch.bfloat16 else "f32"
        C.check_decode(before["x"][ti], before["idx"][ti], before["val"][ti], LR, 0.0, s, pd, after["x"][ti])
    ctx.demo_set_variant(1)


# ---- s = 64, k = 32: worker counts that are multiples of 8 read the payload with 16-byte loads ------------------
# (variant 1: the full-product instance on the float16 matrix pipe; variant 2: the mirror-folded float32 instances)
@pytest.mark.parametrize("variant", [1, 2])
@pytest.mark.parametrize("W", [8, 16, 24, 40, 56, 12, 63])
@pytest.mark.parametrize("pdt", [torch.float32, torch.bfloat16])
def test_s64_decode_worker_counts(ctx, W, pdt, variant):
    ctx.demo_set_variant(variant)
    specs = [synth.TensorSpec("a", 192, 320), synth.TensorSpec("b", 64, 64), synth.TensorSpec("v", 128, 0)]
    case = Case(specs, 64, 32, W=W, param_dtype=pdt, seed=200 + W)
    case.fill_payloads()
    run_decode_check(ctx, case, W=W, wd=0.01)
    ctx.demo_set_variant(1)


# ---- s = 64, other budgets: k a multiple of 4 (16-byte loads of four pairs), of 2 (8-byte loads), odd (one pair) ----
@pytest.mark.parametrize("W,k", [(64, 16), (64, 8), (64, 4), (64, 2), (37, 12), (100, 6), (32, 64), (5, 32), (21, 20),
                                 (64, 3), (33, 2), (128, 16), (17, 4),
                                 # one pair per load with more than 64 workers (odd k)
                                 (200, 3), (100, 1), (400, 5), (65, 31), (40, 51),
                                 # more than 2048 pairs per chunk: streamed in rounds (k a multiple of 4), else generic
                                 (128, 32), (255, 32), (100, 24), (70, 36), (130, 16), (513, 4), (90, 30)])
@pytest.mark.parametrize("variant", [1, 2])
@pytest.mark.parametrize("pdt", [torch.float32, torch.bfloat16])
def test_s64_decode_budgets(ctx, W, k, pdt, variant):
    ctx.demo_set_variant(variant)
    specs = [synth.TensorSpec("a", 192, 320), synth.TensorSpec("b", 64, 64), synth.TensorSpec("v", 128, 0)]
    case = Case(specs, 64, k, W=W, param_dtype=pdt, seed=300 + W + k)
    case.fill_payloads()
    st = run_decode_check(ctx, case, W=W, wd=0.01)
    assert sum(x["elements"] for x in st) == sum(sp.numel for sp in specs)
    ctx.demo_set_variant(1)


@pytest.mark.parametrize("variant", [1, 2])
@pytest.mark.parametrize("pdt", [torch.float32, torch.bfloat16])
def test_s64_decode_when_every_worker_names_the_same_coefficients(ctx, pdt, variant):
    # W equal pairs per coefficient: the sums reach W times the largest value, the top of the block fixed point and of
    # the float16 range the full products are scaled to
    ctx.demo_set_variant(variant)
    W, k = 64, 32
    specs = [synth.TensorSpec("a", 192, 320), synth.TensorSpec("v", 128, 0)]
    case = Case(specs, 64, k, W=W, param_dtype=pdt, seed=77)
    case.fill_payloads()
    for ti in range(len(specs)):
        case.idx[ti][:] = case.idx[ti][0:1]
        case.val[ti][:] = case.val[ti][0:1].abs()
    run_decode_check(ctx, case, W=W)
    ctx.demo_set_variant(1)


# ---- the context caches a few descriptor tables: more distinct tensor lists than that still work, and a list
#      that was evicted is simply uploaded again ------------------------------------------------------------------
def test_many_distinct_tensor_lists(ctx):
    ctx.demo_set_variant(1)
    s, k = 64, 8
    cases = [Case([synth.TensorSpec("a", 64 * (1 + i % 3), 128), synth.TensorSpec("v", 64 * (1 + i % 2), 0)], s, k, seed=300 + i)
             for i in range(12)]
    for rnd in range(2):
        for case in cases:
            case.new_grads(rnd)
            run_encode_check(ctx, case)


# ---- a list of 1500 small tensors (a model of many small layers): descriptor tables of several upload launches, the
#      tensor walk of the persistent kernels at nearly every work item ---------------------------------------------------
@pytest.mark.parametrize("s", [32, 64, 128])
def test_list_of_1500_small_tensors(ctx, s):
    ctx.demo_set_variant(1)
    k = 4
    specs = []
    for i in range(1500):
        if i % 5 == 4:
            specs.append(synth.TensorSpec(f"v{i}", 128 * (1 + i % 2), 0))
        else:
            specs.append(synth.TensorSpec(f"a{i}", 128 * (1 + i % 2), 128 * (1 + (i // 2) % 3)))
    case = Case(specs, s, k, W=2, seed=77)
    run_encode_check(ctx, case)
    run_decode_check(ctx, case, W=2)


# ---- non-finite inputs: the result for the chunks that hold them is undefined, but the call returns and every other
#      chunk comes out as it does without them (no loop of any kernel depends on the data for its end) --------------------
@pytest.mark.parametrize("s", [32, 64, 128])
def test_non_finite_inputs_stay_in_their_chunks(ctx, s):
    ctx.demo_set_variant(1)
    specs = [synth.TensorSpec("a", 256, 384), synth.TensorSpec("v", 4 * s, 0)]
    k, W = 8, 4
    clean = Case(specs, s, k, W=W, seed=77)
    dirty = Case(specs, s, k, W=W, seed=77)
    for c in (clean, dirty):
        c.fill_payloads()
    # one chunk of the matrix (its top-left one) and the first chunk of the vector get NaN / Inf / -Inf
    dirty.g[0][0, 0] = float("nan")
    dirty.g[0][1, 2] = float("inf")
    dirty.m[0][2, 1] = float("-inf")
    dirty.g[1][0] = float("nan")
    dirty.val[0][1, 0, 0] = float("nan")
    dirty.val[0][2, 0, 1] = float("inf")
    dirty.val[1][0, 0, 0] = float("nan")
    for c in (clean, dirty):
        ctx.demo_encode(c.args, BETA, s, k)
    torch.cuda.synchronize()
    nch_cols = 384 // s

    def other_chunks(t):            # everything but chunk (0, 0)
        keep = torch.ones_like(t, dtype=torch.bool)
        keep[:s, :s] = False
        return t[keep]
    assert torch.equal(other_chunks(dirty.m[0]), other_chunks(clean.m[0]))
    assert torch.equal(dirty.idx[0][0, 1:], clean.idx[0][0, 1:]) and torch.equal(dirty.val[0][0, 1:], clean.val[0][0, 1:])
    assert torch.equal(dirty.m[1][s:], clean.m[1][s:])
    # decode with the payloads as filled (worker slot 0 was overwritten by the encode above: make it equal again)
    dirty.idx[0][0].copy_(clean.idx[0][0]); dirty.val[0][0].copy_(clean.val[0][0])
    dirty.idx[1][0].copy_(clean.idx[1][0]); dirty.val[1][0].copy_(clean.val[1][0])
    for c in (clean, dirty):
        ctx.demo_decode(c.args, W, LR, 0.0, s, k)
    torch.cuda.synchronize()
    assert torch.equal(other_chunks(dirty.x[0]), other_chunks(clean.x[0]))
    assert torch.equal(dirty.x[1][s:], clean.x[1][s:])
    assert nch_cols >= 3


# ---- a caller whose buffers move every step presents a new list each time: beyond the cached lists the tables are
#      rewritten in reused memory by a kernel on the call's stream (also from a second stream) ----------------------
@pytest.mark.parametrize("s", [32, 64, 128])
def test_buffers_that_move_every_step(ctx, s):
    ctx.demo_set_variant(1)
    k = 8
    cases = [Case(synth.tensor_set("tiny"), s, k, W=2, grad_dtype=torch.bfloat16, param_dtype=torch.bfloat16, seed=70 + i)
             for i in range(11)]
    side = torch.cuda.Stream()
    for rep in range(2):
        for i, case in enumerate(cases):                 # same shapes and dtypes, other addresses, every call
            on_side = (i % 4 == 3)
            if on_side:
                side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side if on_side else torch.cuda.current_stream()):
                before = case.snapshot()
                ctx.demo_encode(case.args, BETA, s, k, torch.cuda.current_stream())
                torch.cuda.current_stream().synchronize()
                after = case.snapshot()
            torch.cuda.synchronize()
            for ti in range(len(case.specs)):
                C.check_encode(before["m"][ti], before["g"][ti], BETA, s, k, after["idx"][ti][0], after["val"][ti][0],
                               after["m"][ti])
            case.fill_payloads()
            run_decode_check(ctx, case, W=2)
            case.new_grads(rep + 1)


# ---- measurement hooks: cut-down copies of the s = 64 encode kernel and the stream probes run and leave the
#      library in its ordinary state -------------------------------------------------------------------------------
def test_debug_stages_and_stream_probes(ctx):
    ctx.demo_set_variant(1)
    specs = [synth.TensorSpec("a", 512, 1024)]
    case = Case(specs, 64, 32, grad_dtype=torch.bfloat16, seed=3)
    for stage in (1, 2, 3):
        ctx.demo_debug_set_encode_stage(stage)
        ctx.demo_encode(case.args, BETA, 64, 32)
        f32 = Case(specs, 64, 32, seed=3)
        with pytest.raises(B.DemoError) as e:
            ctx.demo_encode(f32.args, BETA, 64, 32)          # the copies exist for bfloat16 gradients only
        assert e.value.status == B.DEMO_ERR_UNSUPPORTED
        with pytest.raises(B.DemoError) as e:
            ctx.demo_encode(case.args, BETA, 128, 32)
        assert e.value.status == B.DEMO_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    ctx.demo_debug_set_encode_stage(0)
    with pytest.raises(B.DemoError):
        ctx.demo_debug_set_encode_stage(4)
    case = Case(specs, 64, 32, grad_dtype=torch.bfloat16, seed=4)
    run_encode_check(ctx, case)
    # ... and of the decode kernel
    dcase = Case(specs, 64, 32, W=8, param_dtype=torch.bfloat16, seed=5)
    dcase.fill_payloads(exact=False)
    for stage in (1, 2):
        ctx.demo_debug_set_decode_stage(stage)
        ctx.demo_decode(dcase.args, 8, LR, 0.0, 64, 32)
        with pytest.raises(B.DemoError) as e:
            ctx.demo_decode(dcase.args, 1, LR, 0.0, 64, 32)      # W k <= 64 runs on another kernel
        assert e.value.status == B.DEMO_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    ctx.demo_debug_set_decode_stage(0)
    with pytest.raises(B.DemoError):
        ctx.demo_debug_set_decode_stage(3)
    dcase = Case(specs, 64, 32, W=8, param_dtype=torch.bfloat16, seed=6)
    dcase.fill_payloads(exact=False)
    run_decode_check(ctx, dcase, W=8)
    src = torch.randn(1 << 20, device=DEV)
    for mode in range(5):
        dst = torch.zeros(1 << 20, device=DEV)
        ctx.demo_stream_probe(dst, src, mode)
        torch.cuda.synchronize()
        if mode < 2:
            assert torch.equal(dst, src)
    with pytest.raises(B.DemoError):
        ctx.demo_stream_probe(dst, src, 5)
