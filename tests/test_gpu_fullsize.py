"""Parity at the workloads' full sizes, in the launch configurations the benchmark times: the 1B-like and
the 300M-like tensor sets.  Every chunk of every order-1 tensor and at least 5 % of the chunks of every
order-2 tensor (first, last and grid hand-over chunks among them) are checked element by element against
the float64 oracle, which runs in a pool of worker processes; properties that hold at any size (index range
and distinctness, energy split of the orthonormal transform) are checked on every tensor."""
import numpy as np
import pytest
import torch

from paper_2411_19870_amd import binding as B
from paper_2411_19870_amd import synth
from tests import fullsize_tools as F

pytestmark = pytest.mark.gpu

BETA, LR = 0.999, 1e-3
DEV = "cuda:0"
FRAC = 0.05


@pytest.fixture(scope="module")
def pool():
    p = F.make_pool()
    yield p
    p.shutdown(cancel_futures=True)


def make_set(name, s, k, W, gdt, pdt, seed, grad=True):
    specs = synth.tensor_set(name) if isinstance(name, str) else list(name)
    tensors = []
    for ti, sp in enumerate(specs):
        g = synth.gaussian(sp, 1e-2, seed, ti, 0, "grad", dtype=gdt, device=DEV) if grad else \
            torch.empty(sp.shape, dtype=gdt, device=DEV)
        m = synth.gaussian(sp, 1e-3, seed, ti, 0, "mom", device=DEV) if grad else \
            torch.zeros(sp.shape, dtype=torch.float32, device=DEV)
        x = synth.gaussian(sp, 0.02, seed, ti, 0, "param", dtype=pdt, device=DEV)
        if W > 1:
            idx, val = synth.payload_fast(sp, s, k, W, 1e-3, seed, ti, device=DEV)
        else:
            nch = sp.nchunks(s)
            idx = torch.zeros((1, nch, k), dtype=torch.int32, device=DEV)
            val = torch.zeros((1, nch, k), dtype=torch.float32, device=DEV)
        tensors.append(B.TensorArgs(g, m, x, idx, val))
    return specs, tensors


def gather(tensors, specs, s, picks, field):
    return {ti: F.gather_blocks(getattr(tensors[ti], field), specs[ti], s, ch) for ti, ch in picks.items()}


def submit_encode(pool, tally, specs, tensors, s, k, picks, m0, g0, tag, P=None):
    m1 = gather(tensors, specs, s, picks, "mom")
    for ti, ch in picks.items():
        ci = torch.as_tensor(ch, device=DEV)
        idx = tensors[ti].idx[0][ci].cpu().numpy()
        val = tensors[ti].val[0][ci].cpu().numpy()
        for a, b in F.split(len(ch), specs[ti].chunk_elems(s)):
            tally.add(pool.submit(F.encode_job, m0[ti][a:b], g0[ti][a:b], BETA, s, k, idx[a:b], val[a:b], m1[ti][a:b],
                                  f"{tag} encode {specs[ti].name} chunks {ch[a]}..{ch[b - 1]}", P))


def submit_decode(pool, tally, specs, tensors, s, k, W, picks, x0, pdt, tag, P=None):
    x1 = gather(tensors, specs, s, picks, "param")
    for ti, ch in picks.items():
        ci = torch.as_tensor(ch, device=DEV)
        idx = tensors[ti].idx[:W][:, ci].cpu().numpy()
        val = tensors[ti].val[:W][:, ci].cpu().numpy()
        for a, b in F.split(len(ch), specs[ti].chunk_elems(s) * max(1, W * k // 1024)):
            tally.add(pool.submit(F.decode_job, x0[ti][a:b], idx[:, a:b], val[:, a:b], LR, 0.0, s, pdt, x1[ti][a:b],
                                  f"{tag} decode W={W} {specs[ti].name} chunks {ch[a]}..{ch[b - 1]}", P))


def check_any_size_properties(specs, tensors, s, energy_mid):
    """Indices in range and distinct in every chunk of every tensor; ||beta m + g||^2 = ||val||^2 + ||m'||^2."""
    for ti, t in enumerate(tensors):
        M = specs[ti].chunk_elems(s)
        i0 = t.idx[0]
        assert int(i0.min()) >= 0 and int(i0.max()) < M, specs[ti].name
        if i0.shape[1] > 1:
            srt = i0.sort(dim=1).values
            assert bool((srt[:, 1:] != srt[:, :-1]).all()), specs[ti].name
        e_after = float(t.val[0].double().pow(2).sum() + t.mom.double().pow(2).sum())
        assert abs(e_after - energy_mid[ti]) <= 1e-5 * energy_mid[ti], (specs[ti].name, e_after, energy_mid[ti])


def energy_of_update(tensors):
    return [float((BETA * t.mom.double() + t.grad.double()).pow(2).sum()) for t in tensors]


def sample_report(specs, s, picks):
    n2 = sum(sp.nchunks(s) for sp in specs if sp.cols)
    c2 = sum(len(ch) for ti, ch in picks.items() if specs[ti].cols)
    c1 = sum(len(ch) for ti, ch in picks.items() if not specs[ti].cols)
    return f"{c2} of {n2} order-2 chunks ({100.0 * c2 / n2:.1f} %), all {c1} order-1 chunks"


def encode_then_decodes(pool, name, s, k, Ws, gdt, pdt, seed, projection_step=None):
    """Encode, then one decode per entry of Ws (W = 1 applies the payload just written; larger W the
    synthetic payloads with the encode output in worker slot 0), each checked on the sample.
    projection_step: use the random orthonormal projection matrix of that step instead of the DCT."""
    Wmax = max(Ws)
    specs, tensors = make_set(name, s, k, Wmax, gdt, pdt, seed)
    tl = B.TensorList(tensors)
    ctx = B.Context()
    P = None
    if projection_step is not None:
        from oracle import demo_oracle as O
        draws = synth.projection_draws(s, projection_step)
        ctx.demo_set_basis(s, B.DEMO_BASIS_GRAM_SCHMIDT, draws)
        P = O.gram_schmidt(draws.double().numpy())
    pd = "bf16" if pdt == torch.bfloat16 else "f32"
    picks = F.pick_chunks(specs, s, FRAC, seed)
    tally_e, tally_d = F.Tally(), F.Tally()
    m0, g0 = gather(tensors, specs, s, picks, "mom"), gather(tensors, specs, s, picks, "grad")
    energy_mid = energy_of_update(tensors)
    ctx.demo_encode(tl, BETA, s, k)
    torch.cuda.synchronize()
    tag = (name if isinstance(name, str) else specs[0].name) + f" s={s} k={k}"
    submit_encode(pool, tally_e, specs, tensors, s, k, picks, m0, g0, tag, P)
    check_any_size_properties(specs, tensors, s, energy_mid)
    for W in Ws:
        x0 = gather(tensors, specs, s, picks, "param")
        ctx.demo_decode(tl, W, LR, 0.0, s, k)
        torch.cuda.synchronize()
        submit_decode(pool, tally_d, specs, tensors, s, k, W, picks, x0, pd, tag, P)
    se, sd = tally_e.drain(), tally_d.drain()
    ctx.close()
    label = name if isinstance(name, str) else "+".join(sp.name for sp in specs)
    print(f"{label} s={s} k={k} W={Ws} {gdt} / {pdt}: {sample_report(specs, s, picks)}; encode {se}; decode {sd}")
    del tensors, tl
    torch.cuda.empty_cache()
    return se, sd


# ---- the benchmark's configuration: 1B-like set, bf16 gradients and parameters, s = 64, k = 32, W = 64 ----------
def test_full_size_1b_encode_then_decode(pool):
    encode_then_decodes(pool, "1b", 64, 32, [64], torch.bfloat16, torch.bfloat16, 0)


# ---- 300M-like set with float32 gradients, momentum and parameters: the float32 instances of the wavefront
#      kernels walk their persistent loops (prefetch of the next chunk, tensor boundaries) --------------------------
def test_full_size_300m_fp32(pool):
    encode_then_decodes(pool, "300m", 64, 32, [1, 64], torch.float32, torch.float32, 2)


@pytest.mark.parametrize("s,k,W", [(32, 8, 16), (32, 32, 1), (128, 32, 8)])
def test_full_size_300m_fp32_other_chunk_sizes(pool, s, k, W):
    encode_then_decodes(pool, "300m", s, k, [W], torch.float32, torch.float32, 3)


# ---- the ablation's random orthonormal projection (Gaussian entries, Gram-Schmidt, seed = step number) at full size:
#      the full-product instances of the s = 64 wavefront kernels walk their persistent loops -------------------------
@pytest.mark.parametrize("gdt", [torch.float32, torch.bfloat16])
def test_full_size_300m_random_projection(pool, gdt):
    encode_then_decodes(pool, "300m", 64, 32, [1, 16], gdt, gdt, 4, projection_step=7)


# ---- the widest tensor the library accepts (cols < 2^22): with float32 elements the last rows of a chunk lie just
#      below the 2 GiB that a buffer resource addresses -------------------------------------------------------------
@pytest.mark.parametrize("s", [32, 64, 128])
def test_widest_tensor_the_kernels_accept(pool, s):
    specs = [synth.TensorSpec("wide", 128, B.DEMO_MAX_COLS - 128), synth.TensorSpec("v", 4096, 0)]
    encode_then_decodes(pool, specs, s, 8, [2], torch.float32, torch.float32, 5)


# ---- one tensor of more than 2^31 elements: chunk origins and payload positions need 64-bit arithmetic ------------------
@pytest.mark.parametrize("s", [64, 128])
def test_tensor_of_more_than_2_pow_31_elements(pool, s):
    specs = [synth.TensorSpec("huge", 65536, 32768 + 64 * s)]
    assert specs[0].numel > 2 ** 31
    encode_then_decodes(pool, specs, s, 8, [1], torch.bfloat16, torch.bfloat16, 6)


# ---- stress sweep at full size: heavy-tailed bf16 gradients (exact magnitude ties), momentum carried over 10
#      steps of encode + decode of the worker's own payload; the oracle starts every step from the GPU's momentum --
@pytest.mark.parametrize("s", [32, 64, 128])
@pytest.mark.parametrize("k", [1, 8, 32])
def test_full_size_ten_carried_steps(pool, s, k):
    specs, tensors = make_set("1b", s, k, 1, torch.bfloat16, torch.bfloat16, 1, grad=False)
    tl = B.TensorList(tensors)
    ctx = B.Context()
    tally_e, tally_d = F.Tally(), F.Tally()
    report = ""
    for step in range(10):
        for ti, sp in enumerate(specs):
            tensors[ti].grad.copy_(synth.student_t3(sp, 1e-2, 1, ti, step, "grad", dtype=torch.bfloat16, device=DEV))
        picks = F.pick_chunks(specs, s, FRAC, 1000 * s + 10 * k + step)
        report = sample_report(specs, s, picks)
        m0, g0 = gather(tensors, specs, s, picks, "mom"), gather(tensors, specs, s, picks, "grad")
        x0 = gather(tensors, specs, s, picks, "param")
        energy_mid = energy_of_update(tensors) if step in (0, 9) else None
        ctx.demo_step(tl, BETA, LR, 0.0, s, k)
        torch.cuda.synchronize()
        tag = f"1b s={s} k={k} step {step}"
        submit_encode(pool, tally_e, specs, tensors, s, k, picks, m0, g0, tag)
        submit_decode(pool, tally_d, specs, tensors, s, k, 1, picks, x0, "bf16", tag)
        if energy_mid is not None:
            check_any_size_properties(specs, tensors, s, energy_mid)
        tally_e.drain(keep=64)
        tally_d.drain(keep=64)
    se, sd = tally_e.drain(), tally_d.drain()
    ctx.close()
    print(f"1b s={s} k={k}, 10 carried steps, per step {report}; encode {se}; decode {sd}")
    del tensors, tl
    torch.cuda.empty_cache()
