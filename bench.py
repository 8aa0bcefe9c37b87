#!/usr/bin/env python3
"""Benchmark of DeMo's per-step compression path on one MI355X.

One step = one pass of the whole hot path over the 1B-like tensor set:
  demo_encode  (bf16 gradients, fp32 momentum, s = 64, k = 32; writes worker slot 0
                of the payload buffers)
  demo_decode  (W = 64 workers' payloads: slot 0 from the encode above, 63 synthetic;
                bf16 parameters, lr = 1e-3)
Inputs are synthetic and resident in HBM before the timed region starts.

Prints ONE JSON line: whole-step throughput in GB/s of algorithmic traffic (and
params/s); the roofline record of the dominant kernel measured with HIP events on
the launch stream inside the timed region, against the published HBM peak and against
the issued fp32 MFMA work, the bound being whichever fraction is larger; the ceilings
this GPU's memory system reaches for the kernels' own traffic (measured after the timed
region); the payload size; and the float64 CPU oracle timed on all host cores on a stated
sample of the same workload.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix, published
MFMA_F16_PEAK_TFLOPS = 2500.0   # MI355X dense fp16 matrix, published
S, K, W = 64, 32, 64
BETA, LR, WD = 0.999, 1e-3, 0.0
CPU_SAMPLE_FRACTION = 0.30


def algorithmic_bytes(specs, s, k, W, grad_bytes, param_bytes):
    """Bytes the method itself must move per step (every tensor read once, written once)."""
    enc2 = enc1 = dec2 = dec1 = 0
    p2 = p1 = 0
    for sp in specs:
        n, pairs = sp.numel, sp.nchunks(s) * k
        e = n * (grad_bytes + 4 + 4) + pairs * 8            # g read, m read, m write, payload write
        d = n * (2 * param_bytes) + W * pairs * 8           # x read, x write, W payloads read
        if sp.cols == 0:
            enc1 += e; dec1 += d; p1 += n
        else:
            enc2 += e; dec2 += d; p2 += n
    return {"enc2d": enc2, "enc1d": enc1, "dec2d": dec2, "dec1d": dec1, "params2d": p2, "params1d": p1}


def source_hash():
    """Hash of the kernel sources: profiles/ records made with other sources are not quoted."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2411_19870_amd", "csrc")
    for name in sorted(os.listdir(d)):
        with open(os.path.join(d, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


F32_MFMA_FLOP = 2048.0      # v_mfma_f32_16x16x4_f32
HALF_MFMA_FLOP = 16384.0    # v_mfma_f32_16x16x32_f16


def mfma_work_per_launch(kernel, s, k, W, nchunks2, idx_tensors, projection="dct", variant=1):
    """Matrix-core work one launch of the order-2 kernel issues, by instruction type, from the kernels' own instruction
    counts: {"f32": flops of v_mfma_f32_16x16x4_f32, "f16": ... of v_mfma_f32_16x16x32_f16 (float32 operands split
    into two float16 parts, three instructions per 16 x 16 tile and 32 contraction indices)}; None where the count depends on the data in a
    way this function does not follow (the few-pairs decode kernels) or the generic kernels run.  For encode the
    float32 reconstruction chain depends on how many selected coefficients fall into each class."""
    import torch
    if variant == 0:
        return None
    dct = projection == "dct"
    if not dct and s != 64:
        return None                                                        # generic kernels
    if kernel == "dec2d":
        if s == 32:
            return {"f32": 32.0 * F32_MFMA_FLOP * nchunks2}                # both products, 1/2 of dense, per chunk
        if W * k <= 64 and dct:
            return None                                                    # the few-pairs kernels: data dependent
        if s == 64:
            if W * k <= 2048 and variant == 1:
                return {"f16": 192.0 * HALF_MFMA_FLOP * nchunks2}          # full products, 96 instructions each
            return {"f32": 192.0 * F32_MFMA_FLOP * nchunks2} if dct else None   # mirror folds: 3/8 of dense
        return {"f16": 768.0 * HALF_MFMA_FLOP * nchunks2}                  # s = 128: four 64^3 quadrant products, twice
    if s == 64 and dct:
        # products with the mirror folds; reconstruction by classes of u: 0 mod 4, 2 mod 4 (4 MFMAs per step of four
        # coefficients), odd (8 per step)
        recon = 0.0
        for idx in idx_tensors:
            u = (idx[0].to(torch.int64) >> 6)
            c0 = ((u & 3) == 0).sum(1)
            c1 = ((u & 3) == 2).sum(1)
            c2 = ((u & 1) == 1).sum(1)
            recon += float((4 * ((c0 + 3) // 4) + 4 * ((c1 + 3) // 4) + 8 * ((c2 + 3) // 4)).sum())
        return {"f32": (192.0 * nchunks2 + recon) * F32_MFMA_FLOP}
    if s == 64:
        # full products of operands split into two float16 parts, 96 instructions each; reconstruction in float32,
        # 16 per four kept coefficients
        return {"f16": 192.0 * HALF_MFMA_FLOP * nchunks2, "f32": 16.0 * math.ceil(k / 4.0) * F32_MFMA_FLOP * nchunks2}
    if s == 32:
        return {"f32": (32.0 + 4.0 * math.ceil(k / 4.0)) * F32_MFMA_FLOP * nchunks2}   # four MFMAs per step of four coefficients
    # s = 128: four quadrant products, twice; reconstruction: 8 wavefronts x 2 tiles x 4 classes per step of four
    # coefficients of the fullest class (u % 2, v % 2)
    recon = 0.0
    for idx in idx_tensors:
        i64 = idx[0].to(torch.int64)
        cls = ((i64 >> 6) & 2) | (i64 & 1)
        nmax = torch.stack([(cls == c).sum(1) for c in range(4)]).max(0).values
        recon += float((64 * ((nmax + 3) // 4)).sum())
    return {"f16": 768.0 * HALF_MFMA_FLOP * nchunks2, "f32": recon * F32_MFMA_FLOP}


def _cpu_worker_init():
    """One thread per worker process: the pool has one process per core, and numerical libraries that each start
    a thread per core would oversubscribe the machine sixteen-fold."""
    import torch
    torch.set_num_threads(1)
    try:
        import threadpoolctl
        global _cpu_thread_limit
        _cpu_thread_limit = threadpoolctl.threadpool_limits(1)
    except ImportError:
        pass


def _cpu_job(job):
    """One tensor slab of the CPU baseline: oracle encode + W-worker decode (runs in a worker process)."""
    import numpy as np
    import torch
    from oracle import demo_oracle as O
    from paper_2411_19870_amd import synth
    name, rows, cols, ti, seed, s, k, Wn = job
    sp = synth.TensorSpec(name, rows, cols)
    g = synth.gaussian(sp, 1e-2, seed, ti, 0, "grad", dtype=torch.bfloat16).double().numpy()
    m = synth.gaussian(sp, 1e-3, seed, ti, 0, "mom").double().numpy()
    x = synth.gaussian(sp, 0.02, seed, ti, 0, "param", dtype=torch.bfloat16).double().numpy()
    idx, val = synth.payload_fast(sp, s, k, Wn, 1e-3, seed, ti)
    idx, val = idx.numpy(), val.numpy()
    t0 = time.perf_counter()
    e = O.encode(m, g, float(np.float32(BETA)), s, k)
    idx[0], val[0] = e["idx"], e["val"].astype(np.float32)
    O.decode(x, idx, val, LR, WD, s, "bf16")
    return time.perf_counter() - t0


def cpu_baseline(specs, seed, s, k, Wn, ab_step_bytes, nparams):
    """The oracle as it stands, on every host core this process may use: one encode + W-worker decode pass over a
    slab of the first CPU_SAMPLE_FRACTION of the rows of every tensor of the workload (rounded up to whole chunks),
    cut into jobs of about 2^20 parameters for a pool of worker processes.  The rate is that of the timed pass; input generation in the
    workers is outside the oracle's timers but inside the wall-clock, so the wall-clock rate is the lower one."""
    import multiprocessing
    from concurrent.futures import ProcessPoolExecutor
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    jobs, sample_params = [], 0
    for ti, sp in enumerate(specs):
        rows = min(sp.rows, max(s, int(math.ceil(sp.rows * CPU_SAMPLE_FRACTION / s)) * s))
        # pieces of about 2^20 parameters (whole chunk rows), so that the cores finish together
        piece = max(s, ((1 << 20) // (sp.cols or 1)) // s * s)
        for r0 in range(0, rows, piece):
            jobs.append((sp.name, min(piece, rows - r0), sp.cols, ti, seed + r0, s, k, Wn))
        sample_params += rows * (sp.cols or 1)
    jobs.sort(key=lambda j: -j[1] * (j[2] or 1))            # largest first
    frac = sample_params / nparams
    w0 = time.perf_counter()
    with ProcessPoolExecutor(max_workers=cores, mp_context=multiprocessing.get_context("spawn"),
                             initializer=_cpu_worker_init) as pool:
        list(pool.map(_cpu_job, jobs[-cores:]))             # start the workers (imports) outside the timed pass
        w1 = time.perf_counter()
        busy = sum(pool.map(_cpu_job, jobs))
        w2 = time.perf_counter()
    wall = w2 - w1
    return {
        "value": ab_step_bytes * frac / wall / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
        "params_per_s": sample_params / wall,
        "core_seconds_in_oracle": busy, "wall_s": wall, "pool_start_s": w1 - w0,
        "sample": f"one pass of encode + W={Wn} decode over the first {100 * CPU_SAMPLE_FRACTION:.0f} % of the rows of each "
                  f"of the {len(specs)} tensors ({sample_params} parameters, {100 * frac:.1f} % of the workload), "
                  f"one single-threaded process per core, wall-clock of the pass",
    }


def main():
    global S, K, W
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="1b", choices=["1b", "300m", "single"])
    ap.add_argument("--variant", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the memory-system probes after the timed region")
    ap.add_argument("--seed", type=int, default=0)
    # other operating points of the same path (the headline configuration is the default)
    ap.add_argument("--s", type=int, default=S, choices=[32, 64, 128], help="chunk size")
    ap.add_argument("--k", type=int, default=K, help="coefficients kept per chunk")
    ap.add_argument("--workers", type=int, default=W, help="payloads decoded per step")
    ap.add_argument("--projection", default="dct", choices=["dct", "random", "identity"],
                    help="projection matrix: the DCT, or the ablation's random orthonormal matrix (seed = step 0) / identity")
    a = ap.parse_args()
    headline = (a.s, a.k, a.workers) == (S, K, W) and a.projection == "dct"
    S, K, W = a.s, a.k, a.workers
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (the W workers' payloads are synthesised on-device); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2411_19870_amd import binding as B
    from paper_2411_19870_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    specs = synth.tensor_set(a.workload)
    gdt = torch.bfloat16 if a.workload == "1b" else torch.float32
    pdt = gdt
    gb = 2 if gdt == torch.bfloat16 else 4

    tensors = []
    for ti, sp in enumerate(specs):
        g = synth.gaussian(sp, 1e-2, a.seed, ti, 0, "grad", dtype=gdt, device=dev)
        m = synth.gaussian(sp, 1e-3, a.seed, ti, 0, "mom", device=dev)
        x = synth.gaussian(sp, 0.02, a.seed, ti, 0, "param", dtype=pdt, device=dev)
        idx, val = synth.payload_fast(sp, S, K, W, 1e-3, a.seed, ti, device=dev)
        tensors.append(B.TensorArgs(g, m, x, idx, val))
    tl = B.TensorList(tensors)
    ab = algorithmic_bytes(specs, S, K, W, gb, gb)
    step_bytes = ab["enc2d"] + ab["enc1d"] + ab["dec2d"] + ab["dec1d"]
    nparams = ab["params2d"] + ab["params1d"]
    nchunks2 = sum(sp.nchunks(S) for sp in specs if sp.cols)
    nchunks = sum(sp.nchunks(S) for sp in specs)

    ctx = B.Context()
    ctx.demo_set_variant(a.variant)
    if a.projection == "random":
        ctx.demo_set_basis(S, B.DEMO_BASIS_GRAM_SCHMIDT, synth.projection_draws(S, 0))
    elif a.projection == "identity":
        ctx.demo_set_basis(S, B.DEMO_BASIS_IDENTITY)
    stream = torch.cuda.current_stream()

    def step():
        ctx.demo_encode(tl, BETA, S, K, stream)
        ctx.demo_decode(tl, W, LR, WD, S, K, stream)

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    ctx.demo_set_timing(True)                 # per-kernel HIP events on the launch stream, no syncs
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / a.steps
    kms = {}
    for which, name in enumerate(("enc2d", "enc1d", "dec2d", "dec1d")):
        try:
            kms[name] = ctx.demo_last_kernel_ms(which)
        except B.DemoError:
            kms[name] = None
    ctx.demo_set_timing(False)

    def timed(fn, reps, slot):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        ctx.demo_set_timing(True)
        for _ in range(reps):
            fn()
        ms = ctx.demo_last_kernel_ms(slot)
        ctx.demo_set_timing(False)
        return ms

    dom = "enc2d" if (kms["enc2d"] or 0) >= (kms["dec2d"] or 0) else "dec2d"
    achieved = ab[dom] / (kms[dom] * 1e-3) / 1e9
    hbm_frac = achieved / HBM_PEAK_GBS
    work = mfma_work_per_launch(dom, S, K, W, nchunks2, [t.idx for t, sp in zip(tensors, specs) if sp.cols],
                                a.projection, a.variant)
    peaks = {"f32": MFMA_F32_PEAK_TFLOPS, "f16": MFMA_F16_PEAK_TFLOPS}
    if work:
        # the fraction is the time the matrix pipe needs at each instruction type's peak over the launch time
        pipe_s = sum(f / (peaks[ty] * 1e12) for ty, f in work.items())
        total_flops = sum(work.values())
        mfma_frac = pipe_s / (kms[dom] * 1e-3)
        mfma_tflops = total_flops / (kms[dom] * 1e-3) / 1e12
        mfma_peak = total_flops / pipe_s / 1e12
    else:
        mfma_tflops = mfma_frac = None
        mfma_peak = MFMA_F32_PEAK_TFLOPS
    other = "dec2d" if dom == "enc2d" else "enc2d"
    work_other = mfma_work_per_launch(other, S, K, W, nchunks2, [], a.projection, a.variant) if other == "dec2d" else None
    split_types = sorted({ty for wk in (work, work_other) if wk for ty in wk if ty != "f32"})
    bound = "mfma" if (mfma_frac or 0.0) > hbm_frac else "hbm"
    roof = {"bound": bound, "kernel": dom, "avg_launch_ms": kms[dom],
            "hbm": {"achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_frac,
                    "algorithmic_bytes_per_launch": ab[dom]},
            "mfma": {"achieved": mfma_tflops, "peak": mfma_peak, "unit": "TFLOP/s", "frac": mfma_frac,
                     "issued_fp32_mfma_flops_per_launch": (work or {}).get("f32"),
                     "issued_f16_mfma_flops_per_launch": (work or {}).get("f16"),
                     "peak_fp32": MFMA_F32_PEAK_TFLOPS, "peak_f16": MFMA_F16_PEAK_TFLOPS},
            "traffic": None, "traffic_source": None}
    roof.update({"achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_frac} if bound == "hbm" else
                {"achieved": mfma_tflops, "peak": mfma_peak, "unit": "TFLOP/s", "frac": mfma_frac})

    out = {
        "metric": "DeMo encode+decode throughput at 1B shape" if a.workload == "1b" and headline
                  else f"DeMo encode+decode throughput ({a.workload}, s={S}, k={K}, W={W}, projection {a.projection})",
        "value": step_bytes / (ms_step * 1e-3) / 1e9, "unit": "GB/s",
        "params_per_s": nparams / (ms_step * 1e-3),
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if not split_types else "f32 (products of float32 operands split into parts on the "
                 + " and ".join(split_types) + " matrix pipe, float32 accumulation)",
        "data": "synthetic",
        "config": {"workload": f"{a.workload}-like tensor set: encode (grad {'bf16' if gb == 2 else 'f32'}, momentum f32) "
                               f"+ decode of W={W} payloads (param {'bf16' if gb == 2 else 'f32'})",
                   "tensors": len(specs), "params": nparams, "s": S, "k": K, "W": W, "beta": BETA, "lr": LR,
                   "kernel_variant": a.variant, "projection": a.projection},
        "roofline": roof,
        "kernels_ms": kms,
        "kernels_gbs": {k: (ab[k] / (v * 1e-3) / 1e9 if v else None) for k, v in kms.items()},
        "encode_params_per_s": nparams / (((kms["enc2d"] or 0) + (kms["enc1d"] or 0)) * 1e-3),
        "decode_params_per_s": nparams / (((kms["dec2d"] or 0) + (kms["dec1d"] or 0)) * 1e-3),
        "algorithmic_bytes_per_step": step_bytes,
        # what one worker sends per step (k pairs of int32 index + float32 value per chunk) and what the decode reads
        "payload_bytes_per_step": {"sent_per_worker": nchunks * K * 8, "received": W * nchunks * K * 8},
    }

    # ---- memory-system ceilings, measured after the timed region -------------------------------------------------
    if not a.no_ceilings:
        probe_src = torch.empty(1 << 30, dtype=torch.float32, device=dev).normal_()     # 4 GiB
        probe_dst = torch.empty_like(probe_src)
        nb = probe_src.numel() * 4
        probe_ms = timed(lambda: ctx.demo_copy_probe(probe_dst, probe_src, stream), 5, 1)
        out["copy_probe"] = {"bytes_moved": 2 * nb, "ms": probe_ms, "gbs": 2 * nb / (probe_ms * 1e-3) / 1e9}
        ceil = {"unit": "GB/s", "bytes_per_probe": nb,
                "note": "stream probes in the launch shape of the wavefront kernels (one 512-thread workgroup per CU, "
                        "16 B per lane, 8 accesses in flight), 4 GiB each"}
        for mode, name, moved in ((1, "copy_nontemporal", 2), (0, "copy_default_policy", 2),
                                  (2, "read_only", 1), (3, "write_only", 1)):
            ms = timed(lambda: ctx.demo_stream_probe(probe_dst, probe_src, mode, stream), 5, 1)
            ceil[name] = moved * nb / (ms * 1e-3) / 1e9
        del probe_src, probe_dst
        # the dominant kernel's own traffic mix at the rates the probes reach for pure reads and pure writes
        rd = ab[dom] - (ab["params2d"] * 4 + nchunks2 * K * 8 if dom == "enc2d" else ab["params2d"] * gb)
        wr = ab[dom] - rd
        t_mix = rd / ceil["read_only"] + wr / ceil["write_only"]
        ceil["kernel_mix_serialised"] = ab[dom] / t_mix
        if dom == "enc2d" and S == 64 and gb == 2 and a.variant == 1 and K <= 64 and a.projection == "dct":
            # the encode kernel's own access pattern with the transform taken out (loads with the cross-chunk
            # prefetch, momentum update, store of m, k payload pairs per chunk)
            ctx.demo_debug_set_encode_stage(1)
            ms = timed(lambda: ctx.demo_encode(tl, BETA, S, K, stream), 5, 0)
            ctx.demo_debug_set_encode_stage(0)
            ceil["kernel_access_pattern_only"] = ab[dom] / (ms * 1e-3) / 1e9
            ceil["kernel_access_pattern_only_ms"] = ms
        best = ceil.get("kernel_access_pattern_only", ceil["kernel_mix_serialised"])
        roof["hbm"]["frac_of_peak"] = hbm_frac
        roof["hbm"]["frac_of_measured"] = achieved / best
        roof["hbm"]["measured_ceiling"] = best
        out["hbm_ceiling"] = ceil

    # HBM traffic of the dominant kernel from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs (scaled by the copy probe)
    # recorded under profiles/: quoted only when that record was made with these kernel sources
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{a.workload}.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            rec = json.load(f)
        same = rec.get("source_hash") == source_hash()
        if headline and rec.get("variant") == a.variant and dom in rec.get("kernels", {}) and same:
            roof["traffic"] = rec["kernels"][dom]["hbm_bytes_per_launch"]
            roof["traffic_source"] = f"profiles/hbm_traffic_{a.workload}.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs " \
                                     f"of these kernel sources, hash {rec['source_hash']})"
        elif not same:
            roof["traffic_source"] = f"profiles/hbm_traffic_{a.workload}.json is from other kernel sources: not quoted"
        else:
            roof["traffic_source"] = "no counter record for this operating point (the records cover the headline configuration of each workload)"
    else:
        roof["traffic_source"] = "no counter record for this workload"
    ctx.close()
    del tensors, tl
    torch.cuda.empty_cache()
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(specs, a.seed, S, K, W, step_bytes, nparams)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
