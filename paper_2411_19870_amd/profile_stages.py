#!/usr/bin/env python3
"""Time attribution of the s = 64 encode and decode kernels on the 1B-like tensor set, and the memory-system
ceilings they are held against: prints markdown tables.

    python -m paper_2411_19870_amd.profile_stages [--k 32] [--reps 10]

Stages are cut-down copies of the kernels selected with demo_debug_set_encode_stage / demo_debug_set_decode_stage
(include/demo_debug.h):
each is timed with HIP events on the launch stream; consecutive differences are the costs of the phases.
The stream probes move 4 GiB in the launch shape of the wavefront kernels.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--k", type=int, default=32)
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--workers", type=int, default=64)
    a = ap.parse_args()
    import torch
    from paper_2411_19870_amd import binding as B
    from paper_2411_19870_amd import synth

    dev, S, K, W = "cuda:0", 64, a.k, a.workers
    specs = synth.tensor_set("1b")
    ts = []
    for ti, sp in enumerate(specs):
        g = synth.gaussian(sp, 1e-2, 0, ti, 0, "grad", dtype=torch.bfloat16, device=dev)
        m = synth.gaussian(sp, 1e-3, 0, ti, 0, "mom", device=dev)
        x = synth.gaussian(sp, 0.02, 0, ti, 0, "param", dtype=torch.bfloat16, device=dev)
        idx, val = synth.payload_fast(sp, S, K, W, 1e-3, 0, ti, device=dev)
        ts.append(B.TensorArgs(g, m, x, idx, val))
    tl = B.TensorList(ts)
    n2 = sum(sp.numel for sp in specs if sp.cols)
    pairs2 = sum(sp.nchunks(S) for sp in specs if sp.cols) * K
    enc_bytes = n2 * 10 + pairs2 * 8
    dec_bytes = n2 * 4 + W * pairs2 * 8
    ctx = B.Context()

    def time_encode(stage):
        ctx.demo_debug_set_encode_stage(stage)
        for _ in range(3):
            ctx.demo_encode(tl, 0.999, S, K)
        torch.cuda.synchronize()
        ctx.demo_set_timing(True)
        for _ in range(a.reps):
            ctx.demo_encode(tl, 0.999, S, K)
        ms = ctx.demo_last_kernel_ms(0)
        ctx.demo_set_timing(False)
        return ms

    rows = []
    names = {1: "memory stream only (loads with prefetch, momentum update, store, k pairs)",
             2: "+ the two DCT products (192 float32 MFMA)", 3: "+ top-k and payload", 0: "+ reconstruction = the kernel"}
    prev = 0.0
    for stage in (1, 2, 3, 0):
        ms = time_encode(stage)
        rows.append((names[stage], ms, ms - prev, enc_bytes / ms / 1e6))
        prev = ms
    ctx.demo_debug_set_encode_stage(0)

    def time_decode(stage):
        ctx.demo_debug_set_decode_stage(stage)
        for _ in range(3):
            ctx.demo_decode(tl, W, 1e-3, 0.0, S, K)
        torch.cuda.synchronize()
        ctx.demo_set_timing(True)
        for _ in range(a.reps):
            ctx.demo_decode(tl, W, 1e-3, 0.0, S, K)
        ms = ctx.demo_last_kernel_ms(2)
        ctx.demo_set_timing(False)
        return ms

    drows = []
    dnames = {1: "memory stream only (payload and parameter loads with prefetch, update, stores)",
              2: "+ scatter-add of the W k pairs into the LDS tile", 0: "+ the two IDCT products (192 float16 MFMA) = the kernel"}
    prev = 0.0
    for stage in (1, 2, 0):
        ms = time_decode(stage)
        drows.append((dnames[stage], ms, ms - prev, dec_bytes / ms / 1e6))
        prev = ms
    ctx.demo_debug_set_decode_stage(0)

    src = torch.empty(1 << 30, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    probes = []
    for mode, name, moved in ((0, "copy, default cache policy", 2), (1, "copy, non-temporal", 2), (2, "read only, non-temporal", 1),
                              (3, "write only, non-temporal", 1), (4, "write only, default cache policy", 1)):
        for _ in range(2):
            ctx.demo_stream_probe(dst, src, mode)
        torch.cuda.synchronize()
        ctx.demo_set_timing(True)
        for _ in range(5):
            ctx.demo_stream_probe(dst, src, mode)
        ms = ctx.demo_last_kernel_ms(1)
        ctx.demo_set_timing(False)
        probes.append((name, ms, moved * src.numel() * 4 / ms / 1e6))
    ctx.close()

    print(f"## encode2d_wave64, 1B-like set, bf16 gradients, s = 64, k = {K}: {enc_bytes} algorithmic bytes per launch\n")
    print("| kernel copy | ms | added ms | algorithmic GB/s | of 8 TB/s |\n|---|---|---|---|---|")
    for name, ms, d, gbs in rows:
        print(f"| {name} | {ms:.3f} | {d:+.3f} | {gbs:.0f} | {gbs / 8000:.3f} |")
    print(f"\n## decode2d_wave64, 1B-like set, bf16 parameters, s = 64, k = {K}, W = {W}: {dec_bytes} algorithmic bytes per launch\n")
    print("| kernel copy | ms | added ms | algorithmic GB/s | of 8 TB/s |\n|---|---|---|---|---|")
    for name, ms, d, gbs in drows:
        print(f"| {name} | {ms:.3f} | {d:+.3f} | {gbs:.0f} | {gbs / 8000:.3f} |")
    print("\n## stream probes over 4 GiB (one 512-thread workgroup per CU, 16 B per lane, 8 accesses in flight)\n")
    print("| probe | ms | GB/s moved | of 8 TB/s |\n|---|---|---|---|")
    for name, ms, gbs in probes:
        print(f"| {name} | {ms:.3f} | {gbs:.0f} | {gbs / 8000:.3f} |")


if __name__ == "__main__":
    main()
