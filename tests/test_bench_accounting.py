"""The benchmark's own arithmetic (no GPU): algorithmic bytes per parameter, MFMA counts, the refusal of more than
one GPU.  The roofline fractions are these figures over measured times, so they are pinned here by hand values."""
import subprocess
import sys

import bench
from paper_2411_19870_amd import synth


def test_algorithmic_bytes_per_parameter():
    # encode: gradient read + momentum read + momentum write + 8 k / s^2 payload bytes per parameter;
    # decode: parameter read + write + 8 W k / s^2.  s = 64, k = 32: 2 + 4 + 4 + 1/16 = 10.0625 and, at W = 64 with
    # bfloat16 parameters, 2 + 2 + 4 = 8 bytes per parameter of an order-2 tensor.
    specs = synth.tensor_set("1b")
    ab = bench.algorithmic_bytes(specs, 64, 32, 64, 2, 2)
    n2 = sum(sp.numel for sp in specs if sp.cols)
    n1 = sum(sp.numel for sp in specs if not sp.cols)
    assert ab["params2d"] == n2 == 908328960 and ab["params1d"] == n1 == 65536
    assert ab["enc2d"] == n2 * 10 + n2 // 16 == 9140060160
    assert ab["dec2d"] == n2 * 8 == 7266631680
    # order-1 chunks hold 64 parameters: 8 k / s = 4 bytes of payload per parameter and worker
    assert ab["enc1d"] == n1 * (2 + 4 + 4 + 4)
    assert ab["dec1d"] == n1 * (2 + 2 + 4 * 64)
    # float32 gradients and parameters (the 300M-like set): 12.0625 and 4 + 4 + 4
    specs = synth.tensor_set("300m")
    ab = bench.algorithmic_bytes(specs, 64, 32, 64, 4, 4)
    n2 = sum(sp.numel for sp in specs if sp.cols)
    assert ab["enc2d"] == n2 * 12 + n2 // 16
    assert ab["dec2d"] == n2 * 12


def test_mfma_count_of_the_decode_products():
    # s = 32: both products of a chunk with the mirror fold, 32 v_mfma_f32_16x16x4_f32 of 2048 flop each
    assert bench.mfma_work_per_launch("dec2d", 32, 32, 16, 1000, []) == {"f32": 32 * 2048.0 * 1000}
    # s = 64, 64 < W k <= 2048: two full 64^3 products, 16 tiles x 2 blocks of 32 contraction indices x 3 partial
    # products = 96 v_mfma_f32_16x16x32_f16 of 16384 flop each; the mirror-folded float32 instances (variant 2, and
    # the streamed payloads beyond 2048 pairs): 192 v_mfma_f32_16x16x4_f32
    assert bench.mfma_work_per_launch("dec2d", 64, 32, 64, 1000, []) == {"f16": 192 * 16384.0 * 1000}
    assert bench.mfma_work_per_launch("dec2d", 64, 32, 64, 1000, [], variant=2) == {"f32": 192 * 2048.0 * 1000}
    assert bench.mfma_work_per_launch("dec2d", 64, 32, 128, 1000, []) == {"f32": 192 * 2048.0 * 1000}
    # s = 128: four 64^3 quadrant products, twice: 4 x 2 x 96 float16 instructions
    assert bench.mfma_work_per_launch("dec2d", 128, 32, 64, 1000, []) == {"f16": 768 * 16384.0 * 1000}
    # few pairs per chunk: data dependent, not counted; generic kernels: not counted
    assert bench.mfma_work_per_launch("dec2d", 128, 32, 1, 1000, []) is None
    assert bench.mfma_work_per_launch("dec2d", 64, 32, 64, 1000, [], variant=0) is None


def test_mfma_count_of_the_s128_encode():
    import torch
    # two chunks of k = 4: all four coefficients in class (0, 0) -> one step; one per class -> one step; the products
    # are 768 float16 instructions, a reconstruction step 8 wavefronts x 2 tiles x 4 classes = 64 float32 ones
    idx = torch.tensor([[[0, 2, 256, 258], [0, 1, 128, 129]]], dtype=torch.int32)
    w = bench.mfma_work_per_launch("enc2d", 128, 4, 1, 2, [idx])
    assert w == {"f16": 768 * 16384.0 * 2, "f32": 2 * 64 * 2048.0}
    # five in one class -> two steps
    idx = torch.tensor([[[0, 2, 4, 6, 8]]], dtype=torch.int32)
    assert bench.mfma_work_per_launch("enc2d", 128, 5, 1, 1, [idx])["f32"] == 2 * 64 * 2048.0


def test_source_hash_is_stable_and_short():
    h = bench.source_hash()
    assert h == bench.source_hash() and len(h) == 16 and int(h, 16) >= 0


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, "bench.py", "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
