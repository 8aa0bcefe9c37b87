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
    # both products of a chunk with the mirror folds: 192 (s = 64), 32 (s = 32, per chunk), 1536 (s = 128)
    # v_mfma_f32_16x16x4_f32 of 2048 flop each
    for s, per_chunk in ((64, 192), (32, 32), (128, 1536)):
        assert bench.mfma_flops_per_launch("dec2d", s, 32, 64 if s != 32 else 16, 1000, []) == per_chunk * 2048.0 * 1000


def test_source_hash_is_stable_and_short():
    h = bench.source_hash()
    assert h == bench.source_hash() and len(h) == 16 and int(h, 16) >= 0


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, "bench.py", "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
