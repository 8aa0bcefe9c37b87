"""Host-side checks that need no GPU: the shared library loads, exports every
function include/*.h declares, and rejects bad arguments before any launch."""
import ctypes
import numpy as np
import os
import re

import pytest

from paper_2411_19870_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(demo_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    names = declared_functions()
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/ but not exported"
    assert sorted(B.EXPORTS) == names


def test_struct_layout():
    assert ctypes.sizeof(B.DemoTensor) == 64
    assert B.DemoTensor.rows.offset == 40 and B.DemoTensor.grad_dtype.offset == 56


def test_payload_elems_and_shape_errors():
    assert B.demo_payload_elems(1024, 1024, 64, 32) == 256 * 32
    assert B.demo_payload_elems(2048, 0, 64, 32) == 32 * 32
    # Sec. 2.1 "Top-k Sparsification": reduction (prod s_i)/k, 4096/32 = 128 at 64 x 64
    assert (1024 * 1024) // B.demo_payload_elems(1024, 1024, 64, 32) == 128
    assert B.demo_payload_elems(64, (1 << 22) - 64, 64, 1) == (1 << 16) - 1
    for args, code in [
        ((1000, 1024, 64, 32), B.DEMO_ERR_SHAPE),
        ((1024, 1000, 64, 32), B.DEMO_ERR_SHAPE),
        ((0, 64, 64, 32), B.DEMO_ERR_SHAPE),
        ((-64, 64, 64, 32), B.DEMO_ERR_SHAPE),
        ((1024, 1024, 48, 32), B.DEMO_ERR_UNSUPPORTED),
        ((1024, 1024, 64, 0), B.DEMO_ERR_ARG),
        ((1024, 0, 64, 65), B.DEMO_ERR_ARG),           # k > M = s
        ((1024, 1024, 32, 1025), B.DEMO_ERR_ARG),      # k > M = s*s
        ((1024, 1024, 64, 257), B.DEMO_ERR_UNSUPPORTED),
        ((1 << 40, 1 << 40, 64, 1), B.DEMO_ERR_UNSUPPORTED),    # more chunks than 32 bits number
        ((1 << 40, 0, 32, 1), B.DEMO_ERR_UNSUPPORTED),
        ((64, 1 << 22, 64, 1), B.DEMO_ERR_UNSUPPORTED),         # row offsets inside a chunk are 32-bit: cols < 2^22
    ]:
        with pytest.raises(B.DemoError) as e:
            B.demo_payload_elems(*args)
        assert e.value.status == code, args


def _tensor(**kw):
    t = B.DemoTensor()
    t.grad, t.mom, t.param, t.idx, t.val = 0x1000, 0x2000, 0x3000, 0x4000, 0x5000   # never dereferenced
    t.rows, t.cols, t.grad_dtype, t.param_dtype = 128, 128, B.DEMO_F32, B.DEMO_F32
    for k, v in kw.items():
        setattr(t, k, v)
    return t


def test_validation_happens_before_any_launch():
    lib = B.load_library()
    h = ctypes.c_void_p()
    assert lib.demo_create(ctypes.byref(h)) == B.DEMO_OK
    arr1 = (B.DemoTensor * 1)

    def enc(t, s=64, k=32, n=1):
        return lib.demo_encode(h, arr1(t), n, 0.999, s, k, None)

    def dec(t, s=64, k=32, W=1):
        return lib.demo_decode(h, arr1(t), 1, W, 1e-3, 0.0, s, k, None)

    def step(t, s=64, k=32):
        return lib.demo_step(h, arr1(t), 1, 0.999, 1e-3, 0.0, s, k, None)

    assert lib.demo_encode(None, arr1(_tensor()), 1, 0.999, 64, 32, None) == B.DEMO_ERR_ARG
    assert lib.demo_encode(h, None, 1, 0.999, 64, 32, None) == B.DEMO_ERR_ARG
    assert enc(_tensor(), n=-1) == B.DEMO_ERR_ARG
    assert enc(_tensor(), n=0) == B.DEMO_OK                       # empty list: nothing to do
    assert enc(_tensor(), s=48) == B.DEMO_ERR_UNSUPPORTED
    assert enc(_tensor(), k=0) == B.DEMO_ERR_ARG
    assert enc(_tensor(rows=100)) == B.DEMO_ERR_SHAPE
    assert enc(_tensor(cols=96)) == B.DEMO_ERR_SHAPE
    assert enc(_tensor(cols=0), k=65) == B.DEMO_ERR_ARG
    assert enc(_tensor(), k=300) == B.DEMO_ERR_UNSUPPORTED
    assert enc(_tensor(grad_dtype=7)) == B.DEMO_ERR_UNSUPPORTED
    assert enc(_tensor(grad=None)) == B.DEMO_ERR_ARG
    assert enc(_tensor(mom=None)) == B.DEMO_ERR_ARG
    assert enc(_tensor(idx=None)) == B.DEMO_ERR_ARG
    assert enc(_tensor(val=None)) == B.DEMO_ERR_ARG
    assert dec(_tensor(param=None)) == B.DEMO_ERR_ARG
    assert dec(_tensor(param_dtype=5)) == B.DEMO_ERR_UNSUPPORTED
    assert dec(_tensor(), W=0) == B.DEMO_ERR_ARG
    assert dec(_tensor(rows=64, cols=96)) == B.DEMO_ERR_SHAPE
    assert enc(_tensor(grad=0x1004)) == B.DEMO_ERR_ARG            # tensor pointers: 16-byte aligned
    assert enc(_tensor(mom=0x2008)) == B.DEMO_ERR_ARG
    assert dec(_tensor(param=0x3002)) == B.DEMO_ERR_ARG
    assert enc(_tensor(idx=0x4002)) == B.DEMO_ERR_ARG             # payload arrays: 4-byte aligned
    assert enc(_tensor(idx=0x4004, val=0x5004), n=0) == B.DEMO_OK
    assert step(_tensor(param=None)) == B.DEMO_ERR_ARG
    assert step(_tensor(grad=None)) == B.DEMO_ERR_ARG
    assert lib.demo_set_variant(h, 5) == B.DEMO_ERR_ARG
    assert lib.demo_set_variant(h, 2) == B.DEMO_OK and lib.demo_set_variant(h, 1) == B.DEMO_OK
    ms = ctypes.c_float()
    assert lib.demo_last_kernel_ms(h, 0, ctypes.byref(ms)) == B.DEMO_ERR_ARG   # nothing recorded
    assert lib.demo_destroy(h) == B.DEMO_OK
    assert lib.demo_destroy(None) == B.DEMO_ERR_ARG
    assert lib.demo_strerror(B.DEMO_ERR_SHAPE) and lib.demo_strerror(12345)


def test_hparams_struct_and_validation():
    lib = B.load_library()
    assert ctypes.sizeof(B.DemoHParams) == 32
    hp = B.demo_hparams_default(0.999, 1e-3, 0.1)
    assert (hp.beta, hp.grad_scale, hp.alpha) == (ctypes.c_float(0.999).value, 1.0, 1.0)
    assert (hp.phi, hp.aggregate, hp.reserved) == (B.DEMO_PHI_SIGN, B.DEMO_AGG_SUM, 0)
    assert lib.demo_hparams_default(None, 0.9, 0.0, 0.0) == B.DEMO_ERR_ARG
    h = ctypes.c_void_p()
    assert lib.demo_create(ctypes.byref(h)) == B.DEMO_OK
    arr1 = (B.DemoTensor * 1)
    t = _tensor()
    assert lib.demo_decode_ex(h, arr1(t), 1, 1, None, 64, 32, None) == B.DEMO_ERR_ARG
    for bad in (dict(phi=2), dict(aggregate=3), dict(reserved=5), dict(weight_decay=float("inf"))):
        hpb = B.demo_hparams_default(**{**dict(beta=0.9, lr=1e-3, weight_decay=0.0), **bad})
        assert lib.demo_decode_ex(h, arr1(t), 1, 1, ctypes.byref(hpb), 64, 32, None) == B.DEMO_ERR_ARG
    cnt = B.demo_hparams_default(0.9, 1e-3, 0.0, aggregate=B.DEMO_AGG_COUNT)
    assert lib.demo_decode_ex(h, arr1(t), 1, 256, ctypes.byref(cnt), 64, 32, None) == B.DEMO_ERR_ARG
    # phi = identity beyond the worker limit of the fixed-point aggregate is refused, not computed coarsely
    ident = B.demo_hparams_default(0.9, 1e-3, 0.0, phi=B.DEMO_PHI_IDENTITY)
    assert lib.demo_decode_ex(h, arr1(t), 1, B.DEMO_MAX_W_IDENTITY + 1, ctypes.byref(ident), 64, 32, None) == B.DEMO_ERR_UNSUPPORTED
    assert lib.demo_decode_ex(h, arr1(t), 1, 3000, ctypes.byref(ident), 64, 32, None) == B.DEMO_ERR_UNSUPPORTED
    nanb = B.demo_hparams_default(float("nan"), 1e-3, 0.0)
    assert lib.demo_encode_ex(h, arr1(t), 1, ctypes.byref(nanb), 64, 32, None) == B.DEMO_ERR_ARG
    assert lib.demo_step_ex(h, arr1(t), 1, ctypes.byref(nanb), 64, 32, None) == B.DEMO_ERR_ARG
    # shape errors are still reported first, and an empty list is fine
    assert lib.demo_encode_ex(h, arr1(_tensor(rows=100)), 1, ctypes.byref(hp), 64, 32, None) == B.DEMO_ERR_SHAPE
    assert lib.demo_encode_ex(h, arr1(t), 0, ctypes.byref(hp), 64, 32, None) == B.DEMO_OK
    assert lib.demo_destroy(h) == B.DEMO_OK


def test_set_basis_validation_on_host():
    lib = B.load_library()
    h = ctypes.c_void_p()
    assert lib.demo_create(ctypes.byref(h)) == B.DEMO_OK
    assert lib.demo_set_basis(None, 64, B.DEMO_BASIS_DCT, None) == B.DEMO_ERR_ARG
    assert lib.demo_set_basis(h, 48, B.DEMO_BASIS_IDENTITY, None) == B.DEMO_ERR_UNSUPPORTED
    assert lib.demo_set_basis(h, 64, 9, None) == B.DEMO_ERR_ARG
    assert lib.demo_set_basis(h, 64, B.DEMO_BASIS_GRAM_SCHMIDT, None) == B.DEMO_ERR_ARG
    # linearly dependent rows are refused before anything touches a device
    a = (ctypes.c_float * (32 * 32))(*([1.0] * (32 * 32)))
    assert lib.demo_set_basis(h, 32, B.DEMO_BASIS_GRAM_SCHMIDT, ctypes.cast(a, ctypes.c_void_p)) == B.DEMO_ERR_ARG
    assert lib.demo_destroy(h) == B.DEMO_OK


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libdemo.so"))
    with pytest.raises(FileNotFoundError):
        B.load_library()


def test_worker_and_position_of_a_pair_from_a_float_product():
    """The decode kernels split pair number p of a chunk into worker p // k and position p % k with one float32
    multiply, w = int((p + 0.5) * (1 / k)), for p < 65536 (the streamed payload limit) and every budget k the
    ABI accepts: emulated here in float32, it must agree with the integer division for all of them."""
    p = np.arange(0, 65536, dtype=np.int64)
    for k in range(1, 257):
        rk = np.float32(1.0) / np.float32(k)
        w = ((p.astype(np.float32) + np.float32(0.5)) * rk).astype(np.int32)
        assert np.array_equal(w, p // k), k


def test_host_code_under_sanitizers(tmp_path):
    """The library's host code (validation of every entry point, Gram-Schmidt, fragment-table
    builders) built with AddressSanitizer + UndefinedBehaviorSanitizer on the host side only and
    driven by tests/host_check/host_check.cpp; no GPU call is reached."""
    import subprocess
    from paper_2411_19870_amd import build

    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    build.build(verbose=False, out=str(tmp_path / "libdemo_san.so"), extra_flags=san)
    exe = str(tmp_path / "host_check")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O1", "-g", "-std=c++17"] + san + [
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2411_19870_amd", "csrc"),
        os.path.join(ROOT, "tests", "host_check", "host_check.cpp"), "-L", str(tmp_path), "-ldemo_san",
        f"-Wl,-rpath,{tmp_path}", "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and "host_check OK" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]
