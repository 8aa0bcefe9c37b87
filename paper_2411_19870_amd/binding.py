"""ctypes binding of libdemo.so: argument marshalling only.

Every function mirrors an entry point of include/demo.h.  Tensors are torch
tensors living on the GPU; torch is used for device memory and streams only, all
arithmetic runs in the HIP kernels.  There is no CPU fallback: if the library is
missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DEMO_LIBRARY_PATH") or os.path.join(_HERE, "libdemo.so")

DEMO_OK, DEMO_ERR_ARG, DEMO_ERR_SHAPE, DEMO_ERR_UNSUPPORTED, DEMO_ERR_HIP, DEMO_ERR_NOMEM, DEMO_ERR_LIMIT = 0, -1, -2, -3, -4, -5, -6
DEMO_F32, DEMO_BF16 = 0, 1
DEMO_MAX_K = 256
DEMO_MAX_W_IDENTITY = 1024
DEMO_MAX_COLS = 1 << 22
DEMO_PHI_SIGN, DEMO_PHI_IDENTITY = 0, 1
DEMO_AGG_SUM, DEMO_AGG_MEAN, DEMO_AGG_COUNT = 0, 1, 2
DEMO_BASIS_DCT, DEMO_BASIS_IDENTITY, DEMO_BASIS_GRAM_SCHMIDT = 0, 1, 2

EXPORTS = [
    "demo_create", "demo_destroy", "demo_payload_elems", "demo_encode", "demo_decode", "demo_step",
    "demo_hparams_default", "demo_encode_ex", "demo_decode_ex", "demo_step_ex", "demo_set_basis",
    "demo_encode_noalloc", "demo_strerror", "demo_last_hip_error",
    # include/demo_debug.h: measurement and test hooks
    "demo_set_timing", "demo_last_kernel_ms", "demo_set_variant", "demo_copy_probe", "demo_stream_probe",
    "demo_debug_set_encode_stage", "demo_debug_set_decode_stage",
]


class DemoTensor(ctypes.Structure):
    _fields_ = [
        ("grad", ctypes.c_void_p), ("mom", ctypes.c_void_p), ("param", ctypes.c_void_p),
        ("idx", ctypes.c_void_p), ("val", ctypes.c_void_p),
        ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
        ("grad_dtype", ctypes.c_int32), ("param_dtype", ctypes.c_int32),
    ]


class DemoHParams(ctypes.Structure):
    _fields_ = [
        ("beta", ctypes.c_float), ("grad_scale", ctypes.c_float), ("alpha", ctypes.c_float),
        ("lr", ctypes.c_float), ("weight_decay", ctypes.c_float),
        ("phi", ctypes.c_int32), ("aggregate", ctypes.c_int32), ("reserved", ctypes.c_int32),
    ]


class DemoError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libdemo status {status}: {text}")
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libdemo.so (built by paper_2411_19870_amd/build.py).  Fails loudly."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2411_19870_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, cf, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_int64
    lib.demo_create.argtypes = [ctypes.POINTER(vp)]
    lib.demo_destroy.argtypes = [vp]
    lib.demo_payload_elems.argtypes = [i64, i64, ci, ci, ctypes.POINTER(i64)]
    lib.demo_encode.argtypes = [vp, ctypes.POINTER(DemoTensor), ci, cf, ci, ci, vp]
    lib.demo_encode_noalloc.argtypes = [vp, ctypes.POINTER(DemoTensor), ci, cf, ci, ci, vp]
    lib.demo_decode.argtypes = [vp, ctypes.POINTER(DemoTensor), ci, ci, cf, cf, ci, ci, vp]
    lib.demo_step.argtypes = [vp, ctypes.POINTER(DemoTensor), ci, cf, cf, cf, ci, ci, vp]
    hpp = ctypes.POINTER(DemoHParams)
    lib.demo_hparams_default.argtypes = [hpp, cf, cf, cf]
    lib.demo_encode_ex.argtypes = [vp, ctypes.POINTER(DemoTensor), ci, hpp, ci, ci, vp]
    lib.demo_decode_ex.argtypes = [vp, ctypes.POINTER(DemoTensor), ci, ci, hpp, ci, ci, vp]
    lib.demo_step_ex.argtypes = [vp, ctypes.POINTER(DemoTensor), ci, hpp, ci, ci, vp]
    lib.demo_set_basis.argtypes = [vp, ci, ci, vp]
    lib.demo_set_timing.argtypes = [vp, ci]
    lib.demo_last_kernel_ms.argtypes = [vp, ci, ctypes.POINTER(cf)]
    lib.demo_set_variant.argtypes = [vp, ci]
    lib.demo_copy_probe.argtypes = [vp, vp, vp, i64, vp]
    lib.demo_stream_probe.argtypes = [vp, vp, vp, i64, ci, vp]
    lib.demo_debug_set_encode_stage.argtypes = [vp, ci]
    lib.demo_debug_set_decode_stage.argtypes = [vp, ci]
    lib.demo_strerror.argtypes = [ci]
    lib.demo_strerror.restype = ctypes.c_char_p
    lib.demo_last_hip_error.argtypes = [vp]
    lib.demo_last_hip_error.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("demo_strerror", "demo_last_hip_error"):
            getattr(lib, name).restype = ci
    _lib = lib
    return lib


def demo_strerror(status: int) -> str:
    return load_library().demo_strerror(status).decode()


def demo_hparams_default(beta: float = 0.0, lr: float = 0.0, weight_decay: float = 0.0, **fields) -> DemoHParams:
    """demo_hparams with the algorithm boxes' values; keyword arguments overwrite single fields."""
    hp = DemoHParams()
    rc = load_library().demo_hparams_default(ctypes.byref(hp), beta, lr, weight_decay)
    if rc != DEMO_OK:
        raise DemoError(rc, demo_strerror(rc))
    for name, value in fields.items():
        if name not in dict(DemoHParams._fields_):
            raise TypeError(f"demo_hparams has no field {name!r}")
        setattr(hp, name, value)
    return hp


def demo_payload_elems(rows: int, cols: int, s: int, k: int) -> int:
    out = ctypes.c_int64(0)
    rc = load_library().demo_payload_elems(rows, cols, s, k, ctypes.byref(out))
    if rc != DEMO_OK:
        raise DemoError(rc, demo_strerror(rc))
    return out.value


@dataclass
class TensorArgs:
    """Device buffers of one tensor (any of grad / mom / param may be None)."""
    grad: Optional[torch.Tensor]
    mom: Optional[torch.Tensor]
    param: Optional[torch.Tensor]
    idx: torch.Tensor          # int32 [W, nchunks, k] (or [nchunks, k])
    val: torch.Tensor          # float32, same shape
    rows: int = 0
    cols: int = 0

    def __post_init__(self):
        ref = next(t for t in (self.mom, self.param, self.grad) if t is not None)
        if self.rows == 0:
            self.rows = ref.shape[0]
            self.cols = ref.shape[1] if ref.dim() == 2 else 0


def _dtype_code(t: Optional[torch.Tensor]) -> int:
    if t is None or t.dtype == torch.float32:
        return DEMO_F32
    if t.dtype == torch.bfloat16:
        return DEMO_BF16
    return 99   # rejected by the library as unsupported


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors handed to libdemo must be contiguous")
    return t.data_ptr()


def marshal(tensors: Sequence[TensorArgs]):
    arr = (DemoTensor * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        arr[i].grad, arr[i].mom, arr[i].param = _ptr(t.grad), _ptr(t.mom), _ptr(t.param)
        arr[i].idx, arr[i].val = _ptr(t.idx), _ptr(t.val)
        arr[i].rows, arr[i].cols = t.rows, t.cols
        arr[i].grad_dtype, arr[i].param_dtype = _dtype_code(t.grad), _dtype_code(t.param)
    return arr


class TensorList:
    """A tensor list marshalled once (the ctypes array plus the tensors it points
    into, kept alive).  Pass it instead of a sequence to skip per-call marshalling."""

    def __init__(self, tensors: Sequence[TensorArgs]):
        self.items = list(tensors)
        self.arr = marshal(self.items)
        self.n = len(self.items)


def _as_list(tensors) -> TensorList:
    return tensors if isinstance(tensors, TensorList) else TensorList(tensors)


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


class Context:
    """Owns a demo_ctx.  Methods carry the names of the C entry points."""

    def __init__(self):
        self._lib = load_library()
        h = ctypes.c_void_p()
        self._check(self._lib.demo_create(ctypes.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self._lib.demo_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != DEMO_OK:
            text = demo_strerror(rc)
            if rc == DEMO_ERR_HIP and getattr(self, "_h", None):
                text += ": " + self._lib.demo_last_hip_error(self._h).decode()
            raise DemoError(rc, text)

    def demo_encode(self, tensors: Sequence[TensorArgs], beta: float, s: int, k: int, stream=None):
        tl = _as_list(tensors)
        self._check(self._lib.demo_encode(self._h, tl.arr, tl.n, beta, s, k, _stream_ptr(stream)))

    def demo_encode_noalloc(self, tensors: Sequence[TensorArgs], beta: float, s: int, k: int, stream=None):
        tl = _as_list(tensors)
        self._check(self._lib.demo_encode_noalloc(self._h, tl.arr, tl.n, beta, s, k, _stream_ptr(stream)))

    def demo_decode(self, tensors: Sequence[TensorArgs], W: int, lr: float, weight_decay: float, s: int, k: int,
                    stream=None):
        tl = _as_list(tensors)
        self._check(self._lib.demo_decode(self._h, tl.arr, tl.n, W, lr, weight_decay, s, k, _stream_ptr(stream)))

    def demo_step(self, tensors: Sequence[TensorArgs], beta: float, lr: float, weight_decay: float, s: int, k: int,
                  stream=None):
        tl = _as_list(tensors)
        self._check(self._lib.demo_step(self._h, tl.arr, tl.n, beta, lr, weight_decay, s, k, _stream_ptr(stream)))

    def demo_encode_ex(self, tensors: Sequence[TensorArgs], hp: DemoHParams, s: int, k: int, stream=None):
        tl = _as_list(tensors)
        self._check(self._lib.demo_encode_ex(self._h, tl.arr, tl.n, ctypes.byref(hp), s, k, _stream_ptr(stream)))

    def demo_decode_ex(self, tensors: Sequence[TensorArgs], W: int, hp: DemoHParams, s: int, k: int, stream=None):
        tl = _as_list(tensors)
        self._check(self._lib.demo_decode_ex(self._h, tl.arr, tl.n, W, ctypes.byref(hp), s, k, _stream_ptr(stream)))

    def demo_step_ex(self, tensors: Sequence[TensorArgs], hp: DemoHParams, s: int, k: int, stream=None):
        tl = _as_list(tensors)
        self._check(self._lib.demo_step_ex(self._h, tl.arr, tl.n, ctypes.byref(hp), s, k, _stream_ptr(stream)))

    def demo_set_basis(self, s: int, kind: int, a: Optional[torch.Tensor] = None):
        """a: CPU float32 tensor of s*s values (DEMO_BASIS_GRAM_SCHMIDT), else None."""
        ptr = None
        if a is not None:
            if a.device.type != "cpu" or a.dtype != torch.float32 or not a.is_contiguous() or a.numel() != s * s:
                raise ValueError("demo_set_basis wants a contiguous CPU float32 tensor of s*s values")
            ptr = a.data_ptr()
        self._check(self._lib.demo_set_basis(self._h, s, kind, ptr))

    def demo_set_timing(self, enabled: bool):
        self._check(self._lib.demo_set_timing(self._h, int(enabled)))

    def demo_set_variant(self, variant: int):
        self._check(self._lib.demo_set_variant(self._h, variant))

    def demo_copy_probe(self, dst: torch.Tensor, src: torch.Tensor, stream=None):
        nbytes = src.numel() * src.element_size()
        assert dst.numel() * dst.element_size() >= nbytes
        self._check(self._lib.demo_copy_probe(self._h, dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr(stream)))

    def demo_stream_probe(self, dst: torch.Tensor, src: torch.Tensor, mode: int, stream=None):
        nbytes = src.numel() * src.element_size()
        assert dst.numel() * dst.element_size() >= (nbytes if mode != 2 else 65536)
        self._check(self._lib.demo_stream_probe(self._h, dst.data_ptr(), src.data_ptr(), nbytes, mode,
                                                _stream_ptr(stream)))

    def demo_debug_set_encode_stage(self, stage: int):
        self._check(self._lib.demo_debug_set_encode_stage(self._h, stage))

    def demo_debug_set_decode_stage(self, stage: int):
        self._check(self._lib.demo_debug_set_decode_stage(self._h, stage))

    def demo_last_kernel_ms(self, which: int) -> float:
        ms = ctypes.c_float(0)
        self._check(self._lib.demo_last_kernel_ms(self._h, which, ctypes.byref(ms)))
        return ms.value
