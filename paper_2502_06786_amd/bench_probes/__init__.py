"""Binding of libmq_probe.so: measurement-only kernels for bench.py (what this GPU sustains on a loop of bf16
matrix-core products and on a kernel that only reads).  Not part of the product library."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmq_probe.so")
EXPORTS = ["mq_probe_mfma", "mq_probe_mfma16", "mq_probe_read"]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    for name in EXPORTS:
        getattr(lib, name).argtypes = [vp, i64, vp, vp]
        getattr(lib, name).restype = ctypes.c_int
    return lib


_lib = _load()


def lib() -> ctypes.CDLL:
    return _lib


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, dtype):
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise ValueError(f"expected a contiguous GPU tensor of {dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _check(status: int, what: str):
    if status != 0:
        raise RuntimeError(f"{what}: status {status}")


def mq_probe_mfma(operands, iters: int, sink=None):
    """Measurement helper: `iters` rounds of 12 bf16 32x32x16 products per wave on 1024 waves, fed with the
    32768 bf16 values of `operands`.  Returns the flop count of the launch."""
    assert operands.numel() >= 32768
    sink = torch.empty(65536, dtype=torch.float32, device=operands.device) if sink is None else sink
    st = _lib.mq_probe_mfma(_ptr(operands, torch.bfloat16), int(iters), _ptr(sink, torch.float32), _stream())
    _check(st, "mq_probe_mfma")
    return 256 * 4 * int(iters) * 12 * 32 * 32 * 16 * 2


def mq_probe_mfma16(operands, iters: int, sink=None):
    """Measurement helper: `iters` rounds of 24 bf16 16x16x32 products per wave on 2048 waves (two per SIMD),
    fed with the 32768 bf16 values of `operands`.  Returns the flop count of the launch."""
    assert operands.numel() >= 32768
    sink = torch.empty(131072, dtype=torch.float32, device=operands.device) if sink is None else sink
    assert sink.numel() >= 131072
    st = _lib.mq_probe_mfma16(_ptr(operands, torch.bfloat16), int(iters), _ptr(sink, torch.float32), _stream())
    _check(st, "mq_probe_mfma16")
    return 256 * 8 * int(iters) * 24 * 16 * 16 * 32 * 2


def mq_probe_read(src, sink=None):
    """Measurement helper: one kernel that reads every byte of `src` (uint8, a multiple of 16 bytes) once."""
    sink = torch.zeros(1, dtype=torch.int32, device=src.device) if sink is None else sink
    st = _lib.mq_probe_read(_ptr(src, torch.uint8), src.numel(), _ptr(sink, torch.int32), _stream())
    _check(st, "mq_probe_read")
    return src.numel()
