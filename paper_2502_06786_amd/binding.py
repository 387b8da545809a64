"""Thin Python binding of the C ABI in include/mq.h.

Argument marshalling only: every function checks dtypes/devices, passes
``tensor.data_ptr()`` and the current HIP stream to libmq.so and raises on a
non-zero status.  PyTorch is used for device memory and streams, nothing else;
there is no CPU fallback: if libmq.so is missing the import fails.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmq.so")

MQ_FLAG_EXTRA_PRECISION = 1
MQ_FLAG_PACKED = 2
MQ_FLAG_ACCUM_DW = 4
MQ_OP_LINEAR_FWD = 0
MQ_OP_LINEAR_BWD = 1
MQ_OP_FFN_DECODE = 2
MQ_OP_L2_LOSS = 3
MQ_OP_LINEAR_FWD_L2 = 4
MQ_OP_LINEAR_BWD_CLIP = 5
MQ_OP_AFFINE_BWD = 6
MQ_OP_GEMV = 7
MQ_FLAG_LOSS_MIX = 64
MQ_FLAG_FFN_SILU = 16
MQ_FLAG_FFN_RESIDUAL = 32

EXPORTS = ["mq_quantize_int8", "mq_slice", "mq_linear_fwd_multi", "mq_linear_bwd", "mq_gemv_sliced",
           "mq_params_to_bf16", "mq_workspace_bytes", "mq_status_string",
           "mq_gemv_sliced_dense_ep", "mq_ffn_mixnmatch", "mq_matquant_l2_loss", "mq_linear_fwd_multi_l2", "mq_linear_bwd_clip",
           "mq_affine_weight", "mq_affine_input", "mq_affine_bwd", "mq_gated_unit_fwd", "mq_gated_unit_bwd",
           "mq_linear_fwd_multi_noalloc", "mq_linear_bwd_gated", "mq_linear_fwd_multi_gated", "mq_slice_multi", "mq_gemv_sliced_ws"]


class MqError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: mq_status {status} ({status_string(status)})")
        self.status = status


class _FfnLayer(ctypes.Structure):
    _fields_ = [("gate_up", ctypes.c_void_p), ("down", ctypes.c_void_p), ("alpha_gu", ctypes.c_void_p),
                ("zero_gu", ctypes.c_void_p), ("alpha_dn", ctypes.c_void_p), ("zero_dn", ctypes.c_void_p),
                ("r", ctypes.c_int)]


class _Overflow(ctypes.Structure):
    _fields_ = [("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p),
                ("capacity", ctypes.c_int64), ("nnz", ctypes.c_void_p)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(the HIP library is the only implementation; there is no fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, ci, u32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32, ctypes.c_size_t
    lib.mq_quantize_int8.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp, vp, vp]
    lib.mq_slice.argtypes = [vp, i64, i64, ci, u32, vp, ctypes.POINTER(_Overflow), vp]
    lib.mq_linear_fwd_multi.argtypes = [vp, vp, vp, vp, i64, i64, i64, ctypes.POINTER(ci), ci, u32,
                                        ctypes.POINTER(vp), vp, sz, vp]
    lib.mq_linear_fwd_multi_noalloc.argtypes = [vp, vp, vp, vp, i64, i64, i64, ctypes.POINTER(ci), ci, u32,
                                                ctypes.POINTER(vp), vp]
    lib.mq_linear_bwd.argtypes = [vp, vp, vp, vp, ctypes.POINTER(vp), ctypes.POINTER(ctypes.c_float), i64, i64,
                                  i64, ctypes.POINTER(ci), ci, u32, vp, vp, vp, sz, vp]
    lib.mq_slice_multi.argtypes = [vp, i64, i64, ctypes.POINTER(ci), ci, u32, ctypes.POINTER(vp), ci, ctypes.POINTER(_Overflow), vp]
    lib.mq_linear_fwd_multi_gated.argtypes = [vp, vp, vp, vp, i64, i64, i64, ctypes.POINTER(ci), ci, u32, ctypes.POINTER(vp),
                                              ctypes.POINTER(vp), vp, sz, vp]
    lib.mq_linear_bwd_gated.argtypes = [vp, vp, vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(ctypes.c_float),
                                        i64, i64, i64, ctypes.POINTER(ci), ci, u32, vp, vp, vp, sz, vp]
    lib.mq_gemv_sliced.argtypes = [vp, vp, vp, vp, ctypes.POINTER(_Overflow), i64, i64, i64, ci, vp, vp]
    lib.mq_gemv_sliced_ws.argtypes = [vp, vp, vp, vp, ctypes.POINTER(_Overflow), i64, i64, i64, ci, vp, vp, sz, vp]
    lib.mq_workspace_bytes.argtypes = [ci, i64, i64, i64, ci]
    lib.mq_workspace_bytes.restype = sz
    lib.mq_status_string.argtypes = [ci]
    lib.mq_status_string.restype = ctypes.c_char_p
    lib.mq_params_to_bf16.argtypes = [vp, vp, i64, vp, vp, vp]
    lib.mq_gemv_sliced_dense_ep.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, vp, vp]
    lib.mq_matquant_l2_loss.argtypes = [ctypes.POINTER(vp), vp, ctypes.POINTER(ci), ctypes.POINTER(ctypes.c_float), i64,
                                        i64, ci, u32, ctypes.POINTER(vp), vp, vp, sz, vp]
    lib.mq_gated_unit_fwd.argtypes = [ctypes.POINTER(vp), ci, i64, i64, u32, ctypes.POINTER(vp), vp]
    lib.mq_gated_unit_bwd.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(vp), ci, i64, i64, u32, ctypes.POINTER(vp), vp]
    lib.mq_affine_weight.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp, vp, vp]
    lib.mq_affine_input.argtypes = [vp, i64, i64, vp, vp, vp, vp]
    lib.mq_affine_bwd.argtypes = [vp, vp, vp, i64, vp, ctypes.POINTER(vp), ctypes.POINTER(ctypes.c_float), ci, i64, i64, i64,
                                  vp, vp, vp, vp, vp, vp, sz, vp]
    lib.mq_linear_fwd_multi_l2.argtypes = [vp, vp, vp, vp, i64, i64, i64, ctypes.POINTER(ci), ci, u32, vp, vp,
                                           ctypes.POINTER(ci), ctypes.POINTER(ctypes.c_float), ctypes.POINTER(vp),
                                           ctypes.POINTER(vp), vp, vp, sz, vp]
    lib.mq_linear_bwd_clip.argtypes = [vp, i64, vp, vp, vp, vp, vp, vp, ctypes.POINTER(vp), ctypes.POINTER(ctypes.c_float),
                                       i64, i64, i64, ctypes.POINTER(ci), ci, u32, vp, vp, vp, vp, vp, sz, vp]
    lib.mq_ffn_mixnmatch.argtypes = [vp, ctypes.POINTER(_FfnLayer), ci, i64, i64, i64, u32, vp, vp, sz, vp]
    for name in EXPORTS:
        if name not in ("mq_workspace_bytes", "mq_status_string"):
            getattr(lib, name).restype = ci
    return lib


_lib = _load()


def lib() -> ctypes.CDLL:
    return _lib


MQ_FLAG_EP_DENSE = 8


def status_string(status: int) -> str:
    return _lib.mq_status_string(int(status)).decode()


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _check(status: int, what: str):
    if status != 0:
        raise MqError(status, what)


class Overflow:
    """Device buffers of the extra-precision overflow set (CSR rows, uint16 columns)."""

    def __init__(self, N: int, capacity: int, device="cuda"):
        self.row_ptr = torch.empty(N + 1, dtype=torch.int32, device=device)
        self.col_idx = torch.empty(max(capacity, 1), dtype=torch.int16, device=device)  # uint16 bit patterns
        self.nnz = torch.zeros(1, dtype=torch.int64, device=device)
        self.capacity = capacity

    def c_struct(self) -> _Overflow:
        return _Overflow(self.row_ptr.data_ptr(), self.col_idx.data_ptr(), self.capacity, self.nnz.data_ptr())


def mq_workspace_bytes(op: int, M: int, N: int, K: int, nr: int) -> int:
    return int(_lib.mq_workspace_bytes(op, M, N, K, nr))


def mq_quantize_int8(W, gamma=None, beta=None, Q=None, alpha=None, zero=None):
    """W fp32 [N, K] (row stride allowed) -> (Q uint8 [N, K], alpha fp32 [N], zero fp32 [N])."""
    if W.dtype != torch.float32 or not W.is_cuda or W.dim() != 2 or W.stride(1) != 1:
        raise ValueError("W must be a 2-D fp32 GPU tensor with unit column stride")
    N, K = W.shape
    ldw = W.stride(0) if N > 1 else max(K, W.stride(0))
    Q = torch.empty(N, K, dtype=torch.uint8, device=W.device) if Q is None else Q
    alpha = torch.empty(N, dtype=torch.float32, device=W.device) if alpha is None else alpha
    zero = torch.empty(N, dtype=torch.float32, device=W.device) if zero is None else zero
    st = _lib.mq_quantize_int8(ctypes.c_void_p(W.data_ptr()), N, K, ldw, _ptr(gamma, torch.float32),
                               _ptr(beta, torch.float32), _ptr(Q, torch.uint8), _ptr(alpha, torch.float32),
                               _ptr(zero, torch.float32), _stream())
    _check(st, "mq_quantize_int8")
    return Q, alpha, zero


def mq_params_to_bf16(alpha, zero, alpha_bf16=None, zero_bf16=None):
    """fp32 [N] scale and zero-point -> bf16 copies for the decode GEMV."""
    N = alpha.numel()
    alpha_bf16 = torch.empty(N, dtype=torch.bfloat16, device=alpha.device) if alpha_bf16 is None else alpha_bf16
    zero_bf16 = torch.empty(N, dtype=torch.bfloat16, device=alpha.device) if zero_bf16 is None else zero_bf16
    st = _lib.mq_params_to_bf16(_ptr(alpha, torch.float32), _ptr(zero, torch.float32), N,
                                _ptr(alpha_bf16, torch.bfloat16), _ptr(zero_bf16, torch.bfloat16), _stream())
    _check(st, "mq_params_to_bf16")
    return alpha_bf16, zero_bf16


def mq_gemv_sliced_dense_ep(x, packed, alpha_bf16, zero_bf16, r: int, K: int, y=None):
    """x bf16 [B, K], packed uint8 [N, K*(r+1)/8] holding the unclamped extra-precision codes -> y bf16 [B, N]."""
    B = x.shape[0]
    N = packed.shape[0]
    if x.shape[1] != K or packed.shape[1] != K * (r + 1) // 8:
        raise ValueError("shape mismatch")
    if y is None:
        y = torch.empty(B, N, dtype=torch.bfloat16, device=x.device)
    st = _lib.mq_gemv_sliced_dense_ep(_ptr(x, torch.bfloat16), _ptr(packed, torch.uint8), _ptr(alpha_bf16, torch.bfloat16),
                                      _ptr(zero_bf16, torch.bfloat16), B, N, K, r, _ptr(y, torch.bfloat16), _stream())
    _check(st, "mq_gemv_sliced_dense_ep")
    return y


def mq_slice(Q, r: int, packed: bool = False, extra_precision: bool = False, out=None, ovf: Overflow | None = None,
             capacity: int | None = None, dense_ep: bool = False):
    """Slice int8 codes to r bits.  Returns `out`, or (out, Overflow) with extra_precision; with dense_ep (and
    packed, extra_precision) a single plane of r + 1 bits per code."""
    N, K = Q.shape
    flags = (MQ_FLAG_PACKED if packed else 0) | (MQ_FLAG_EXTRA_PRECISION if extra_precision else 0)
    flags |= MQ_FLAG_EP_DENSE if dense_ep else 0
    if out is None:
        cols = K * (r + 1 if dense_ep else r) // 8 if packed else K
        out = torch.empty(N, cols, dtype=torch.uint8, device=Q.device)
    if dense_ep:
        st = _lib.mq_slice(_ptr(Q, torch.uint8), N, K, r, flags, _ptr(out, torch.uint8), None, _stream())
        _check(st, "mq_slice")
        return out
    c_ovf = None
    if extra_precision:
        if ovf is None:
            ovf = Overflow(N, N * K if capacity is None else capacity, Q.device)
        c_ovf = ctypes.byref(ovf.c_struct())
    st = _lib.mq_slice(_ptr(Q, torch.uint8), N, K, r, flags, _ptr(out, torch.uint8), c_ovf, _stream())
    _check(st, "mq_slice")
    return (out, ovf) if extra_precision else out


def mq_slice_multi(Q, rs, out=None, ovf_r: int | None = None, ovf: Overflow | None = None, capacity: int | None = None):
    """Packed planes of the codes for every r in rs in one call; with ovf_r also the overflow list of that bit-width.
    Returns the list of planes, or (planes, Overflow)."""
    N, K = Q.shape
    rs = list(rs)
    if out is None:
        out = [torch.empty(N, K * r // 8, dtype=torch.uint8, device=Q.device) for r in rs]
    c_ovf, idx, flags = None, -1, 0
    if ovf_r is not None:
        idx, flags = rs.index(ovf_r), MQ_FLAG_EXTRA_PRECISION
        if ovf is None:
            ovf = Overflow(N, N * K if capacity is None else capacity, Q.device)
        c_ovf = ctypes.byref(ovf.c_struct())
    st = _lib.mq_slice_multi(_ptr(Q, torch.uint8), N, K, _int_array(rs), len(rs), flags, _ptr_array(out, torch.uint8), idx,
                             c_ovf, _stream())
    _check(st, "mq_slice_multi")
    return (out, ovf) if ovf_r is not None else out


def _int_array(vals):
    return (ctypes.c_int * len(vals))(*[int(v) for v in vals])


def _ptr_array(tensors, dtype):
    return (ctypes.c_void_p * len(tensors))(*[t.data_ptr() if _ptr(t, dtype) else None for t in tensors])


def mq_linear_fwd_multi(X, Q, alpha, zero, rs, extra_precision: bool = False, Y=None, ws=None):
    """X bf16 [M, K], Q uint8 [N, K] -> list of Y_r bf16 [M, N], one per r in rs."""
    M, K = X.shape
    N = Q.shape[0]
    if Q.shape[1] != K:
        raise ValueError("X and Q disagree on K")
    nr = len(rs)
    if Y is None:
        Y = [torch.empty(M, N, dtype=torch.bfloat16, device=X.device) for _ in range(nr)]
    need = mq_workspace_bytes(MQ_OP_LINEAR_FWD, M, N, K, nr)
    if ws is None:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=X.device)
    flags = MQ_FLAG_EXTRA_PRECISION if extra_precision else 0
    st = _lib.mq_linear_fwd_multi(_ptr(X, torch.bfloat16), _ptr(Q, torch.uint8), _ptr(alpha, torch.float32),
                                  _ptr(zero, torch.float32), M, N, K, _int_array(rs), nr, flags,
                                  _ptr_array(Y, torch.bfloat16), _ptr(ws), ws.numel(), _stream())
    _check(st, "mq_linear_fwd_multi")
    return Y


def mq_linear_fwd_multi_noalloc(X, Q, alpha, zero, rs, Y, extra_precision: bool = False):
    """mq_linear_fwd_multi without a workspace (the library's built-in scratch; at most 262144 tokens).  The
    outputs Y are the caller's: nothing is allocated here either."""
    M, K = X.shape
    N = Q.shape[0]
    if Q.shape[1] != K or len(Y) != len(rs):
        raise ValueError("shape mismatch")
    flags = MQ_FLAG_EXTRA_PRECISION if extra_precision else 0
    st = _lib.mq_linear_fwd_multi_noalloc(_ptr(X, torch.bfloat16), _ptr(Q, torch.uint8), _ptr(alpha, torch.float32),
                                          _ptr(zero, torch.float32), M, N, K, _int_array(rs), len(rs), flags,
                                          _ptr_array(Y, torch.bfloat16), _stream())
    _check(st, "mq_linear_fwd_multi_noalloc")
    return Y


def mq_linear_bwd(X, Q, alpha, zero, dY, lambdas, rs, extra_precision: bool = False, need_dX: bool = True,
                  need_dW: bool = True, dX=None, dW=None, accumulate_dW: bool = False, ws=None):
    """STE backward: returns (dX bf16 [M, K] or None, dW fp32 [N, K] or None)."""
    M, K = X.shape
    N = Q.shape[0]
    nr = len(rs)
    if len(dY) != nr:
        raise ValueError("one dY per r")
    if need_dX and dX is None:
        dX = torch.empty(M, K, dtype=torch.bfloat16, device=X.device)
    if need_dW and dW is None:
        dW = torch.zeros(N, K, dtype=torch.float32, device=X.device) if accumulate_dW else \
            torch.empty(N, K, dtype=torch.float32, device=X.device)
    need = mq_workspace_bytes(MQ_OP_LINEAR_BWD, M, N, K, nr)
    if ws is None:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=X.device)
    lam = None
    if lambdas is not None:
        lam = (ctypes.c_float * nr)(*[float(v) for v in lambdas])
    flags = (MQ_FLAG_EXTRA_PRECISION if extra_precision else 0) | (MQ_FLAG_ACCUM_DW if accumulate_dW else 0)
    st = _lib.mq_linear_bwd(_ptr(X, torch.bfloat16), _ptr(Q, torch.uint8), _ptr(alpha, torch.float32),
                            _ptr(zero, torch.float32), _ptr_array(dY, torch.bfloat16), lam, M, N, K,
                            _int_array(rs), nr, flags, _ptr(dX if need_dX else None, torch.bfloat16),
                            _ptr(dW if need_dW else None, torch.float32), _ptr(ws), ws.numel(), _stream())
    _check(st, "mq_linear_bwd")
    return (dX if need_dX else None), (dW if need_dW else None)


def mq_linear_fwd_multi_gated(X, Q, alpha, zero, rs, silu: bool = False, extra_precision: bool = False, GU=None, A=None,
                              store_GU: bool = True, ws=None):
    """Stacked gate / up layer with the gated unit in its epilogue: returns (list of GU_r bf16 [M, 2F] or None, list of
    A_r bf16 [M, F])."""
    M, K = X.shape
    N = Q.shape[0]
    nr = len(rs)
    if Q.shape[1] != K or N % 2:
        raise ValueError("shape mismatch")
    if GU is None and store_GU:
        GU = [torch.empty(M, N, dtype=torch.bfloat16, device=X.device) for _ in range(nr)]
    if A is None:
        A = [torch.empty(M, N // 2, dtype=torch.bfloat16, device=X.device) for _ in range(nr)]
    if ws is None:
        ws = torch.empty(max(mq_workspace_bytes(MQ_OP_LINEAR_FWD, M, N, K, nr), 16), dtype=torch.uint8, device=X.device)
    flags = (MQ_FLAG_EXTRA_PRECISION if extra_precision else 0) | (MQ_FLAG_FFN_SILU if silu else 0)
    st = _lib.mq_linear_fwd_multi_gated(_ptr(X, torch.bfloat16), _ptr(Q, torch.uint8), _ptr(alpha, torch.float32),
                                        _ptr(zero, torch.float32), M, N // 2, K, _int_array(rs), nr, flags,
                                        _ptr_array(GU, torch.bfloat16) if GU is not None else None,
                                        _ptr_array(A, torch.bfloat16), _ptr(ws), ws.numel(), _stream())
    _check(st, "mq_linear_fwd_multi_gated")
    return GU, A


def mq_linear_bwd_gated(X, Q, alpha, zero, GU, dA, lambdas, rs, silu: bool = False, extra_precision: bool = False,
                        need_dX: bool = True, need_dW: bool = True, dX=None, dW=None, accumulate_dW: bool = False, ws=None):
    """Backward of the stacked gate / up layer with the gradient of the gated unit formed on the way: GU[i] bf16
    [M, 2F], dA[i] bf16 [M, F] -> (dX bf16 [M, K] or None, dW fp32 [2F, K] or None)."""
    M, K = X.shape
    N = Q.shape[0]
    nr = len(rs)
    if len(GU) != nr or len(dA) != nr or N % 2:
        raise ValueError("one GU and one dA per r, an even number of stacked rows")
    if need_dX and dX is None:
        dX = torch.empty(M, K, dtype=torch.bfloat16, device=X.device)
    if need_dW and dW is None:
        dW = (torch.zeros if accumulate_dW else torch.empty)(N, K, dtype=torch.float32, device=X.device)
    if ws is None:
        ws = torch.empty(max(mq_workspace_bytes(MQ_OP_LINEAR_BWD, M, N, K, nr), 16), dtype=torch.uint8, device=X.device)
    lam = None if lambdas is None else (ctypes.c_float * nr)(*[float(v) for v in lambdas])
    flags = (MQ_FLAG_EXTRA_PRECISION if extra_precision else 0) | (MQ_FLAG_ACCUM_DW if accumulate_dW else 0) | \
            (MQ_FLAG_FFN_SILU if silu else 0)
    st = _lib.mq_linear_bwd_gated(_ptr(X, torch.bfloat16), _ptr(Q, torch.uint8), _ptr(alpha, torch.float32),
                                  _ptr(zero, torch.float32), _ptr_array(GU, torch.bfloat16), _ptr_array(dA, torch.bfloat16), lam,
                                  M, N // 2, K, _int_array(rs), nr, flags, _ptr(dX if need_dX else None, torch.bfloat16),
                                  _ptr(dW if need_dW else None, torch.float32), _ptr(ws), ws.numel(), _stream())
    _check(st, "mq_linear_bwd_gated")
    return (dX if need_dX else None), (dW if need_dW else None)


def mq_gemv_sliced(x, packed, alpha_bf16, zero_bf16, r: int, K: int, ovf: Overflow | None = None, y=None):
    """x bf16 [B, K], packed uint8 [N, K*r/8] -> y bf16 [B, N]."""
    B = x.shape[0]
    N = packed.shape[0]
    if x.shape[1] != K or packed.shape[1] != K * r // 8:
        raise ValueError("shape mismatch")
    if y is None:
        y = torch.empty(B, N, dtype=torch.bfloat16, device=x.device)
    c_ovf = ctypes.byref(ovf.c_struct()) if ovf is not None else None
    st = _lib.mq_gemv_sliced(_ptr(x, torch.bfloat16), _ptr(packed, torch.uint8), _ptr(alpha_bf16, torch.bfloat16),
                             _ptr(zero_bf16, torch.bfloat16), c_ovf, B, N, K, r, _ptr(y, torch.bfloat16), _stream())
    _check(st, "mq_gemv_sliced")
    return y


def mq_gemv_sliced_ws(x, packed, alpha_bf16, zero_bf16, r: int, K: int, ovf: Overflow | None = None, y=None, ws=None):
    """mq_gemv_sliced with a workspace (allocated here when not given): K may be split over workgroups."""
    B = x.shape[0]
    N = packed.shape[0]
    if x.shape[1] != K or packed.shape[1] != K * r // 8:
        raise ValueError("shape mismatch")
    if y is None:
        y = torch.empty(B, N, dtype=torch.bfloat16, device=x.device)
    if ws is None:
        ws = torch.empty(mq_workspace_bytes(MQ_OP_GEMV, B, N, K, r), dtype=torch.uint8, device=x.device)
    c_ovf = ctypes.byref(ovf.c_struct()) if ovf is not None else None
    st = _lib.mq_gemv_sliced_ws(_ptr(x, torch.bfloat16), _ptr(packed, torch.uint8), _ptr(alpha_bf16, torch.bfloat16),
                                _ptr(zero_bf16, torch.bfloat16), c_ovf, B, N, K, r, _ptr(y, torch.bfloat16),
                                _ptr(ws, torch.uint8), ws.numel(), _stream())
    _check(st, "mq_gemv_sliced_ws")
    return y


def mq_ffn_mixnmatch(x, layers, F: int, silu: bool = False, residual: bool = False, y=None, ws=None):
    """Stack of gated feed-forward layers on the decode path, one bit-width per layer.
    x bf16 [B, d]; layers: sequence of dicts with the device tensors gate_up uint8 [2F, d*r/8],
    down uint8 [d, F*r/8], alpha_gu, zero_gu bf16 [2F], alpha_dn, zero_dn bf16 [d] and the int r."""
    B, d = x.shape
    arr = (_FfnLayer * max(len(layers), 1))()
    for i, L in enumerate(layers):
        r = int(L["r"])
        if tuple(L["gate_up"].shape) != (2 * F, d * r // 8) or tuple(L["down"].shape) != (d, F * r // 8):
            raise ValueError("plane shapes do not match B, d, F, r")
        if L["alpha_gu"].numel() != 2 * F or L["zero_gu"].numel() != 2 * F or L["alpha_dn"].numel() != d \
                or L["zero_dn"].numel() != d:
            raise ValueError("parameter sizes do not match d, F")
        arr[i] = _FfnLayer(_ptr(L["gate_up"], torch.uint8), _ptr(L["down"], torch.uint8),
                           _ptr(L["alpha_gu"], torch.bfloat16), _ptr(L["zero_gu"], torch.bfloat16),
                           _ptr(L["alpha_dn"], torch.bfloat16), _ptr(L["zero_dn"], torch.bfloat16), r)
    if y is None:
        y = torch.empty(B, d, dtype=torch.bfloat16, device=x.device)
    nbytes = mq_workspace_bytes(MQ_OP_FFN_DECODE, B, F, d, 1)
    if ws is None:
        ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=x.device)
    flags = (MQ_FLAG_FFN_SILU if silu else 0) | (MQ_FLAG_FFN_RESIDUAL if residual else 0)
    st = _lib.mq_ffn_mixnmatch(_ptr(x, torch.bfloat16), arr, len(layers), B, d, F, flags, _ptr(y, torch.bfloat16),
                               _ptr(ws, torch.uint8), ws.numel(), _stream())
    _check(st, "mq_ffn_mixnmatch")
    return y


def mq_matquant_l2_loss(Y, target=None, teacher=None, lambdas=None, mix: bool = False, dY=None, losses=None, ws=None):
    """L2 reconstruction losses of the bit-widths' outputs Y (list of bf16 [M, N]) against the target (bf16 [M, N])
    or against another output (teacher[i] = its index, -1 = the target), and the gradients dY the backward takes.
    Returns (losses fp32 [nr] on the GPU, list of dY bf16 [M, N])."""
    nr = len(Y)
    M, N = Y[0].shape
    if dY is None:
        dY = [torch.empty(M, N, dtype=torch.bfloat16, device=Y[0].device) for _ in range(nr)]
    if losses is None:
        losses = torch.empty(nr, dtype=torch.float32, device=Y[0].device)
    nbytes = mq_workspace_bytes(MQ_OP_L2_LOSS, M, N, 0, max(1, min(nr, 3)))
    if ws is None:
        ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=Y[0].device)
    c_teacher = (ctypes.c_int * nr)(*teacher) if teacher is not None else None
    c_lambda = (ctypes.c_float * nr)(*lambdas) if lambdas is not None else None
    st = _lib.mq_matquant_l2_loss(_ptr_array(Y, torch.bfloat16), _ptr(target, torch.bfloat16), c_teacher, c_lambda, M, N, nr,
                                  MQ_FLAG_LOSS_MIX if mix else 0, _ptr_array(dY, torch.bfloat16),
                                  _ptr(losses, torch.float32), _ptr(ws, torch.uint8), ws.numel(), _stream())
    _check(st, "mq_matquant_l2_loss")
    return losses, dY


def mq_linear_fwd_multi_l2(X, Q, alpha, zero, rs, target=None, teacher=None, lambdas=None, mix: bool = False,
                           extra_precision: bool = False, Y=None, dY=None, losses=None, ws=None, bias=None):
    """Forward for every r in rs with the L2 objective evaluated in the same pass: returns (losses fp32 [nr] on the
    GPU, list of dY bf16 [M, N]).  Y, if given, is a list of nr bf16 [M, N] tensors or None entries; only the tensors
    present are written."""
    M, K = X.shape
    N = Q.shape[0]
    if Q.shape[1] != K:
        raise ValueError("X and Q disagree on K")
    nr = len(rs)
    if dY is None:
        dY = [torch.empty(M, N, dtype=torch.bfloat16, device=X.device) for _ in range(nr)]
    if losses is None:
        losses = torch.empty(nr, dtype=torch.float32, device=X.device)
    need = mq_workspace_bytes(MQ_OP_LINEAR_FWD_L2, M, N, K, max(1, min(nr, 3)))
    if ws is None:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=X.device)
    flags = (MQ_FLAG_EXTRA_PRECISION if extra_precision else 0) | (MQ_FLAG_LOSS_MIX if mix else 0)
    c_teacher = (ctypes.c_int * nr)(*teacher) if teacher is not None else None
    c_lambda = (ctypes.c_float * nr)(*lambdas) if lambdas is not None else None
    c_Y = None
    if Y is not None:
        c_Y = (ctypes.c_void_p * nr)(*[_ptr(t, torch.bfloat16) if t is not None else None for t in Y])
    st = _lib.mq_linear_fwd_multi_l2(_ptr(X, torch.bfloat16), _ptr(Q, torch.uint8), _ptr(alpha, torch.float32),
                                     _ptr(zero, torch.float32), M, N, K, _int_array(rs), nr, flags,
                                     _ptr(bias, torch.float32), _ptr(target, torch.bfloat16), c_teacher, c_lambda, c_Y,
                                     _ptr_array(dY, torch.bfloat16), _ptr(losses, torch.float32), _ptr(ws),
                                     ws.numel(), _stream())
    _check(st, "mq_linear_fwd_multi_l2")
    return losses, dY


def mq_linear_bwd_clip(W, X, Q, alpha, zero, dY, lambdas, rs, gamma=None, beta=None, extra_precision: bool = False,
                       want_dalpha_dzero: bool = False, ws=None):
    """Gradients with respect to the clip factors of the quantizer: returns (dgamma, dbeta) fp32 [N], or
    (dgamma, dbeta, dalpha, dzero) with want_dalpha_dzero."""
    M, K = X.shape
    N = Q.shape[0]
    nr = len(rs)
    if len(dY) != nr:
        raise ValueError("one dY per r")
    if W.stride(1) != 1 or W.shape != (N, K):
        raise ValueError("W must be [N, K] with unit column stride")
    out = [torch.empty(N, dtype=torch.float32, device=X.device) for _ in range(4 if want_dalpha_dzero else 2)]
    need = mq_workspace_bytes(MQ_OP_LINEAR_BWD_CLIP, M, N, K, max(1, min(nr, 3)))
    if ws is None:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=X.device)
    lam = (ctypes.c_float * nr)(*lambdas) if lambdas is not None else None
    flags = MQ_FLAG_EXTRA_PRECISION if extra_precision else 0
    if W.dtype != torch.float32 or not W.is_cuda:
        raise ValueError("W must be a float32 tensor on the GPU")
    st = _lib.mq_linear_bwd_clip(ctypes.c_void_p(W.data_ptr()), W.stride(0), _ptr(X, torch.bfloat16), _ptr(Q, torch.uint8),
                                 _ptr(alpha, torch.float32), _ptr(zero, torch.float32), _ptr(gamma, torch.float32),
                                 _ptr(beta, torch.float32), _ptr_array(dY, torch.bfloat16), lam, M, N, K, _int_array(rs), nr,
                                 flags, _ptr(out[0]), _ptr(out[1]), _ptr(out[2]) if want_dalpha_dzero else None,
                                 _ptr(out[3]) if want_dalpha_dzero else None, _ptr(ws), ws.numel(), _stream())
    _check(st, "mq_linear_bwd_clip")
    return tuple(out)


def mq_affine_weight(W, s=None, delta=None, b=None, want_Ws: bool = True, want_c: bool = True):
    """Weight side of the affine re-parameterisation: returns (Ws fp32 [N, K] or None, c fp32 [N] or None)."""
    N, K = W.shape
    if W.dtype != torch.float32 or not W.is_cuda or W.stride(1) != 1:
        raise ValueError("W must be a float32 GPU tensor with unit column stride")
    Ws = torch.empty(N, K, dtype=torch.float32, device=W.device) if want_Ws else None
    c = torch.empty(N, dtype=torch.float32, device=W.device) if want_c else None
    st = _lib.mq_affine_weight(ctypes.c_void_p(W.data_ptr()), N, K, W.stride(0), _ptr(s, torch.float32),
                               _ptr(delta, torch.float32), _ptr(b, torch.float32), _ptr(Ws), _ptr(c), _stream())
    _check(st, "mq_affine_weight")
    return Ws, c


def mq_affine_input(X, s=None, delta=None, Xt=None):
    """Xt = bf16((X - delta) / s) per input feature."""
    M, K = X.shape
    if Xt is None:
        Xt = torch.empty_like(X)
    st = _lib.mq_affine_input(_ptr(X, torch.bfloat16), M, K, _ptr(s, torch.float32), _ptr(delta, torch.float32),
                              _ptr(Xt, torch.bfloat16), _stream())
    _check(st, "mq_affine_input")
    return Xt


def mq_affine_bwd(X, dXt, W, dWs, dY, lambdas, s=None, delta=None, ws=None):
    """Gradients with respect to delta and s (and the bias gradient dc): returns (ddelta [K], ds [K], dc [N]) fp32."""
    M, K = X.shape
    N = W.shape[0]
    nr = len(dY)
    out = (torch.empty(K, dtype=torch.float32, device=X.device), torch.empty(K, dtype=torch.float32, device=X.device),
           torch.empty(N, dtype=torch.float32, device=X.device))
    need = mq_workspace_bytes(MQ_OP_AFFINE_BWD, M, N, K, max(1, min(nr, 3)))
    if ws is None:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=X.device)
    lam = (ctypes.c_float * nr)(*lambdas) if lambdas is not None else None
    if W.dtype != torch.float32 or W.stride(1) != 1:
        raise ValueError("W must be float32 with unit column stride")
    st = _lib.mq_affine_bwd(_ptr(X, torch.bfloat16), _ptr(dXt, torch.bfloat16), ctypes.c_void_p(W.data_ptr()), W.stride(0),
                            _ptr(dWs, torch.float32), _ptr_array(dY, torch.bfloat16), lam, nr, M, N, K,
                            _ptr(s, torch.float32), _ptr(delta, torch.float32), _ptr(out[0]), _ptr(out[1]), _ptr(out[2]),
                            _ptr(ws), ws.numel(), _stream())
    _check(st, "mq_affine_bwd")
    return out


def mq_gated_unit_fwd(GU, silu: bool = False, A=None):
    """GU: list of bf16 [M, 2F] (gate / up columns interleaved) -> list of A bf16 [M, F] = act(gate) * up."""
    M, F2 = GU[0].shape
    F = F2 // 2
    if A is None:
        A = [torch.empty(M, F, dtype=torch.bfloat16, device=GU[0].device) for _ in GU]
    st = _lib.mq_gated_unit_fwd(_ptr_array(GU, torch.bfloat16), len(GU), M, F, MQ_FLAG_FFN_SILU if silu else 0,
                                _ptr_array(A, torch.bfloat16), _stream())
    _check(st, "mq_gated_unit_fwd")
    return A


def mq_gated_unit_bwd(GU, dA, silu: bool = False, dGU=None):
    """Backward of mq_gated_unit_fwd: list of dGU bf16 [M, 2F]."""
    M, F2 = GU[0].shape
    F = F2 // 2
    if dGU is None:
        dGU = [torch.empty(M, F2, dtype=torch.bfloat16, device=GU[0].device) for _ in GU]
    st = _lib.mq_gated_unit_bwd(_ptr_array(GU, torch.bfloat16), _ptr_array(dA, torch.bfloat16), len(GU), M, F,
                                MQ_FLAG_FFN_SILU if silu else 0, _ptr_array(dGU, torch.bfloat16), _stream())
    _check(st, "mq_gated_unit_bwd")
    return dGU

