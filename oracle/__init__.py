"""CPU oracle for the Matryoshka-Quantization nested quantized linear layer.

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the bench's cpu_baseline
leg may import this package; the product path never does.  It wraps the plain
C functions of ``mq_oracle.c`` (numpy arrays in, numpy arrays out) and shares
nothing with the HIP path.  bf16 tensors travel as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mq_oracle.c")
_LIB = os.path.join(_HERE, "libmq_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile mq_oracle.c with gcc (fp contraction off, OpenMP on)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.mqo_overflow_csr.restype = ctypes.c_int64
        _lib.mqo_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i64(v):
    return ctypes.c_int64(int(v))


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(_load().mqo_num_threads())


# --------------------------------------------------------------------------
# quantize / slice / pack
# --------------------------------------------------------------------------
def quantize_int8(W, gamma=None, beta=None):
    """MinMax quantizer (section 3.1.1), optional clip factors (section 3.1.2).

    W float32 [N, K] -> (q uint8 [N, K], alpha float32 [N], zero float32 [N]).
    """
    W = _c(W, np.float32)
    N, K = W.shape
    g = None if gamma is None else _c(gamma, np.float32)
    b = None if beta is None else _c(beta, np.float32)
    q = np.empty((N, K), np.uint8)
    alpha = np.empty(N, np.float32)
    zero = np.empty(N, np.float32)
    _load().mqo_quantize_int8(_p(W), _i64(N), _i64(K), _i64(K), _p(g), _p(b), _p(q), _p(alpha), _p(zero))
    return q, alpha, zero


def slice_codes(q, r: int, ep: bool = False):
    """r-bit code of every int8 code (slicing equation, section 3.2; ep: errata)."""
    q = _c(q, np.uint8)
    out = np.empty(q.shape, np.uint8)
    _load().mqo_slice_codes(_p(q), _i64(q.size), ctypes.c_int(r), ctypes.c_int(int(ep)), _p(out))
    return out


def slice_values(q, r: int, ep: bool = False):
    """S(q, r) on the int8 grid as uint16 (256 is reachable with ep)."""
    q = _c(q, np.uint8)
    out = np.empty(q.shape, np.uint16)
    _load().mqo_slice_values(_p(q), _i64(q.size), ctypes.c_int(r), ctypes.c_int(int(ep)), _p(out))
    return out


def pack(codes, r: int):
    codes = _c(codes, np.uint8)
    N, K = codes.shape
    assert 1 <= r <= 8 and (K * r) % 8 == 0
    assert int(codes.max(initial=0)) < (1 << r)
    out = np.empty((N, K * r // 8), np.uint8)
    _load().mqo_pack(_p(codes), _i64(N), _i64(K), ctypes.c_int(r), _p(out))
    return out


def unpack(packed, K: int, r: int):
    packed = _c(packed, np.uint8)
    N = packed.shape[0]
    out = np.empty((N, K), np.uint8)
    _load().mqo_unpack(_p(packed), _i64(N), _i64(K), ctypes.c_int(r), _p(out))
    return out


def overflow_csr(q, r: int):
    """Extra-precision overflow set as (row_ptr int32 [N+1], col_idx uint16 [nnz])."""
    q = _c(q, np.uint8)
    N, K = q.shape
    assert K <= 65536
    row_ptr = np.empty(N + 1, np.int32)
    cap = q.size
    col = np.empty(cap, np.uint16)
    nnz = _load().mqo_overflow_csr(_p(q), _i64(N), _i64(K), ctypes.c_int(r), _p(row_ptr), _p(col), _i64(cap))
    return row_ptr, col[:nnz].copy()


def dequant(q, alpha, zero, r: int, ep: bool = False):
    q = _c(q, np.uint8)
    N, K = q.shape
    alpha = _c(alpha, np.float32)
    zero = _c(zero, np.float32)
    out = np.empty((N, K), np.float64)
    _load().mqo_dequant(_p(q), _p(alpha), _p(zero), _i64(N), _i64(K), ctypes.c_int(r), ctypes.c_int(int(ep)), _p(out))
    return out


# --------------------------------------------------------------------------
# forward / backward / gemv
# --------------------------------------------------------------------------
def linear_fwd(X_bf16, q, alpha, zero, r: int, ep: bool = False):
    """Y_r = X . What_r^T in fp64.  X_bf16: uint16 [M, K]."""
    X = _c(X_bf16, np.uint16)
    q = _c(q, np.uint8)
    M, K = X.shape
    N = q.shape[0]
    assert q.shape[1] == K
    alpha = _c(alpha, np.float32)
    zero = _c(zero, np.float32)
    Y = np.empty((M, N), np.float64)
    _load().mqo_linear_fwd(_p(X), _p(q), _p(alpha), _p(zero), _i64(M), _i64(N), _i64(K),
                           ctypes.c_int(r), ctypes.c_int(int(ep)), _p(Y))
    return Y


def linear_fwd_sampled(X_bf16, q, alpha, zero, r: int, ms, ns, ep: bool = False):
    X = _c(X_bf16, np.uint16)
    q = _c(q, np.uint8)
    M, K = X.shape
    N = q.shape[0]
    alpha = _c(alpha, np.float32)
    zero = _c(zero, np.float32)
    ms = _c(ms, np.int64)
    ns = _c(ns, np.int64)
    out = np.empty(ms.size, np.float64)
    _load().mqo_linear_fwd_sampled(_p(X), _p(q), _p(alpha), _p(zero), _i64(M), _i64(N), _i64(K),
                                   ctypes.c_int(r), ctypes.c_int(int(ep)), _p(ms), _p(ns),
                                   _i64(ms.size), _p(out))
    return out


def _ptr_array(arrs):
    arr_t = ctypes.c_void_p * len(arrs)
    return arr_t(*[a.ctypes.data for a in arrs])


def _lam(lambdas, nr):
    if lambdas is None:
        return None
    lam = _c(lambdas, np.float32)
    assert lam.size == nr
    return lam


def linear_bwd_dx(q, alpha, zero, dYs_bf16, lambdas, rs, ep: bool = False):
    """dX = sum_r lambda_r dY_r . What_r in fp64 (identity STE)."""
    q = _c(q, np.uint8)
    N, K = q.shape
    dYs = [_c(d, np.uint16) for d in dYs_bf16]
    M = dYs[0].shape[0]
    alpha = _c(alpha, np.float32)
    zero = _c(zero, np.float32)
    lam = _lam(lambdas, len(rs))
    rs_c = (ctypes.c_int * len(rs))(*rs)
    dX = np.empty((M, K), np.float64)
    _load().mqo_linear_bwd_dx(_p(q), _p(alpha), _p(zero), _ptr_array(dYs), _p(lam), _i64(M), _i64(N),
                              _i64(K), rs_c, ctypes.c_int(len(rs)), ctypes.c_int(int(ep)), _p(dX))
    return dX


def linear_bwd_dx_sampled(q, alpha, zero, dYs_bf16, lambdas, rs, ms, ks, ep: bool = False):
    q = _c(q, np.uint8)
    N, K = q.shape
    dYs = [_c(d, np.uint16) for d in dYs_bf16]
    M = dYs[0].shape[0]
    alpha = _c(alpha, np.float32)
    zero = _c(zero, np.float32)
    lam = _lam(lambdas, len(rs))
    rs_c = (ctypes.c_int * len(rs))(*rs)
    ms = _c(ms, np.int64)
    ks = _c(ks, np.int64)
    out = np.empty(ms.size, np.float64)
    _load().mqo_linear_bwd_dx_sampled(_p(q), _p(alpha), _p(zero), _ptr_array(dYs), _p(lam), _i64(M),
                                      _i64(N), _i64(K), rs_c, ctypes.c_int(len(rs)),
                                      ctypes.c_int(int(ep)), _p(ms), _p(ks), _i64(ms.size), _p(out))
    return out


def linear_bwd_dw(X_bf16, dYs_bf16, lambdas):
    """dW = (sum_r lambda_r dY_r)^T . X in fp64; independent of the codes."""
    X = _c(X_bf16, np.uint16)
    M, K = X.shape
    dYs = [_c(d, np.uint16) for d in dYs_bf16]
    N = dYs[0].shape[1]
    lam = _lam(lambdas, len(dYs))
    dW = np.empty((N, K), np.float64)
    _load().mqo_linear_bwd_dw(_p(X), _ptr_array(dYs), _p(lam), _i64(M), _i64(N), _i64(K),
                              ctypes.c_int(len(dYs)), _p(dW))
    return dW


def linear_bwd_dw_sampled(X_bf16, dYs_bf16, lambdas, ns, ks):
    X = _c(X_bf16, np.uint16)
    M, K = X.shape
    dYs = [_c(d, np.uint16) for d in dYs_bf16]
    N = dYs[0].shape[1]
    lam = _lam(lambdas, len(dYs))
    ns = _c(ns, np.int64)
    ks = _c(ks, np.int64)
    out = np.empty(ns.size, np.float64)
    _load().mqo_linear_bwd_dw_sampled(_p(X), _ptr_array(dYs), _p(lam), _i64(M), _i64(N), _i64(K),
                                      ctypes.c_int(len(dYs)), _p(ns), _p(ks), _i64(ns.size), _p(out))
    return out


def gemv_sliced(x_bf16, packed, alpha_bf16, zero_bf16, r: int, K: int, ovf=None, shift: int = -1):
    """y = x . What_r^T from a packed plane with bf16 alpha, z; ovf = (row_ptr, col_idx) or None.
    shift: s of the grid the stored codes live on (default 8 - r); a dense extra-precision plane of the
    rv-bit slice is read with r = rv + 1, shift = 8 - rv."""
    x = _c(x_bf16, np.uint16)
    B = x.shape[0]
    assert x.shape[1] == K
    packed = _c(packed, np.uint8)
    N = packed.shape[0]
    assert packed.shape[1] == K * r // 8
    a = _c(alpha_bf16, np.uint16)
    z = _c(zero_bf16, np.uint16)
    rp = ci = None
    if ovf is not None:
        rp = _c(ovf[0], np.int32)
        ci = _c(ovf[1], np.uint16)
    y = np.empty((B, N), np.float64)
    _load().mqo_gemv_sliced(_p(x), _p(packed), _p(a), _p(z), _p(rp), _p(ci), _i64(B), _i64(N), _i64(K),
                            ctypes.c_int(r), ctypes.c_int(shift), _p(y))
    return y


def bf16_round(v):
    """fp64 array -> bf16 bit patterns (uint16): to fp32, then round-to-nearest-even on the upper 16 bits."""
    u = np.ascontiguousarray(v, dtype=np.float64).astype(np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f64(bits):
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def ffn_mixnmatch(x_bf16, layers, d: int, F: int, silu: bool = False, residual: bool = False):
    """Layer-wise Mix'n'Match on the decode path (section 4.3, appendix B): a stack of gated feed-forward
    layers, layer l read at its own bit-width r_l,
        g, u = W_gate h, W_up h;  a = act(g) * u;  o = W_down a;  h <- o  (or h + o)
    with the matrix-vector products of gemv_sliced (fp64) and every intermediate rounded to bf16.
    act = GELU in its tanh form (default) or SiLU.  layers: dicts with gate_up [2F, d*r/8] (gate and up rows interleaved, gate first), down
    [d, F*r/8] (packed uint8), alpha_gu, zero_gu [2F], alpha_dn, zero_dn [d] (bf16 bit patterns), r.
    Returns (y as bf16 bit patterns [B, d], the last layer's output before its final rounding, fp64)."""
    h = _c(x_bf16, np.uint16)
    last = bf16_to_f64(h)
    for L in layers:
        r = int(L["r"])
        gu = bf16_to_f64(bf16_round(gemv_sliced(h, L["gate_up"], L["alpha_gu"], L["zero_gu"], r, d)))
        g, u = gu[:, 0::2], gu[:, 1::2]      # row 2 f of the plane is gate row f, row 2 f + 1 up row f
        if silu:
            with np.errstate(over="ignore"):  # exp(-g) = inf for very negative g gives the limit -0
                act = g / (1.0 + np.exp(-g))
        else:
            act = 0.5 * g * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (g + 0.044715 * g ** 3)))
        a = bf16_round(act * u)
        o = gemv_sliced(a, L["down"], L["alpha_dn"], L["zero_dn"], r, F)
        if residual:
            o = bf16_to_f64(h) + bf16_to_f64(bf16_round(o))
        last = o
        h = bf16_round(o)
    return h, last


def matquant_l2_loss(Ys_bf16, target_bf16=None, teacher=None, lambdas=None, mix: bool = False):
    """Joint objective of section 3.2 with the layer-wise L2 loss of section 3.1.2 and the co-distillation
    targets of section 5.2, in fp64: loss_i = mean((Y_i - T_i)^2) with T_i the target (teacher[i] < 0) or the
    output Y_teacher[i] held constant; with mix, the equal-weight mean of both losses.  Returns
    (losses [nr], dYs = d(sum_i lambda_i loss_i)/dY_i as fp64 arrays)."""
    Ys = [bf16_to_f64(y) for y in Ys_bf16]
    nr = len(Ys)
    T = None if target_bf16 is None else bf16_to_f64(target_bf16)
    teacher = [-1] * nr if teacher is None else list(teacher)
    lam = [1.0] * nr if lambdas is None else [float(v) for v in lambdas]
    mn = Ys[0].size
    losses, dYs = [], []
    for i in range(nr):
        t = teacher[i]
        if t < 0:
            diff = Ys[i] - T
            losses.append(float((diff ** 2).sum() / mn))
            dYs.append(lam[i] * 2.0 * diff / mn)
        elif not mix:
            diff = Ys[i] - Ys[t]
            losses.append(float((diff ** 2).sum() / mn))
            dYs.append(lam[i] * 2.0 * diff / mn)
        else:
            d1, d2 = Ys[i] - Ys[t], Ys[i] - T
            losses.append(float(0.5 * ((d1 ** 2).sum() + (d2 ** 2).sum()) / mn))
            dYs.append(lam[i] * (d1 + d2) / mn)
    return np.array(losses), dYs


def clip_factor_grads(W, X_bf16, dYs_bf16, lambdas, rs, gamma=None, beta=None, ep: bool = False):
    """Gradients of  sum_r lambda_r <dY_r, X What_r^T>  with respect to the clip factors gamma, beta of the
    quantizer of section 3.1.2 (alpha = (gamma max - beta min) / 255, z = -beta min / alpha), under the
    straight-through estimator the section names: both roundings (to the 8-bit code and, in the slicing of
    section 3.2, to the r-bit code) pass the gradient unchanged, both clamps (to 0..255, and to the top code
    2^r - 1 of a slice) pass it only where they do not act.  With u = w / alpha + z and What_r = alpha (S_r - z):
        d What_r / d alpha = (S_r - z) - m_r w / alpha        d What_r / d z = -alpha (1 - m_r)
    where m_r = 1 where neither clamp acts.  The clamp decisions are the quantizer's own (fp32); everything
    else is fp64.  Rows with gamma max == beta min (alpha set to 1 by the quantizer) get zero gradients.
    Returns (dgamma, dbeta, dalpha, dzero), each [N] fp64."""
    W32 = _c(W, np.float32)
    N, K = W32.shape
    g32 = None if gamma is None else _c(gamma, np.float32)
    b32 = None if beta is None else _c(beta, np.float32)
    q, alpha32, zero32 = quantize_int8(W32, g32, b32)
    # the quantizer's rounding, before its clamp, in its own precision and operation order
    t32 = (W32 / alpha32[:, None]).astype(np.float32)
    u32 = (t32 + zero32[:, None]).astype(np.float32)
    rounded = np.rint(u32)
    inside = (rounded >= 0.0) & (rounded <= 255.0)
    Wd, a, z = W32.astype(np.float64), alpha32.astype(np.float64), zero32.astype(np.float64)
    X = bf16_to_f64(X_bf16)
    dalpha, dzero = np.zeros(N), np.zeros(N)
    for r, dY, lam in zip(rs, dYs_bf16, lambdas):
        dWhat = float(lam) * (bf16_to_f64(dY).T @ X)                     # [N, K]: d objective / d What_r
        s = 8 - int(r)
        raw = (q.astype(np.int64) + ((1 << s) >> 1)) >> s
        top = np.zeros_like(inside) if ep else raw > (1 << r) - 1
        code = raw if ep else np.minimum(raw, (1 << r) - 1)
        S = (code << s).astype(np.float64)
        m = (inside & ~top).astype(np.float64)
        dalpha += (dWhat * ((S - z[:, None]) - m * Wd / a[:, None])).sum(axis=1)
        dzero += (dWhat * (-a[:, None] * (1.0 - m))).sum(axis=1)
    mn, mx = Wd.min(axis=1), Wd.max(axis=1)
    gam = np.ones(N) if g32 is None else g32.astype(np.float64)
    bet = np.ones(N) if b32 is None else b32.astype(np.float64)
    live = (gam * mx != bet * mn).astype(np.float64)
    da_dg, da_db = mx / 255.0, -mn / 255.0
    dz_dg = (bet * mn / a ** 2) * da_dg
    dz_db = -mn / a + (bet * mn / a ** 2) * da_db
    dgamma = live * (dalpha * da_dg + dzero * dz_dg)
    dbeta = live * (dalpha * da_db + dzero * dz_db)
    return dgamma, dbeta, dalpha, dzero


def affine_weight(W, s=None, delta=None, b=None):
    """Weight side of the learnable affine re-parameterisation of a projection (section 3.1.2, the equation
    X W + b -> ((X - delta) / s) Q(W * s) + b + delta W):  Ws = W * s is what the quantizer is given, so it is formed
    exactly as the quantizer will see it, one fp32 product per weight;  c = b + W delta (fp64) is the bias of
    the transformed layer.  W is [N, K] (out x in), s and delta are per input feature [K].  Returns (Ws fp32, c fp64)."""
    W32 = _c(W, np.float32)
    N, K = W32.shape
    Ws = W32 if s is None else (W32 * _c(s, np.float32)[None, :]).astype(np.float32)
    c = np.zeros(N) if b is None else np.asarray(b, dtype=np.float64).copy()
    if delta is not None:
        c = c + W32.astype(np.float64) @ np.asarray(delta, dtype=np.float64)
    return Ws, c


def affine_input(X_bf16, s=None, delta=None):
    """Input side of the same equation: (X - delta) / s per input feature, fp64, rounded once to bf16 (bit patterns)."""
    X = bf16_to_f64(X_bf16)
    if delta is not None:
        X = X - np.asarray(delta, dtype=np.float64)[None, :]
    if s is not None:
        X = X / np.asarray(s, dtype=np.float64)[None, :]
    return bf16_round(X)


def affine_bwd(X_bf16, dXt_bf16, W, dWs, dYs_bf16, lambdas, s, delta):
    """Gradients of the objective with respect to delta and s of the same equation, given the gradients the
    straight-through backward of the transformed layer returns: dXt = d/d((X - delta)/s) [M, K] and
    dWs = d/d(W * s) [N, K] (identity through the quantizer).  With dc_n = sum_r lambda_r sum_m dY_r[m, n],
        ddelta_k = -(1/s_k) sum_m dXt[m,k] + sum_n dc_n W[n,k]
        ds_k     = -(1/s_k^2) sum_m dXt[m,k] (X[m,k] - delta_k) + sum_n dWs[n,k] W[n,k]
    The dependence of the quantizer's range on s (through max and min of W * s) carries no gradient, like the
    weights themselves under the clip-factor reading.  Returns (ddelta, ds, dc), fp64."""
    X = bf16_to_f64(X_bf16)
    dXt = bf16_to_f64(dXt_bf16)
    Wd = np.asarray(W, dtype=np.float64)
    dWs = np.asarray(dWs, dtype=np.float64)
    s = np.asarray(s, dtype=np.float64)
    delta = np.asarray(delta, dtype=np.float64)
    dc = np.zeros(Wd.shape[0])
    for dY, lam in zip(dYs_bf16, lambdas):
        dc += float(lam) * bf16_to_f64(dY).sum(axis=0)
    ddelta = -dXt.sum(axis=0) / s + dc @ Wd
    ds = -(dXt * (X - delta[None, :])).sum(axis=0) / s ** 2 + (dWs * Wd).sum(axis=0)
    return ddelta, ds, dc


def _gate_act(g, silu: bool):
    if silu:
        with np.errstate(over="ignore"):
            return g / (1.0 + np.exp(-g))
    return 0.5 * g * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (g + 0.044715 * g ** 3)))


def gated_unit(GU_bf16, silu: bool = False):
    """The gate of the feed-forward block on the training path: GU [M, 2F] bf16 holds the outputs of the stacked
    gate / up projection with the columns of a pair next to each other (gate first, as the rows of the plane in
    ffn_mixnmatch); a[m, f] = act(g) * u in fp64, rounded once to bf16 (bit patterns)."""
    GU = bf16_to_f64(GU_bf16)
    return bf16_round(_gate_act(GU[:, 0::2], silu) * GU[:, 1::2])


def gated_unit_bwd(GU_bf16, dA_bf16, silu: bool = False):
    """Its backward: dg = dA u act'(g), du = dA act(g), interleaved like GU; fp64.
    GELU (tanh form): act'(g) = (1 + th)/2 + g (1 - th^2) c (1 + 3 * 0.044715 g^2) / 2 with th = tanh(c (g + 0.044715 g^3)),
    c = sqrt(2 / pi);  SiLU: act'(g) = sig (1 + g (1 - sig))."""
    GU = bf16_to_f64(GU_bf16)
    dA = bf16_to_f64(dA_bf16)
    g, u = GU[:, 0::2], GU[:, 1::2]
    if silu:
        with np.errstate(over="ignore"):
            sig = 1.0 / (1.0 + np.exp(-g))
        dact = sig * (1.0 + g * (1.0 - sig))
    else:
        c = np.sqrt(2.0 / np.pi)
        th = np.tanh(c * (g + 0.044715 * g ** 3))
        dact = 0.5 * (1.0 + th) + 0.5 * g * (1.0 - th ** 2) * c * (1.0 + 3 * 0.044715 * g ** 2)
    out = np.empty_like(GU)
    out[:, 0::2] = dA * u * dact
    out[:, 1::2] = dA * _gate_act(g, silu)
    return out

