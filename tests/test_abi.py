"""The C-ABI library without a GPU: it loads, exports every function include/mq.h declares, and its
host-side argument checks answer with the documented status codes before anything is launched.

Only calls that return before the first launch are made here (bad sizes, bad bit-widths, null
pointers, sizes of zero); compute calls live in the GPU tests.
"""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mq.h")
LIB = os.path.join(ROOT, "paper_2502_06786_amd", "libmq.so")

OK, NULL, SHAPE, BITS, ALIGN, WORKSPACE, CAPACITY, DEVICE = range(8)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"\b(mq_[a-z0-9_]+)\s*\(", text)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} is not built (python -c 'import __graft_entry__ as g; g.build()')")
    lib_ = ctypes.CDLL(LIB)
    vp, i64, ci, u32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32, ctypes.c_size_t
    lib_.mq_quantize_int8.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp, vp, vp]
    lib_.mq_slice.argtypes = [vp, i64, i64, ci, u32, vp, vp, vp]
    lib_.mq_linear_fwd_multi.argtypes = [vp, vp, vp, vp, i64, i64, i64, ctypes.POINTER(ci), ci, u32, vp, vp, sz, vp]
    lib_.mq_linear_fwd_multi_noalloc.argtypes = [vp, vp, vp, vp, i64, i64, i64, ctypes.POINTER(ci), ci, u32, vp, vp]
    lib_.mq_slice_multi.argtypes = [vp, i64, i64, ctypes.POINTER(ci), ci, u32, vp, ci, vp, vp]
    lib_.mq_linear_fwd_multi_gated.argtypes = [vp, vp, vp, vp, i64, i64, i64, ctypes.POINTER(ci), ci, u32, vp, vp, vp, sz, vp]
    lib_.mq_linear_bwd_gated.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, ctypes.POINTER(ci), ci, u32, vp, vp, vp, sz, vp]
    lib_.mq_linear_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, ctypes.POINTER(ci), ci, u32, vp, vp, vp, sz, vp]
    lib_.mq_gemv_sliced.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, vp]
    lib_.mq_gemv_sliced_ws.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, vp, sz, vp]
    lib_.mq_params_to_bf16.argtypes = [vp, vp, i64, vp, vp, vp]
    lib_.mq_gemv_sliced_dense_ep.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, vp, vp]
    lib_.mq_matquant_l2_loss.argtypes = [vp, vp, ctypes.POINTER(ci), vp, i64, i64, ci, u32, vp, vp, vp, sz, vp]
    lib_.mq_linear_fwd_multi_l2.argtypes = [vp, vp, vp, vp, i64, i64, i64, ctypes.POINTER(ci), ci, u32, vp, vp,
                                            ctypes.POINTER(ci), vp, vp, vp, vp, vp, sz, vp]
    lib_.mq_gated_unit_fwd.argtypes = [vp, ci, i64, i64, u32, vp, vp]
    lib_.mq_gated_unit_bwd.argtypes = [vp, vp, ci, i64, i64, u32, vp, vp]
    lib_.mq_affine_weight.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp, vp, vp]
    lib_.mq_affine_input.argtypes = [vp, i64, i64, vp, vp, vp, vp]
    lib_.mq_affine_bwd.argtypes = [vp, vp, vp, i64, vp, vp, vp, ci, i64, i64, i64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib_.mq_linear_bwd_clip.argtypes = [vp, i64, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, ctypes.POINTER(ci), ci, u32,
                                        vp, vp, vp, vp, vp, sz, vp]
    lib_.mq_ffn_mixnmatch.argtypes = [vp, vp, ci, i64, i64, i64, u32, vp, vp, sz, vp]
    lib_.mq_workspace_bytes.argtypes = [ci, i64, i64, i64, ci]
    lib_.mq_workspace_bytes.restype = sz
    lib_.mq_status_string.argtypes = [ci]
    lib_.mq_status_string.restype = ctypes.c_char_p
    return lib_


def test_header_declares_the_five_calls():
    names = set(declared_functions())
    assert {"mq_quantize_int8", "mq_slice", "mq_linear_fwd_multi", "mq_linear_bwd", "mq_gemv_sliced"} <= names


def test_library_exports_every_declared_function(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_names_match_the_header():
    # (the binding module itself needs torch and loads the library on import)
    from paper_2502_06786_amd import binding
    assert sorted(binding.EXPORTS) == sorted(set(declared_functions()))
    for name in binding.EXPORTS:
        public = "status_string" if name == "mq_status_string" else name
        assert callable(getattr(binding, public)), name


def test_status_strings(lib):
    seen = {lib.mq_status_string(c).decode() for c in range(8)}
    assert len(seen) == 8 and "ok" in seen
    assert lib.mq_status_string(99).decode() == "unknown status"


def test_workspace_bytes(lib):
    f = lib.mq_workspace_bytes
    M, N, K = 4096, 9216, 2304
    fwd, bwd = f(0, M, N, K, 3), f(1, M, N, K, 3)
    assert fwd >= 4 * M
    # three scaled gradient copies + transposed gradient sum + X^T + Q^T
    assert bwd >= 3 * M * N * 2 + M * N * 2 + M * K * 2 + N * K
    assert f(1, M, N, K, 1) < bwd
    # dW tiles of 256 x 256 on 256 compute units: the tiles of a last partial round (at most half a round) are cut into
    # token ranges that leave fp32 partial tiles in the workspace: 784 tiles on the 9B gate shape = 3 rounds + 16 tiles,
    # 16 ranges each; none when the last round is more than half full (289 + ... tiles) or there is less than one round
    base9 = 3 * 8192 * 14336 * 2 + 8192 * 14336 * 2 + 8192 * 3584 * 2 + 14336 * 3584
    assert f(1, 8192, 14336, 3584, 3) >= base9 + 16 * 16 * 256 * 256 * 4
    assert f(1, 8192, 14336, 3584, 3) < base9 + 16 * 16 * 256 * 256 * 4 + (8 << 20)
    assert f(1, 8192, 2048, 2048, 3) < 3 * 8192 * 2048 * 2 + 8192 * 2048 * 2 + 8192 * 2048 * 2 + 2048 * 2048 + (4 << 20)   # 64 tiles
    assert f(0, -1, N, K, 3) == 0 and f(1, M, N, K, 4) == 0 and f(1, M, N, K, 0) == 0
    # decode feed-forward stack (M = B, N = F, K = d): the gated product and two copies of the state
    assert f(2, 4, 14336, 4096, 1) >= 4 * (14336 + 2 * 4096) * 2
    assert f(2, 17, 14336, 4096, 1) == 0 and f(2, 0, 14336, 4096, 1) == 0


def test_slice_argument_checks(lib):
    assert lib.mq_slice(None, 4, 64, 9, 0, None, None, None) == BITS
    assert lib.mq_slice(None, 4, 64, 0, 0, None, None, None) == BITS
    assert lib.mq_slice(None, -1, 64, 4, 0, None, None, None) == SHAPE
    assert lib.mq_slice(None, 4, 64, 5, 2, None, None, None) == BITS       # packed 5-bit planes are not built
    assert lib.mq_slice(None, 4, 62, 6, 2, None, None, None) == ALIGN      # 372 bits per row
    assert lib.mq_slice(None, 4, 63, 2, 2, None, None, None) == ALIGN      # K not a whole number of bytes
    assert lib.mq_slice(None, 4, 64, 2, 1, None, None, None) == NULL       # extra precision without a list
    assert lib.mq_slice(None, 0, 64, 4, 0, None, None, None) == OK         # empty input: nothing to do
    assert lib.mq_slice(None, 4, 64, 4, 0, None, None, None) == NULL


def test_quantize_argument_checks(lib):
    assert lib.mq_quantize_int8(None, 4, 64, 64, None, None, None, None, None, None) == NULL
    assert lib.mq_quantize_int8(None, -4, 64, 64, None, None, None, None, None, None) == SHAPE
    assert lib.mq_quantize_int8(None, 4, 64, 32, None, None, None, None, None, None) == SHAPE   # ldw < K
    assert lib.mq_quantize_int8(None, 0, 64, 64, None, None, None, None, None, None) == OK


def test_linear_argument_checks(lib):
    ci = ctypes.c_int
    rs = (ci * 3)(8, 4, 2)
    dup = (ci * 2)(4, 4)
    bad = (ci * 1)(9)
    fwd, bwd = lib.mq_linear_fwd_multi, lib.mq_linear_bwd
    assert fwd(None, None, None, None, 16, 256, 256, rs, 4, 0, None, None, 0, None) == BITS
    assert fwd(None, None, None, None, 16, 256, 256, dup, 2, 0, None, None, 0, None) == BITS
    assert fwd(None, None, None, None, 16, 256, 256, bad, 1, 0, None, None, 0, None) == BITS
    assert fwd(None, None, None, None, 16, 256, 256, None, 3, 0, None, None, 0, None) == NULL
    assert fwd(None, None, None, None, -1, 256, 256, rs, 3, 0, None, None, 0, None) == SHAPE
    assert fwd(None, None, None, None, 16, 256, 250, rs, 3, 0, None, None, 0, None) == ALIGN
    assert bwd(None, None, None, None, None, None, 16, 256, 256, rs, 0, 0, None, None, None, 0, None) == BITS
    assert bwd(None, None, None, None, None, None, 16, 256, 250, rs, 3, 0, None, None, None, 0, None) == ALIGN
    assert bwd(None, None, None, None, None, None, 12, 250, 256, rs, 3, 0, None, None, None, 0, None) == ALIGN
    assert bwd(None, None, None, None, None, None, 13, 256, 256, rs, 3, 0, None, None, None, 0, None) == NULL     # any M: no dY
    assert bwd(None, None, None, None, None, None, 16, 256, 256, rs, 3, 0, None, None, None, 0, None) == NULL
    assert bwd(None, None, None, None, None, None, 0, 256, 256, rs, 3, 0, None, None, None, 0, None) == OK


def test_gemv_argument_checks(lib):
    g = lib.mq_gemv_sliced
    assert g(None, None, None, None, None, 1, 64, 256, 5, None, None) == BITS
    assert g(None, None, None, None, None, 1, 64, 200, 6, None, None) == ALIGN   # 1200 bits: not whole 12-byte units
    assert g(None, None, None, None, None, 17, 64, 256, 2, None, None) == SHAPE
    assert g(None, None, None, None, None, 0, 64, 256, 2, None, None) == SHAPE
    assert g(None, None, None, None, None, 1, 64, 100, 2, None, None) == ALIGN   # 200 bits per row
    assert g(None, None, None, None, None, 16, 64, 1 << 26, 2, None, None) == SHAPE  # B * K beyond 2^29
    assert g(None, None, None, None, None, 1, 0, 256, 2, None, None) == OK
    assert g(None, None, None, None, None, 1, 64, 256, 2, None, None) == NULL


def test_dense_extra_precision_argument_checks(lib):
    g = lib.mq_gemv_sliced_dense_ep
    assert g(None, None, None, None, 1, 64, 256, 4, None, None) == BITS     # 5 bits per code are not built
    assert g(None, None, None, None, 1, 64, 256, 8, None, None) == BITS
    assert g(None, None, None, None, 1, 64, 100, 2, None, None) == ALIGN    # 300 bits per row
    assert g(None, None, None, None, 1, 64, 256, 2, None, None) == NULL
    s = lib.mq_slice
    assert s(None, 4, 64, 2, 8, None, None, None) == BITS                   # dense needs packed + extra precision
    assert s(None, 4, 64, 4, 11, None, None, None) == BITS                  # 5 bits per code
    assert s(None, 4, 64, 2, 11, None, None, None) == NULL                  # fine up to the pointers (no list needed)


def test_probe_library_argument_checks():
    """The measurement-only library of bench.py loads, exports what its header declares and checks its arguments."""
    import re
    from paper_2502_06786_amd import build as mq_build
    hdr = open(os.path.join(mq_build.PROBE_DIR, "probes.h")).read()
    declared = set(re.findall(r"\b(mq_probe_\w+)\s*\(", hdr))
    plib = ctypes.CDLL(mq_build.PROBE_LIB)
    assert declared == {"mq_probe_mfma", "mq_probe_mfma16", "mq_probe_read"}
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    for name in declared:
        getattr(plib, name).argtypes = [vp, i64, vp, vp]
    assert plib.mq_probe_mfma(None, 10, None, None) == NULL
    assert plib.mq_probe_mfma16(None, 10, None, None) == NULL
    assert plib.mq_probe_read(None, 1024, None, None) == NULL


def test_ffn_mixnmatch_argument_checks(lib):
    f = lib.mq_ffn_mixnmatch

    class Layer(ctypes.Structure):
        _fields_ = [(n, ctypes.c_void_p) for n in ("gate_up", "down", "alpha_gu", "zero_gu", "alpha_dn", "zero_dn")] + \
                   [("r", ctypes.c_int)]

    bad_bits = (Layer * 1)(Layer(None, None, None, None, None, None, 5))
    nulls = (Layer * 1)(Layer(None, None, None, None, None, None, 4))
    x = ctypes.c_void_p(4096)    # never dereferenced: every call below returns before the first launch
    y = ctypes.c_void_p(8192)
    assert f(None, None, 1, 1, 256, 512, 0, None, None, 0, None) == NULL
    assert f(x, None, 1, 17, 256, 512, 0, y, None, 0, None) == SHAPE
    assert f(x, None, -1, 1, 256, 512, 0, y, None, 0, None) == SHAPE
    assert f(x, None, 1, 1, 256, 500, 0, y, None, 0, None) == ALIGN
    assert f(x, None, 1, 1, 256, 512, 0, y, None, 0, None) == NULL          # layers missing
    assert f(x, bad_bits, 1, 1, 256, 512, 0, y, None, 0, None) == BITS
    assert f(x, nulls, 1, 1, 256, 512, 0, y, None, 0, None) == NULL
    assert f(x, nulls, 1, 1, 256, 512, 0, x, None, 0, None) == SHAPE        # y aliases x
    # every layer is checked before the first launch: a second layer with a misaligned plane (first layer fine)
    # is refused with its own status, not with the launch error the first layer would meet without a GPU
    p = 1 << 20
    good = Layer(p, p, p, p, p, p, 4)
    odd_plane = Layer(p + 4, p, p, p, p, p, 4)
    two = (Layer * 2)(good, odd_plane)
    assert f(x, two, 2, 1, 256, 512, 0, y, None, 0, None) == ALIGN
    two = (Layer * 2)(good, Layer(p, p, p, p, p, p, 2))       # d = 96: 384 bits per row at int4, 192 at int2
    assert f(x, two, 2, 1, 96, 512, 0, y, None, 0, None) == ALIGN


def test_overflow_capacity_checks(lib):
    class Ovf(ctypes.Structure):
        _fields_ = [("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p), ("capacity", ctypes.c_int64),
                    ("nnz", ctypes.c_void_p)]

    p = 1 << 20
    neg = Ovf(p, p, -1, p)
    assert lib.mq_slice(p, 4, 64, 2, 1 | 2, p, ctypes.byref(neg), None) == CAPACITY
    assert lib.mq_gemv_sliced(p, p, p, p, ctypes.byref(neg), 1, 64, 256, 2, p, None) == CAPACITY


def test_l2_loss_argument_checks(lib):
    f = lib.mq_matquant_l2_loss
    ci = ctypes.c_int
    assert f(None, None, None, None, 16, 64, 4, 0, None, None, None, 0, None) == BITS      # at most three outputs
    assert f(None, None, None, None, 16, 64, 0, 0, None, None, None, 0, None) == BITS
    assert f(None, None, None, None, 3, 5, 3, 0, None, None, None, 0, None) == ALIGN       # 15 elements
    assert f(None, None, (ci * 3)(-1, 1, 0), None, 16, 64, 3, 0, None, None, None, 0, None) == SHAPE   # its own teacher
    assert f(None, None, (ci * 3)(-1, 3, 0), None, 16, 64, 3, 0, None, None, None, 0, None) == SHAPE
    assert f(None, None, None, None, 0, 64, 3, 0, None, None, None, 0, None) == OK
    assert f(None, None, None, None, 16, 64, 3, 0, None, None, None, 0, None) == NULL
    assert lib.mq_workspace_bytes(3, 4096, 9216, 0, 3) >= 4096 * 9216 // 8 // 512 * 16


def test_fwd_l2_argument_checks(lib):
    f = lib.mq_linear_fwd_multi_l2
    ci = ctypes.c_int
    rs = (ci * 3)(8, 4, 2)
    p = ctypes.c_void_p(4096)    # never dereferenced: every call below returns before the first launch
    assert f(p, p, p, p, 16, 64, 64, (ci * 2)(4, 4), 2, 0, None, p, None, None, None, None, None, None, 0, None) == BITS
    assert f(p, p, p, p, 16, 64, 40, rs, 3, 0, None, p, None, None, None, None, None, None, 0, None) == ALIGN
    assert f(p, p, p, p, 16, 64, 64, rs, 3, 0, None, p, (ci * 3)(-1, 1, 0), None, None, None, None, None, 0, None) == SHAPE
    assert f(p, p, p, p, 16, 64, 64, rs, 3, 0, None, p, (ci * 3)(-1, 0, 3), None, None, None, None, None, 0, None) == SHAPE
    assert f(p, p, p, p, 0, 64, 64, rs, 3, 0, None, None, None, None, None, None, None, None, 0, None) == OK
    assert f(p, p, p, p, 16, 64, 64, rs, 3, 0, None, p, None, None, None, None, None, None, 0, None) == NULL   # no dY
    # the partial sums of the objective sit behind the row sums of X
    assert lib.mq_workspace_bytes(4, 4096, 9216, 2304, 3) >= lib.mq_workspace_bytes(0, 4096, 9216, 2304, 3) + 32 * 72 * 16


def test_bwd_clip_argument_checks(lib):
    f = lib.mq_linear_bwd_clip
    ci = ctypes.c_int
    rs = (ci * 3)(8, 4, 2)
    p = ctypes.c_void_p(4096)    # never dereferenced: every call below returns before the first launch
    def call(M=16, N=64, K=64, ldw=64, rs_=rs, nr=3, W=p, dg=p):
        return f(W, ldw, p, p, p, p, None, None, None, None, M, N, K, rs_, nr, 0, dg, p, None, None, None, 0, None)
    assert call(nr=4) == BITS
    assert call(rs_=(ci * 2)(4, 4), nr=2) == BITS
    assert call(ldw=32) == SHAPE
    assert call(K=40, ldw=40) == ALIGN
    assert call(ldw=66) == ALIGN
    assert call(N=0) == OK
    assert call(W=None) == NULL
    assert call(dg=None) == NULL
    assert call() == NULL                                         # dY missing
    # the per-bit-width contraction goes into a scratch matrix next to the backward's own workspace
    assert lib.mq_workspace_bytes(5, 4096, 9216, 2304, 3) >= 9216 * 2304 * 4 + lib.mq_workspace_bytes(1, 4096, 9216, 2304, 1)


def test_affine_argument_checks(lib):
    p = ctypes.c_void_p(4096)    # never dereferenced: every call below returns before the first launch
    assert lib.mq_affine_weight(p, 8, 64, 32, None, None, None, p, p, None) == SHAPE        # ldw < K
    assert lib.mq_affine_weight(p, 8, 66, 66, None, None, None, p, p, None) == ALIGN
    assert lib.mq_affine_weight(p, 0, 64, 64, None, None, None, None, None, None) == OK
    assert lib.mq_affine_weight(p, 8, 64, 64, None, None, None, None, None, None) == NULL   # nothing to write
    assert lib.mq_affine_input(p, 4, 60, None, None, p, None) == ALIGN
    assert lib.mq_affine_input(p, 0, 64, None, None, p, None) == OK
    assert lib.mq_affine_input(None, 4, 64, None, None, p, None) == NULL
    f = lib.mq_affine_bwd
    assert f(p, p, p, 64, p, None, None, 4, 8, 16, 64, None, None, p, p, p, None, 0, None) == BITS
    assert f(p, p, p, 64, p, None, None, 3, 8, 18, 64, None, None, p, p, p, None, 0, None) == ALIGN
    assert f(p, p, p, 64, p, None, None, 3, 8, 16, 64, None, None, p, p, p, None, 0, None) == NULL   # dY missing
    assert lib.mq_workspace_bytes(6, 4096, 9216, 2304, 3) > 0


def test_gated_unit_argument_checks(lib):
    assert lib.mq_gated_unit_fwd(None, 4, 8, 64, 0, None, None) == BITS
    assert lib.mq_gated_unit_fwd(None, 3, 8, 60, 0, None, None) == ALIGN
    assert lib.mq_gated_unit_fwd(None, 3, 0, 64, 0, None, None) == OK
    assert lib.mq_gated_unit_fwd(None, 3, 8, 64, 0, None, None) == NULL
    assert lib.mq_gated_unit_bwd(None, None, 0, 8, 64, 0, None, None) == BITS
    assert lib.mq_gated_unit_bwd(None, None, 2, 8, 64, 0, None, None) == NULL



def test_noalloc_forward_argument_checks(lib):
    """The entry point without a workspace refuses bad arguments before it touches a device."""
    f = lib.mq_linear_fwd_multi_noalloc
    rs = (ctypes.c_int * 3)(8, 4, 2)
    assert f(None, None, None, None, (1 << 18) + 1, 256, 256, rs, 3, 0, None, None) == SHAPE   # beyond the built-in scratch
    assert f(None, None, None, None, 16, 256, 250, rs, 3, 0, None, None) == ALIGN
    assert f(None, None, None, None, 16, 256, 256, rs, 4, 0, None, None) == BITS
    assert f(None, None, None, None, 16, 256, 256, rs, 3, 0, None, None) == NULL
    assert f(None, None, None, None, 0, 256, 256, rs, 3, 0, None, None) == OK


def test_gated_backward_argument_checks(lib):
    f = lib.mq_linear_bwd_gated
    rs = (ctypes.c_int * 3)(8, 4, 2)
    assert f(None, None, None, None, None, None, None, 16, 128, 256, rs, 0, 0, None, None, None, 0, None) == BITS
    assert f(None, None, None, None, None, None, None, 16, 128, 250, rs, 3, 0, None, None, None, 0, None) == ALIGN
    assert f(None, None, None, None, None, None, None, 16, 60, 256, rs, 3, 0, None, None, None, 0, None) == ALIGN    # 2F = 120
    assert f(None, None, None, None, None, None, None, 16, -1, 256, rs, 3, 0, None, None, None, 0, None) == SHAPE
    assert f(None, None, None, None, None, None, None, 16, 128, 256, rs, 3, 0, None, None, None, 0, None) == NULL    # no GU, no dA
    assert f(None, None, None, None, None, None, None, 0, 128, 256, rs, 3, 0, None, None, None, 0, None) == OK


def test_gated_forward_argument_checks(lib):
    f = lib.mq_linear_fwd_multi_gated
    rs = (ctypes.c_int * 3)(8, 4, 2)
    assert f(None, None, None, None, 16, 128, 256, rs, 4, 0, None, None, None, 0, None) == BITS
    assert f(None, None, None, None, 16, 126, 256, rs, 3, 0, None, None, None, 0, None) == ALIGN   # F not a multiple of 4
    assert f(None, None, None, None, 16, 128, 250, rs, 3, 0, None, None, None, 0, None) == ALIGN
    assert f(None, None, None, None, 16, -4, 256, rs, 3, 0, None, None, None, 0, None) == SHAPE
    assert f(None, None, None, None, 16, 128, 256, rs, 3, 0, None, None, None, 0, None) == NULL    # X, Q, ... and A missing
    assert f(None, None, None, None, 0, 128, 256, rs, 3, 0, None, None, None, 0, None) == OK


def test_slice_multi_argument_checks(lib):
    f = lib.mq_slice_multi
    ci = ctypes.c_int
    assert f(None, 4, 64, (ci * 2)(4, 2), 0, 0, None, -1, None, None) == BITS
    assert f(None, 4, 64, (ci * 2)(4, 5), 2, 0, None, -1, None, None) == BITS       # no packed 5-bit planes
    assert f(None, 4, 64, (ci * 2)(4, 4), 2, 0, None, -1, None, None) == BITS       # duplicate
    assert f(None, 4, 62, (ci * 2)(4, 6), 2, 0, None, -1, None, None) == ALIGN      # 372 bits per row at r = 6
    assert f(None, 4, 64, (ci * 2)(4, 2), 2, 1, None, 5, None, None) == BITS        # overflow index outside rs
    assert f(None, 4, 64, (ci * 2)(4, 2), 2, 1, None, 1, None, None) == NULL        # extra precision without a list
    assert f(None, 4, 64, (ci * 2)(4, 2), 2, 8 | 1, None, 1, None, None) == BITS    # dense extra-precision plane: mq_slice
    assert f(None, 0, 64, (ci * 2)(4, 2), 2, 0, None, -1, None, None) == OK
    assert f(None, 4, 64, (ci * 2)(4, 2), 2, 0, None, -1, None, None) == NULL


def test_gemv_with_workspace_argument_checks(lib):
    f, wsb = lib.mq_gemv_sliced_ws, lib.mq_workspace_bytes
    # (MQ_OP_GEMV = 7: M = B, nr = bits per code) four floats per (group of four slices, row, batch column) where K is
    # split: 14336 int2 codes = 28 lines = 7 groups; at least 256 bytes otherwise
    assert wsb(7, 16, 4096, 14336, 2) >= 7 * 4096 * 16 * 4
    assert wsb(7, 16, 4096, 14336, 4) >= 7 * 4096 * 16 * 4
    assert wsb(7, 16, 4096, 14336, 8) == 256 and wsb(7, 16, 4096, 100, 2) == 256
    assert wsb(7, 17, 4096, 14336, 2) == 0 and wsb(7, 0, 4096, 14336, 2) == 0 and wsb(7, 4, 4096, 14336, 9) == 0
    p = ctypes.c_void_p(256)   # never dereferenced: every call below fails (or has nothing to do) on the host
    assert f(p, p, p, p, None, 16, 64, 14336, 9, p, p, 1 << 30, None) == BITS
    assert f(p, p, p, p, None, 16, 64, 14336, 2, p, None, 1 << 30, None) == WORKSPACE
    assert f(p, p, p, p, None, 16, 64, 14336, 2, p, p, wsb(7, 16, 64, 14336, 2) - 1, None) == WORKSPACE
    assert f(p, p, p, p, None, 16, 64, 14336, 2, p, ctypes.c_void_p(264), 1 << 30, None) == WORKSPACE   # not 16-byte aligned
    assert f(p, p, p, p, None, 16, 64, 100, 8, p, p, 255, None) == WORKSPACE
    assert f(p, p, p, p, None, 17, 64, 14336, 2, p, p, 1 << 30, None) == SHAPE
    assert f(p, p, p, p, None, 16, 64, 14330, 2, p, p, 1 << 30, None) == ALIGN
    assert f(None, p, p, p, None, 16, 64, 14336, 2, p, p, 1 << 30, None) == NULL
    assert f(p, p, p, p, None, 16, 0, 14336, 2, p, p, 1 << 30, None) == OK
