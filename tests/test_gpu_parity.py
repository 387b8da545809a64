"""HIP path vs CPU oracle through the C ABI, at sizes the oracle finishes in seconds.

Bars: bit-exact for codes, slices, packed bytes and overflow lists; rel-L2 <= 1e-2 against the
fp64 oracle for Y, dX, dW, y (expected ~2e-3 from the bf16 output rounding; dW is fp32 and only
sees the bf16 rounding of the summed gradient operand).
"""
import numpy as np
import pytest
import torch

from tests.util import accumulation_allowance, assert_close, bf16_bits, first_overflow_code, rel_l2

pytestmark = pytest.mark.gpu

TOL = 1e-2


@pytest.fixture(scope="module")
def mq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_06786_amd as mq_

    mq_.lib()
    return mq_


def dev(t):
    return t.to("cuda")


def _randn(seed, *shape, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, generator=g) * scale


# --------------------------------------------------------------------------
# quantize
# --------------------------------------------------------------------------
@pytest.mark.parametrize("N,K", [(256, 256), (7, 100), (5, 2304), (3, 9216), (2, 36864), (3, 4100), (9, 3),
                                 (1, 1), (130, 4608), (2, 70000)])
def test_quantize_bit_exact(mq, oracle, N, K):
    W = _randn(N * 1000 + K, N, K, scale=0.02)
    if N > 2:
        W[1] = 0.125            # constant row
        W[2, 0] = 3.0           # outlier
    Q, a, z = mq.mq_quantize_int8(dev(W))
    qo, ao, zo = oracle.quantize_int8(W.numpy())
    assert np.array_equal(a.cpu().numpy(), ao)
    assert np.array_equal(z.cpu().numpy(), zo)
    assert np.array_equal(Q.cpu().numpy(), qo)


def test_quantize_config1_and_stride_and_clip(mq, oracle):
    from paper_2502_06786_amd import synth
    W = synth.weight(1, "gate")
    Q, a, z = mq.mq_quantize_int8(dev(W))
    qo, ao, zo = oracle.quantize_int8(W.numpy())
    assert np.array_equal(Q.cpu().numpy(), qo) and np.array_equal(a.cpu().numpy(), ao)
    # row stride: a [N, K] view of a wider buffer
    big = dev(_randn(5, 40, 512, scale=0.02))
    view = big[:, :256]
    Q, a, z = mq.mq_quantize_int8(view)
    qo, ao, zo = oracle.quantize_int8(view.cpu().contiguous().numpy())
    assert np.array_equal(Q.cpu().numpy(), qo) and np.array_equal(z.cpu().numpy(), zo)
    # clip factors (section 3.1.2)
    g = torch.rand(40, generator=torch.Generator().manual_seed(1)) * 0.5 + 0.5
    b = torch.rand(40, generator=torch.Generator().manual_seed(2)) * 0.5 + 0.5
    Wc = big[:, 256:].contiguous()
    Q, a, z = mq.mq_quantize_int8(Wc, dev(g), dev(b))
    qo, ao, zo = oracle.quantize_int8(Wc.cpu().numpy(), g.numpy(), b.numpy())
    assert np.array_equal(Q.cpu().numpy(), qo) and np.array_equal(a.cpu().numpy(), ao)
    assert np.array_equal(z.cpu().numpy(), zo)


# --------------------------------------------------------------------------
# slice / pack / overflow list
# --------------------------------------------------------------------------
def test_slice_all_codes_all_r(mq, oracle):
    q = torch.arange(256, dtype=torch.int32).repeat(5).to(torch.uint8).reshape(5, 256)
    for r in range(1, 9):
        got = mq.mq_slice(dev(q), r).cpu().numpy()
        assert np.array_equal(got, oracle.slice_codes(q.numpy(), r)), r


@pytest.mark.parametrize("N,K", [(256, 256), (3, 40), (1, 8), (33, 1000), (257, 4104)])
def test_slice_packed_and_ragged(mq, oracle, N, K):
    g = torch.Generator().manual_seed(N + K)
    q = torch.randint(0, 256, (N, K), generator=g, dtype=torch.int32).to(torch.uint8)
    for r in (8, 6, 4, 3, 2):   # K is a multiple of 8 in every case: rows are whole bytes at every r
        got = mq.mq_slice(dev(q), r, packed=True).cpu().numpy()
        assert np.array_equal(got, oracle.pack(oracle.slice_codes(q.numpy(), r), r)), r
    for r in (3, 6):
        got = mq.mq_slice(dev(q), r).cpu().numpy()
        assert np.array_equal(got, oracle.slice_codes(q.numpy(), r)), r


@pytest.mark.parametrize("r", [2, 4, 3, 6, 8])
def test_slice_extra_precision_overflow_list(mq, oracle, r):
    g = torch.Generator().manual_seed(r)
    N, K = 70, 1000
    q = torch.randint(0, 256, (N, K), generator=g, dtype=torch.int32).to(torch.uint8)
    q[5] = 0          # empty row
    q[6] = 255        # full row
    packed = r in (8, 4, 2)
    out, ovf = mq.mq_slice(dev(q), r, packed=packed, extra_precision=True)
    torch.cuda.synchronize()
    codes = oracle.slice_codes(q.numpy(), r)
    want = oracle.pack(codes, r) if packed else codes
    assert np.array_equal(out.cpu().numpy(), want)          # dense plane == plain slice
    rp, ci = oracle.overflow_csr(q.numpy(), r)
    nnz = int(ovf.nnz.item())
    assert nnz == ci.size
    assert np.array_equal(ovf.row_ptr.cpu().numpy(), rp)
    assert np.array_equal(ovf.col_idx.cpu().numpy().view(np.uint16)[:nnz], ci)


@pytest.mark.parametrize("N,K,rs,ovf_r", [(257, 4112, (4, 2), 2), (33, 1008, (2,), 2), (100, 2048, (4, 2, 8), None), (64, 512, (6, 4), 6),
                                          (9, 1000, (4, 2), 4), (300, 1024, (3, 6, 2), 2), (5, 64, (4,), None)])
def test_slice_multi_matches_single_planes(mq, oracle, N, K, rs, ovf_r):
    """mq_slice_multi = one mq_slice per plane (bit for bit, planes and overflow list), against the oracle; rows that are
    whole 16-byte chunks take the single pass, K = 1000 the plane-by-plane route."""
    from paper_2502_06786_amd import synth
    q = synth.uniform_codes(N + K, N, K)
    if ovf_r is None:
        planes = mq.mq_slice_multi(dev(q), rs)
    else:
        planes, ovf = mq.mq_slice_multi(dev(q), rs, ovf_r=ovf_r)
        torch.cuda.synchronize()
        rp, ci = oracle.overflow_csr(q.numpy(), ovf_r)
        assert int(ovf.nnz.item()) == ci.size
        assert np.array_equal(ovf.row_ptr.cpu().numpy(), rp)
        assert np.array_equal(ovf.col_idx.cpu().numpy().view(np.uint16)[:ci.size], ci)
    for r, plane in zip(rs, planes):
        assert np.array_equal(plane.cpu().numpy(), oracle.pack(oracle.slice_codes(q.numpy(), r), r)), r


def test_slice_overflow_capacity(mq, oracle):
    g = torch.Generator().manual_seed(77)
    q = torch.randint(0, 256, (20, 512), generator=g, dtype=torch.int32).to(torch.uint8)
    rp, ci = oracle.overflow_csr(q.numpy(), 2)
    cap = ci.size // 2
    ovf = mq.Overflow(20, cap)
    ovf.col_idx = torch.full((cap + 64,), -1, dtype=torch.int16, device="cuda")  # guard region after capacity
    mq.mq_slice(dev(q), 2, extra_precision=True, ovf=ovf)
    torch.cuda.synchronize()
    assert int(ovf.nnz.item()) == ci.size > cap                  # the caller sees the shortfall
    got = ovf.col_idx.cpu().numpy().view(np.uint16)
    assert np.array_equal(got[:cap], ci[:cap])
    assert np.all(got[cap:] == 0xFFFF)                            # nothing written past capacity


# --------------------------------------------------------------------------
# fused multi-precision forward
# --------------------------------------------------------------------------
def _quantized(mq, oracle, W):
    Q, a, z = mq.mq_quantize_int8(dev(W))
    qo, ao, zo = oracle.quantize_int8(W.numpy())
    assert np.array_equal(Q.cpu().numpy(), qo)
    return Q, a, z, qo, ao, zo


FWD_SHAPES = [(16, 256, 256), (300, 264, 208), (1, 8, 16), (257, 136, 1040), (520, 392, 64)]
RS_SETS = [(8, 4, 2), (2,), (8,), (4, 2), (2, 8), (6, 3), (8, 6, 3), (7, 5, 1)]


@pytest.mark.parametrize("M,N,K", FWD_SHAPES)
def test_fwd_multi_shapes(mq, oracle, M, N, K):
    W = _randn(M + N + K, N, K, scale=0.02)
    X = _randn(M * 3 + 1, M, K).to(torch.bfloat16)
    Q, a, z, qo, ao, zo = _quantized(mq, oracle, W)
    for ep in (False, True):
        Ys = mq.mq_linear_fwd_multi(dev(X), Q, a, z, (8, 4, 2), extra_precision=ep)
        for r, Y in zip((8, 4, 2), Ys):
            want = oracle.linear_fwd(bf16_bits(X), qo, ao, zo, r, ep=ep)
            assert_close(Y.float().cpu().numpy(), want, what=(r, ep))


@pytest.mark.parametrize("rs", RS_SETS)
def test_fwd_multi_bit_width_sets(mq, oracle, rs):
    M, N, K = 200, 136, 336
    W = _randn(11, N, K, scale=0.02)
    W[:, 5] *= 6.0                                  # a heavy column so the top bucket is populated
    X = _randn(12, M, K).to(torch.bfloat16)
    Q, a, z, qo, ao, zo = _quantized(mq, oracle, W)
    for ep in (False, True):
        Ys = mq.mq_linear_fwd_multi(dev(X), Q, a, z, rs, extra_precision=ep)
        assert len(Ys) == len(rs)
        for r, Y in zip(rs, Ys):
            want = oracle.linear_fwd(bf16_bits(X), qo, ao, zo, r, ep=ep)
            assert_close(Y.float().cpu().numpy(), want, what=(rs, r, ep))


def test_fwd_uniform_codes_hit_every_bucket(mq, oracle):
    # codes uniform on 0..255 (all buckets incl. the clamped top one), alpha/z arbitrary
    from paper_2502_06786_amd import synth
    M, N, K = 64, 128, 512
    q = synth.uniform_codes(3, N, K)
    a = (torch.rand(N, generator=torch.Generator().manual_seed(4)) * 1e-3 + 1e-4)
    z = torch.rand(N, generator=torch.Generator().manual_seed(5)) * 255
    X = _randn(6, M, K).to(torch.bfloat16)
    for ep in (False, True):
        Ys = mq.mq_linear_fwd_multi(dev(X), dev(q), dev(a), dev(z), (8, 4, 2), extra_precision=ep)
        for r, Y in zip((8, 4, 2), Ys):
            want = oracle.linear_fwd(bf16_bits(X), q.numpy(), a.numpy(), z.numpy(), r, ep=ep)
            assert_close(Y.float().cpu().numpy(), want, what=(r, ep))


def test_fwd_exact_small_integers(mq, oracle):
    # alpha = 1, z = 0, X small integers: every product and sum is exact in fp32 and the outputs are
    # integers below 2^8 * ... representable in bf16 only if small, so compare before rounding matters:
    # one-hot X rows select single codes -> Y must equal the sliced value exactly.
    N, K = 64, 64
    q = torch.arange(N * K, dtype=torch.int32).remainder(256).to(torch.uint8).reshape(N, K)
    a = torch.ones(N)
    z = torch.zeros(N)
    X = torch.eye(K).to(torch.bfloat16)
    Ys = mq.mq_linear_fwd_multi(dev(X), dev(q), dev(a), dev(z), (8, 4, 2))
    for r, Y in zip((8, 4, 2), Ys):
        want = oracle.slice_values(q.numpy(), r).astype(np.float64).T     # Y[k, n] = S(q[n, k])
        assert np.array_equal(Y.float().cpu().numpy().astype(np.float64), want), r
    Ys = mq.mq_linear_fwd_multi(dev(X), dev(q), dev(a), dev(z), (4, 2), extra_precision=True)
    for r, Y in zip((4, 2), Ys):
        want = oracle.slice_values(q.numpy(), r, ep=True).astype(np.float64).T
        assert np.array_equal(Y.float().cpu().numpy().astype(np.float64), want), r


# --------------------------------------------------------------------------
# STE backward
# --------------------------------------------------------------------------
BWD_SHAPES = [(16, 256, 256), (264, 272, 208), (8, 16, 16), (520, 400, 320), (301, 272, 208), (1, 16, 16), (77, 48, 96)]


@pytest.mark.parametrize("M,N,K", BWD_SHAPES)
def test_bwd_shapes(mq, oracle, M, N, K):
    W = _randn(M + N + K + 1, N, K, scale=0.02)
    X = _randn(M * 5 + 1, M, K).to(torch.bfloat16)
    dYs = [_randn(100 + i, M, N, scale=1e-3).to(torch.bfloat16) for i in range(3)]
    lambdas = (0.1, 0.1, 1.0)
    rs = (8, 4, 2)
    Q, a, z, qo, ao, zo = _quantized(mq, oracle, W)
    for ep in (False, True):
        dX, dW = mq.mq_linear_bwd(dev(X), Q, a, z, [dev(d) for d in dYs], lambdas, rs, extra_precision=ep)
        want_dx = oracle.linear_bwd_dx(qo, ao, zo, [bf16_bits(d) for d in dYs], lambdas, rs, ep=ep)
        want_dw = oracle.linear_bwd_dw(bf16_bits(X), [bf16_bits(d) for d in dYs], lambdas)
        assert_close(dX.float().cpu().numpy(), want_dx, c_rms=2.0 ** -6, what=("dX", ep))
        assert_close(dW.cpu().numpy(), want_dw, c_rms=2.0 ** -6, what=("dW", ep))


@pytest.mark.parametrize("rs,lambdas", [((2,), None), ((8,), (0.5,)), ((4, 2), (0.4, 1.0)), ((6, 3), None),
                                        ((2, 8, 4), (1.0, 0.2, 0.2))])
def test_bwd_bit_width_sets_and_accumulate(mq, oracle, rs, lambdas):
    M, N, K = 136, 144, 176
    W = _randn(21, N, K, scale=0.02)
    X = _randn(22, M, K).to(torch.bfloat16)
    dYs = [_randn(200 + i, M, N, scale=1e-3).to(torch.bfloat16) for i in range(len(rs))]
    Q, a, z, qo, ao, zo = _quantized(mq, oracle, W)
    dX, dW = mq.mq_linear_bwd(dev(X), Q, a, z, [dev(d) for d in dYs], lambdas, rs)
    want_dx = oracle.linear_bwd_dx(qo, ao, zo, [bf16_bits(d) for d in dYs], lambdas, rs)
    want_dw = oracle.linear_bwd_dw(bf16_bits(X), [bf16_bits(d) for d in dYs], lambdas)
    assert_close(dX.float().cpu().numpy(), want_dx, c_rms=2.0 ** -6, what="dX")
    assert_close(dW.cpu().numpy(), want_dw, c_rms=2.0 ** -6, what="dW")
    # accumulate into an existing dW; skip dX
    base = dev(_randn(23, N, K, scale=1e-2))
    dW2 = base.clone()
    none, dW2 = mq.mq_linear_bwd(dev(X), Q, a, z, [dev(d) for d in dYs], lambdas, rs, need_dX=False, dW=dW2,
                                 accumulate_dW=True)
    assert none is None
    assert_close((dW2 - base).cpu().numpy(), want_dw, c_rms=2.0 ** -6, what="dW accumulated")
    # dX only
    dX3, none = mq.mq_linear_bwd(dev(X), Q, a, z, [dev(d) for d in dYs], lambdas, rs, need_dW=False)
    assert none is None and torch.equal(dX3, dX)


def test_bwd_dw_last_round_split_over_tokens(mq, oracle):
    """289 tiles of dW on 256 compute units: the 33 tiles of the last partial round are computed as four token ranges
    each and summed by a second kernel.  Ragged in all three sizes (the last tile row and column are 16 wide, the last
    token block holds 8 tokens), with and without accumulation; only dW is asked for."""
    M, N, K = 1000, 4112, 4112
    X = _randn(31, M, K).to(torch.bfloat16)
    dYs = [_randn(300 + i, M, N, scale=1e-3).to(torch.bfloat16) for i in range(2)]
    lambdas, rs = (0.5, 1.0), (4, 2)
    Q = dev(torch.zeros(N, K, dtype=torch.uint8))
    a = dev(torch.ones(N))
    z = dev(torch.zeros(N))
    none, dW = mq.mq_linear_bwd(dev(X), Q, a, z, [dev(d) for d in dYs], lambdas, rs, need_dX=False)
    assert none is None
    want_dw = oracle.linear_bwd_dw(bf16_bits(X), [bf16_bits(d) for d in dYs], lambdas)
    assert_close(dW.cpu().numpy(), want_dw, c_rms=2.0 ** -6, what="dW")
    base = dev(_randn(33, N, K, scale=1e-2))
    dW2 = base.clone()
    mq.mq_linear_bwd(dev(X), Q, a, z, [dev(d) for d in dYs], lambdas, rs, need_dX=False, dW=dW2, accumulate_dW=True)
    assert_close((dW2 - base).cpu().numpy(), want_dw, c_rms=2.0 ** -6, what="dW accumulated",
                 extra=2.0 ** -22 * np.abs(base.cpu().numpy()))      # (fp32 rounding of base + dW, then of the difference)


@pytest.mark.parametrize("rs", RS_SETS)
@pytest.mark.parametrize("ep", [False, True])
def test_bwd_exact_integers(mq, oracle, rs, ep):
    """alpha = 1, z = 0, lambda = 1 and gradients / activations that select single terms: every product and sum
    is an integer that fp32 and the outputs hold exactly, so the backward must equal the oracle bit for bit.
    dX: token m carries a one-hot gradient for bit-width m mod nr only, so dX[m, :] is one row of sliced values
    (0 .. 256).  dW: one-hot activations and small integer gradients, so dW[n, k] is a sum of a few integers.
    Several tiles in each dimension of both kernels (tokens, channels, features) with ragged ends."""
    M, N, K = 400, 272, 544
    nr = len(rs)
    q = ((torch.arange(N * K, dtype=torch.int64) * 37 + torch.arange(N * K, dtype=torch.int64) // K * 11) % 256)
    q = q.to(torch.uint8).reshape(N, K)
    a, z = torch.ones(N), torch.zeros(N)
    g = torch.Generator().manual_seed(1234 + nr)
    hot = torch.randint(0, N, (M,), generator=g)
    dYs = []
    for i in range(nr):
        d = torch.zeros(M, N)
        rows = torch.arange(i, M, nr)
        d[rows, hot[rows]] = 1.0
        dYs.append(d.to(torch.bfloat16))
    X = torch.zeros(M, K)
    X[torch.arange(M), (torch.arange(M) * 7 + 3) % K] = 1.0
    X = X.to(torch.bfloat16)
    dX, _ = mq.mq_linear_bwd(dev(X), dev(q), dev(a), dev(z), [dev(d) for d in dYs], None, rs, extra_precision=ep,
                             need_dW=False)
    want_dx = oracle.linear_bwd_dx(q.numpy(), a.numpy(), z.numpy(), [bf16_bits(d) for d in dYs], None, rs, ep=ep)
    sliced = [oracle.slice_values(q.numpy(), r, ep=ep).astype(np.float64) for r in rs]
    for m in (0, 1, 2, 161, M - 1):   # the oracle's rows are what the description says
        assert np.array_equal(want_dx[m], sliced[m % nr][int(hot[m])])
    assert np.array_equal(dX.float().cpu().numpy().astype(np.float64), want_dx), (rs, ep)
    # dW: integer gradients in -8 .. 8 per bit-width (their sum is exact in bf16), one-hot activations
    dYi = [torch.randint(-8, 9, (M, N), generator=g).to(torch.bfloat16) for _ in range(nr)]
    _, dW = mq.mq_linear_bwd(dev(X), dev(q), dev(a), dev(z), [dev(d) for d in dYi], None, rs, extra_precision=ep,
                             need_dX=False)
    want_dw = oracle.linear_bwd_dw(bf16_bits(X), [bf16_bits(d) for d in dYi], None)
    assert np.abs(want_dw).max() >= 8 and np.array_equal(want_dw, np.round(want_dw))
    assert np.array_equal(dW.cpu().numpy().astype(np.float64), want_dw), (rs, ep)


# --------------------------------------------------------------------------
# decode GEMV
# --------------------------------------------------------------------------
@pytest.mark.parametrize("N,K", [(256, 256), (100, 512), (16, 64), (1000, 1344), (4096, 4096), (40, 14336)])
@pytest.mark.parametrize("r", [2, 4, 8, 6, 3])
def test_gemv_plain(mq, oracle, N, K, r):
    W = _randn(N + K + r, N, K, scale=0.02)
    Q, a, z, qo, ao, zo = _quantized(mq, oracle, W)
    packed = mq.mq_slice(Q, r, packed=True)
    a16, z16 = a.to(torch.bfloat16), z.to(torch.bfloat16)
    for B in (1, 3, 4, 16):
        x = _randn(B * 7 + r, B, K).to(torch.bfloat16)
        y = mq.mq_gemv_sliced(dev(x), packed, a16, z16, r, K)
        want = oracle.gemv_sliced(bf16_bits(x), packed.cpu().numpy(), bf16_bits(a16), bf16_bits(z16), r, K)
        assert_close(y.float().cpu().numpy(), want, what=(B,))


@pytest.mark.parametrize("r,frac", [(2, 0.05), (4, 0.02), (2, 0.125), (6, 0.02), (3, 0.03)])
def test_gemv_extra_precision(mq, oracle, r, frac):
    from paper_2502_06786_amd import synth
    N, K = 300, 1024
    q = synth.uniform_codes(9, N, K) if frac == 0.125 else synth.planted_codes(9, N, K, first_overflow_code(r), frac)
    a = (torch.rand(N, generator=torch.Generator().manual_seed(4)) * 1e-3 + 1e-4).to(torch.bfloat16)
    z = (torch.rand(N, generator=torch.Generator().manual_seed(5)) * 255).to(torch.bfloat16)
    packed, ovf = mq.mq_slice(dev(q), r, packed=True, extra_precision=True)
    torch.cuda.synchronize()
    rp, ci = oracle.overflow_csr(q.numpy(), r)
    assert int(ovf.nnz.item()) == ci.size and abs(ci.size / q.numel() - frac) < 0.01
    for B in (1, 4, 16):
        x = _randn(B + r, B, K).to(torch.bfloat16)
        y = mq.mq_gemv_sliced(dev(x), packed, dev(a), dev(z), r, K, ovf=ovf)
        want = oracle.gemv_sliced(bf16_bits(x), packed.cpu().numpy(), bf16_bits(a), bf16_bits(z), r, K, ovf=(rp, ci))
        assert_close(y.float().cpu().numpy(), want, what=(B,))
        # (the overflow term itself, a few per cent of y, is pinned entry by entry in
        # test_gemv_extra_precision_one_hot_exact below)


def _all_codes_matrix(N, K):
    """Codes that run through 0 .. 255 along every row and every column (all buckets, the top one included)."""
    idx = torch.arange(N * K, dtype=torch.int64)
    return ((idx * 29 + (idx // K) * 5) % 256).to(torch.uint8).reshape(N, K)


@pytest.mark.parametrize("B", [1, 4, 16])
@pytest.mark.parametrize("r", [2, 3, 4, 6])
def test_gemv_extra_precision_one_hot_exact(mq, oracle, r, B):
    """alpha = 1, z = 0 and one-hot activations through the overflow LIST: y[b, n] is exactly the extra-precision
    value of code [n, k_b], i.e. one of the levels 0, 2^s, ..., 2^r 2^s of the errata section (256 included).
    Every column is visited (B = 16: all of them, 16 per launch; B = 1 and 4: a stride through them), so every
    entry of the list is pinned by an output that is wrong if the entry is dropped, read twice or misplaced."""
    N, K = 328, 512
    q = _all_codes_matrix(N, K)
    a, z = torch.ones(N).to(torch.bfloat16), torch.zeros(N).to(torch.bfloat16)
    packed, ovf = mq.mq_slice(dev(q), r, packed=True, extra_precision=True)
    torch.cuda.synchronize()
    rp, ci = oracle.overflow_csr(q.numpy(), r)
    assert int(ovf.nnz.item()) == ci.size > 0
    levels = oracle.slice_values(q.numpy(), r, ep=True).astype(np.float64)       # [N, K]
    assert levels.max() == 256.0 and set(np.unique(levels)) == set(float(v << (8 - r)) for v in range((1 << r) + 1))
    starts = range(0, K, B) if B == 16 else range(0, K, 37)
    for k0 in starts:
        cols = (k0 + torch.arange(B) * (1 if B == 16 else 5)) % K
        x = torch.zeros(B, K)
        x[torch.arange(B), cols] = 1.0
        y = mq.mq_gemv_sliced(dev(x.to(torch.bfloat16)), packed, dev(a), dev(z), r, K, ovf=ovf)
        want = levels[:, cols.numpy()].T
        assert np.array_equal(y.float().cpu().numpy().astype(np.float64), want), (r, B, k0)
    # the oracle's GEMV agrees with the level table on one of these inputs (it is the expected value elsewhere)
    chk = oracle.gemv_sliced(bf16_bits(x.to(torch.bfloat16)), packed.cpu().numpy(), bf16_bits(a), bf16_bits(z), r, K, ovf=(rp, ci))
    assert np.array_equal(chk, want)


@pytest.mark.parametrize("B", [1, 4, 16])
@pytest.mark.parametrize("r", [1, 2, 3, 5, 7])
def test_gemv_dense_extra_precision_one_hot_exact(mq, oracle, r, B):
    """The same pin for the dense extra-precision plane (r + 1 bits per code, code 2^r kept)."""
    N, K = 200, 768
    q = _all_codes_matrix(N, K)
    a, z = torch.ones(N).to(torch.bfloat16), torch.zeros(N).to(torch.bfloat16)
    dense = mq.mq_slice(dev(q), r, packed=True, extra_precision=True, dense_ep=True)
    levels = oracle.slice_values(q.numpy(), r, ep=True).astype(np.float64)
    assert levels.max() == 256.0
    for k0 in (range(0, K, 16) if B == 16 else range(0, K, 53)):
        cols = (k0 + torch.arange(B) * (1 if B == 16 else 7)) % K
        x = torch.zeros(B, K)
        x[torch.arange(B), cols] = 1.0
        y = mq.mq_gemv_sliced_dense_ep(dev(x.to(torch.bfloat16)), dense, dev(a), dev(z), r, K)
        assert np.array_equal(y.float().cpu().numpy().astype(np.float64), levels[:, cols.numpy()].T), (r, B, k0)


@pytest.mark.parametrize("B", [1, 16])
def test_gemv_truncated_overflow_list(mq, oracle, B):
    """A list that mq_slice had to cut short (capacity below the size of the set): row_ptr still describes the
    full set, and the GEMV uses exactly the entries that were stored - the result is the oracle's on the CSR
    clamped to the capacity, and nothing past col_idx is read (the guard region stays a poison pattern that
    would otherwise show up as columns beyond K)."""
    r, N, K = 2, 300, 1024
    from paper_2502_06786_amd import synth
    q = synth.planted_codes(77, N, K, first_overflow_code(r), 0.05)
    rp, ci = oracle.overflow_csr(q.numpy(), r)
    cap = int(ci.size) // 2 + 3
    ovf = mq.Overflow(N, cap, "cuda")
    ovf.col_idx = torch.full((cap + 4096,), -1, dtype=torch.int16, device="cuda")      # 0xFFFF behind the capacity
    packed, ovf = mq.mq_slice(dev(q), r, packed=True, extra_precision=True, ovf=ovf)
    torch.cuda.synchronize()
    assert int(ovf.nnz.item()) == ci.size > cap
    a = (torch.rand(N, generator=torch.Generator().manual_seed(4)) * 1e-3 + 1e-4).to(torch.bfloat16)
    z = (torch.rand(N, generator=torch.Generator().manual_seed(5)) * 255).to(torch.bfloat16)
    x = _randn(B + 50, B, K).to(torch.bfloat16)
    y = mq.mq_gemv_sliced(dev(x), packed, dev(a), dev(z), r, K, ovf=ovf)
    rp_cut = np.minimum(rp, cap).astype(rp.dtype)
    want = oracle.gemv_sliced(bf16_bits(x), packed.cpu().numpy(), bf16_bits(a), bf16_bits(z), r, K, ovf=(rp_cut, ci[:cap]))
    assert_close(y.float().cpu().numpy(), want, what="truncated list")
    full = oracle.gemv_sliced(bf16_bits(x), packed.cpu().numpy(), bf16_bits(a), bf16_bits(z), r, K, ovf=(rp, ci))
    assert rel_l2(want, full) > 5e-3        # the dropped half of the list matters at this density
    # exact version: alpha = 1, z = 0, one-hot activations on a column of the kept and of the dropped part
    ones, zeros = torch.ones(N).to(torch.bfloat16), torch.zeros(N).to(torch.bfloat16)
    for k in (int(ci[0]), int(ci[cap - 1]), int(ci[-1])):
        x1 = torch.zeros(B, K)
        x1[:, k] = 1.0
        y1 = mq.mq_gemv_sliced(dev(x1.to(torch.bfloat16)), packed, dev(ones), dev(zeros), r, K, ovf=ovf)
        w1 = oracle.gemv_sliced(bf16_bits(x1.to(torch.bfloat16)), packed.cpu().numpy(), bf16_bits(ones), bf16_bits(zeros), r, K,
                                ovf=(rp_cut, ci[:cap]))
        assert np.array_equal(y1.float().cpu().numpy().astype(np.float64), w1), k


@pytest.mark.parametrize("r", [2, 3, 5, 1, 7])
def test_dense_extra_precision_plane_and_gemv(mq, oracle, r):
    """One plane of r + 1 bits per code holding the unclamped extra-precision codes, and the GEMV that reads it."""
    from paper_2502_06786_amd import synth
    N, K = 200, 1536
    q = synth.uniform_codes(40 + r, N, K) if r != 2 else synth.planted_codes(41, N, K, first_overflow_code(2), 0.05)
    a = (torch.rand(N, generator=torch.Generator().manual_seed(8)) * 1e-3 + 1e-4).to(torch.bfloat16)
    z = (torch.rand(N, generator=torch.Generator().manual_seed(9)) * 255).to(torch.bfloat16)
    dense = mq.mq_slice(dev(q), r, packed=True, extra_precision=True, dense_ep=True)
    want_plane = oracle.pack(oracle.slice_codes(q.numpy(), r, ep=True), r + 1)
    assert np.array_equal(dense.cpu().numpy(), want_plane)
    rp, ci = oracle.overflow_csr(q.numpy(), r)
    plain = oracle.pack(oracle.slice_codes(q.numpy(), r), r) if r in (2, 3) else None
    for B in (1, 4, 16):
        x = _randn(B + r, B, K).to(torch.bfloat16)
        y = mq.mq_gemv_sliced_dense_ep(dev(x), dense, dev(a), dev(z), r, K)
        want = oracle.gemv_sliced(bf16_bits(x), want_plane, bf16_bits(a), bf16_bits(z), r + 1, K, shift=8 - r)
        assert_close(y.float().cpu().numpy(), want, what=(B,))
        if plain is not None:   # the same weights as clamped plane + list
            same = oracle.gemv_sliced(bf16_bits(x), plain, bf16_bits(a), bf16_bits(z), r, K, ovf=(rp, ci))
            assert np.array_equal(want, same)


@pytest.mark.parametrize("r,B", [(2, 1), (4, 3), (8, 16)])
def test_gemv_many_rows(mq, oracle, r, B):
    """More groups of row blocks than workgroups are resident at once (every workgroup walks over several
    groups), a row count that is not a multiple of 16, and a single 128-byte weight line per row."""
    from paper_2502_06786_amd import synth
    N, K = 66001 if B == 1 else 131075, 128 * 8 // r
    q = synth.uniform_codes(31 + r, N, K)
    a = (torch.rand(N, generator=torch.Generator().manual_seed(6)) * 1e-3 + 1e-4).to(torch.bfloat16)
    z = (torch.rand(N, generator=torch.Generator().manual_seed(7)) * 255).to(torch.bfloat16)
    packed = mq.mq_slice(dev(q), r, packed=True)
    x = _randn(B + r, B, K).to(torch.bfloat16)
    y = mq.mq_gemv_sliced(dev(x), packed, dev(a), dev(z), r, K)
    want = oracle.gemv_sliced(bf16_bits(x), packed.cpu().numpy(), bf16_bits(a), bf16_bits(z), r, K)
    assert_close(y.float().cpu().numpy(), want)
    # every row, not just the norm: a group that was skipped or written twice shows up here
    err = np.abs(y.float().cpu().numpy().astype(np.float64) - want)
    assert np.all(err <= 2.0 ** -7 * np.abs(want) + 1e-4 * np.abs(want).max())


@pytest.mark.parametrize("r,N,K,B", [(2, 16400, 4608, 1), (2, 16384, 1344, 3), (4, 17000, 4608, 4), (4, 16384, 14336, 1),
                                     (2, 16387, 14336, 2), (4, 16384, 544, 4)])
def test_gemv_small_batch_tall_matrix(mq, oracle, r, N, K, B):
    """At least 16384 rows and B <= 4 on int4 / int2 planes: the kernel that keeps the activations of a K slice
    in registers.  Shapes with one, several and padded 128-byte lines per slice, more slices than waves
    (several rounds per wave), a ragged last line, ragged row counts; checked row by row."""
    from paper_2502_06786_amd import synth
    q = synth.uniform_codes(50 + r + B, N, K)
    a = (torch.rand(N, generator=torch.Generator().manual_seed(16)) * 1e-3 + 1e-4).to(torch.bfloat16)
    z = (torch.rand(N, generator=torch.Generator().manual_seed(17)) * 255).to(torch.bfloat16)
    packed = mq.mq_slice(dev(q), r, packed=True)
    x = _randn(B + r + 3, B, K).to(torch.bfloat16)
    y = mq.mq_gemv_sliced(dev(x), packed, dev(a), dev(z), r, K)
    want = oracle.gemv_sliced(bf16_bits(x), packed.cpu().numpy(), bf16_bits(a), bf16_bits(z), r, K)
    got = y.float().cpu().numpy().astype(np.float64)
    assert_close(got, want)
    err = np.abs(got - want)
    assert np.all(err <= 2.0 ** -7 * np.abs(want) + 1e-3 * np.abs(want).max())


@pytest.mark.parametrize("r,N,K,B,with_list", [(2, 32775, 1024, 16, False), (4, 32808, 2048, 5, False), (2, 32768, 4608, 9, False),
                                               (4, 36864, 512, 16, False), (2, 32776, 1536, 8, True), (4, 32768, 1024, 13, True),
                                               (2, 32776, 8192, 5, False)])     # (16 slices: the plane runs in two rounds of workgroups)
def test_gemv_mid_batch_tall_matrix(mq, oracle, r, N, K, B, with_list):
    """At least 32768 rows and 5 <= B <= 16 on int4 / int2 planes: the kernel that keeps the activations of a K slice
    in registers as 16-column matrix-core operands.  One and several lines per slice, several slices per workgroup,
    ragged row counts, batch sizes that leave operand columns empty, and the overflow list on top; checked output
    by output."""
    from paper_2502_06786_amd import synth
    q = synth.planted_codes(60 + r + B, N, K, first_overflow_code(r), 0.03) if with_list else synth.uniform_codes(60 + r + B, N, K)
    a = (torch.rand(N, generator=torch.Generator().manual_seed(26)) * 1e-3 + 1e-4).to(torch.bfloat16)
    z = (torch.rand(N, generator=torch.Generator().manual_seed(27)) * 255).to(torch.bfloat16)
    x = _randn(B + r + 13, B, K).to(torch.bfloat16)
    if with_list:
        packed, ovf = mq.mq_slice(dev(q), r, packed=True, extra_precision=True)
        torch.cuda.synchronize()
        lists = oracle.overflow_csr(q.numpy(), r)
        assert int(ovf.nnz.item()) == lists[1].size > 0
    else:
        packed, ovf, lists = mq.mq_slice(dev(q), r, packed=True), None, None
    y = mq.mq_gemv_sliced(dev(x), packed, dev(a), dev(z), r, K, ovf=ovf)
    want = oracle.gemv_sliced(bf16_bits(x), packed.cpu().numpy(), bf16_bits(a), bf16_bits(z), r, K, ovf=lists)
    assert_close(y.float().cpu().numpy(), want, what=(r, N, K, B, with_list))


def test_gemv_mid_batch_tall_matrix_one_hot_exact(mq, oracle):
    # alpha = 1, z = 0, one-hot activations: y[b, n] is exactly the sliced value of code [n, k_b] (tall matrix, 5 <= B <= 16)
    N, K = 32790, 1024
    q = torch.arange(N * K, dtype=torch.int64).mul(7).add(torch.arange(N * K, dtype=torch.int64) // K).remainder(256)
    q = q.to(torch.uint8).reshape(N, K)
    a = torch.ones(N).to(torch.bfloat16)
    z = torch.zeros(N).to(torch.bfloat16)
    for r in (2, 4):
        packed = mq.mq_slice(dev(q), r, packed=True)
        sliced = oracle.slice_values(q.numpy(), r)
        for B, k0 in ((16, 0), (16, 500), (11, 1008), (5, 37)):
            cols = (k0 + torch.arange(B) * 3) % K
            x = torch.zeros(B, K)
            x[torch.arange(B), cols] = 1.0
            y = mq.mq_gemv_sliced(dev(x.to(torch.bfloat16)), packed, dev(a), dev(z), r, K)
            want = sliced[:, cols.numpy()].T.astype(np.float64)
            assert np.array_equal(y.float().cpu().numpy().astype(np.float64), want), (r, B, k0)


def test_gemv_small_batch_tall_matrix_one_hot_exact(mq, oracle):
    # alpha = 1, z = 0, one-hot activations: y[b, n] is exactly the sliced value of code [n, k_b] (tall matrix, B <= 4)
    N, K = 16400, 1024
    q = torch.arange(N * K, dtype=torch.int64).mul(7).add(torch.arange(N * K, dtype=torch.int64) // K).remainder(256)
    q = q.to(torch.uint8).reshape(N, K)
    a = torch.ones(N).to(torch.bfloat16)
    z = torch.zeros(N).to(torch.bfloat16)
    for r in (2, 4):
        packed = mq.mq_slice(dev(q), r, packed=True)
        for k0 in (0, 17, 511, 1020):
            x = torch.zeros(4, K)
            x[torch.arange(4), k0 + torch.arange(4)] = 1.0
            y = mq.mq_gemv_sliced(dev(x.to(torch.bfloat16)), packed, dev(a), dev(z), r, K)
            want = oracle.slice_values(q.numpy(), r)[:, k0:k0 + 4].T.astype(np.float64)
            assert np.array_equal(y.float().cpu().numpy().astype(np.float64), want), (r, k0)


@pytest.mark.parametrize("r,N,K,B,with_list", [(2, 150, 7168, 16, False), (4, 150, 7168, 5, False), (4, 64, 6912, 9, False),
                                               (2, 8192, 6656, 8, False), (2, 200, 14336, 16, True), (4, 40, 36864, 13, True),
                                               (2, 100, 4096, 16, False), (8, 100, 7168, 16, False), (2, 100, 7168, 3, False)])
def test_gemv_with_workspace_split_k(mq, oracle, r, N, K, B, with_list):
    """mq_gemv_sliced_ws: long rows and few of them at 5 <= B <= 16 on int4 / int2 planes run with K split over
    workgroups (groups of four slices, the last group partial; one and two lines per slice; ragged row blocks; the
    overflow sums added by the reducing kernel), other shapes as mq_gemv_sliced does; all against the oracle, output
    by output."""
    from paper_2502_06786_amd import synth
    q = synth.planted_codes(80 + r + B, N, K, first_overflow_code(r), 0.03) if with_list else synth.uniform_codes(80 + r + B, N, K)
    a = (torch.rand(N, generator=torch.Generator().manual_seed(28)) * 1e-3 + 1e-4).to(torch.bfloat16)
    z = (torch.rand(N, generator=torch.Generator().manual_seed(29)) * 255).to(torch.bfloat16)
    x = _randn(B + r + 17, B, K).to(torch.bfloat16)
    if with_list:
        packed, ovf = mq.mq_slice(dev(q), r, packed=True, extra_precision=True)
        torch.cuda.synchronize()
        lists = oracle.overflow_csr(q.numpy(), r)
        assert int(ovf.nnz.item()) == lists[1].size > 0
    else:
        packed, ovf, lists = mq.mq_slice(dev(q), r, packed=True), None, None
    y = mq.mq_gemv_sliced_ws(dev(x), packed, dev(a), dev(z), r, K, ovf=ovf)
    want = oracle.gemv_sliced(bf16_bits(x), packed.cpu().numpy(), bf16_bits(a), bf16_bits(z), r, K, ovf=lists)
    assert_close(y.float().cpu().numpy(), want, what=(r, N, K, B, with_list),
                 extra=accumulation_allowance(K, 1.0, a.double().numpy() * float(1 << (8 - r)))[None, :])


def test_gemv_with_workspace_one_hot_exact(mq, oracle):
    # alpha = 1, z = 0, one-hot activations: y[b, n] is exactly the sliced value of code [n, k_b], through the split form
    N, K = 72, 7168
    q = torch.arange(N * K, dtype=torch.int64).mul(7).add(torch.arange(N * K, dtype=torch.int64) // K).remainder(256)
    q = q.to(torch.uint8).reshape(N, K)
    a = torch.ones(N).to(torch.bfloat16)
    z = torch.zeros(N).to(torch.bfloat16)
    for r in (2, 4):
        packed = mq.mq_slice(dev(q), r, packed=True)
        sliced = oracle.slice_values(q.numpy(), r)
        for B, k0 in ((16, 0), (16, 5000), (11, 7150), (5, 37)):
            cols = (k0 + torch.arange(B) * 449) % K     # the batch entries fall into different slices and groups
            x = torch.zeros(B, K)
            x[torch.arange(B), cols] = 1.0
            y = mq.mq_gemv_sliced_ws(dev(x.to(torch.bfloat16)), packed, dev(a), dev(z), r, K)
            want = sliced[:, cols.numpy()].T.astype(np.float64)
            assert np.array_equal(y.float().cpu().numpy().astype(np.float64), want), (r, B, k0)


def test_gemv_one_hot_exact(mq, oracle):
    # alpha = 1, z = 0, one-hot activations: y[b, n] is exactly the sliced value of code [n, b].
    N, K = 64, 256
    q = torch.arange(N * K, dtype=torch.int32).mul(7).remainder(256).to(torch.uint8).reshape(N, K)
    a = torch.ones(N).to(torch.bfloat16)
    z = torch.zeros(N).to(torch.bfloat16)
    for r in (2, 4, 8, 6, 3):
        packed = mq.mq_slice(dev(q), r, packed=True)
        for k0 in (0, 100, 240):
            x = torch.zeros(16, K)
            x[torch.arange(16), k0 + torch.arange(16)] = 1.0
            y = mq.mq_gemv_sliced(dev(x.to(torch.bfloat16)), packed, dev(a), dev(z), r, K)
            want = oracle.slice_values(q.numpy(), r)[:, k0:k0 + 16].T.astype(np.float64)
            assert np.array_equal(y.float().cpu().numpy().astype(np.float64), want), (r, k0)


# --------------------------------------------------------------------------
# layer-wise Mix'n'Match feed-forward stack (decode path)
# --------------------------------------------------------------------------
def _ffn_stack(mq, oracle, seed, d, F, rs, scale):
    """Layers quantized by the library from seeded fp32 weights; planes and bf16 parameters on the GPU."""
    layers, host = [], []
    for i, r in enumerate(rs):
        w_gu = _randn(seed + 10 * i, 2 * F, d, scale=scale / d ** 0.5)
        w_dn = _randn(seed + 10 * i + 1, d, F, scale=scale / F ** 0.5)
        L = {"r": r}
        for name, w in (("gu", w_gu), ("dn", w_dn)):
            Q, a, z = mq.mq_quantize_int8(dev(w))
            a16, z16 = mq.mq_params_to_bf16(a, z)
            L["gate_up" if name == "gu" else "down"] = mq.mq_slice(Q, r, packed=True)
            L["alpha_" + name], L["zero_" + name] = a16, z16
        layers.append(L)
        host.append({k: (v if k == "r" else (bf16_bits(v) if v.dtype == torch.bfloat16 else v.cpu().numpy()))
                     for k, v in L.items()})
    return layers, host


def _ffn_layer_by_layer(mq, oracle, layers, host, x, d, F, silu, residual):
    """Parity of the stack at a bar that does not depend on its depth: every layer is run on the ORACLE's input of
    that layer (the bf16 state the oracle's own chain reached) and compared with the oracle's output of that layer.
    What remains is one layer's arithmetic: two GEMVs and the bf16 roundings of g, u, a, o, where a value that the fp32
    and the fp64 evaluation round to different neighbours moves what follows by a bf16 step (measured on 7B-shaped
    layers: rel-L2 1e-3 at int2, 4e-4 at int4, 4 to 15 % of the outputs on the neighbouring bf16 number)."""
    h = bf16_bits(x)
    for l, (L, H) in enumerate(zip(layers, host)):
        nxt, _ = oracle.ffn_mixnmatch(h, [H], d, F, silu=silu, residual=residual)
        h_dev = torch.from_numpy(h.view(np.int16).copy()).view(torch.bfloat16).reshape(h.shape).cuda()
        y = mq.mq_ffn_mixnmatch(h_dev, [L], F, silu=silu, residual=residual)
        want = oracle.bf16_to_f64(nxt)
        # (with the residual the output is rounded twice, bf16(h + bf16(o)): a second bf16 step of the value is allowed)
        assert_close(y.float().cpu().numpy(), want, c_rms=2.0 ** -6, what=("layer", l, L["r"]), extra=2.0 ** -7 * np.abs(want))
        h = nxt


@pytest.mark.parametrize("d,F,rs,B,silu,residual", [
    (256, 512, (2, 8, 4), 1, False, False), (256, 512, (2, 8, 4), 4, True, False), (256, 512, (3, 6, 2, 4), 16, False, True),
    (512, 1536, (4,), 3, False, False), (128, 256, (), 2, False, False),
    (128, 7168, (2, 4), 16, False, True), (128, 6912, (4, 2), 6, True, False)])   # (down product: K split over workgroups)
def test_ffn_mixnmatch_small(mq, oracle, d, F, rs, B, silu, residual):
    layers, host = _ffn_stack(mq, oracle, 70, d, F, rs, scale=1.5)
    x = _randn(77 + B, B, d).to(torch.bfloat16)
    y = mq.mq_ffn_mixnmatch(dev(x), layers, F, silu=silu, residual=residual)
    want_bits, _ = oracle.ffn_mixnmatch(bf16_bits(x), host, d, F, silu=silu, residual=residual)
    want = oracle.bf16_to_f64(want_bits)
    assert np.isfinite(want).all() and np.abs(want).max() > 1e-3
    _ffn_layer_by_layer(mq, oracle, layers, host, x, d, F, silu, residual)
    # End to end the two sides drift apart with the depth: a layer adds its own rounding differences (about 1e-3, see
    # _ffn_layer_by_layer) and passes on what it received multiplied by the sensitivity of the layer itself, which for
    # these random gated layers (nearly quadratic in their input) is 1.5 to 2.  The layer-by-layer check above is the
    # parity bar; this one only bounds the drift of the whole stack.
    assert rel_l2(y.float().cpu().numpy(), want) <= TOL * max(len(rs), 1)


@pytest.mark.parametrize("B,silu,residual", [(1, True, False), (3, False, True)])
def test_ffn_mixnmatch_7b_shaped_pyramid(mq, oracle, B, silu, residual):
    """Mistral-7B-shaped layers (d 4096, F 14336), int2 - int4 - int2: the gate/up plane has 28672 rows (the
    tall-matrix kernel at int2 / int4 with the gate activation in its epilogue), B = 1 and 3."""
    d, F, rs = 4096, 14336, (2, 4, 2)
    layers, host = _ffn_stack(mq, oracle, 90, d, F, rs, scale=1.5)
    x = _randn(91, B, d).to(torch.bfloat16)
    y = mq.mq_ffn_mixnmatch(dev(x), layers, F, silu=silu, residual=residual)
    want_bits, _ = oracle.ffn_mixnmatch(bf16_bits(x), host, d, F, silu=silu, residual=residual)
    want = oracle.bf16_to_f64(want_bits)
    assert np.abs(want).max() > 1e-3
    _ffn_layer_by_layer(mq, oracle, layers, host, x, d, F, silu, residual)
    assert rel_l2(y.float().cpu().numpy(), want) <= TOL * len(rs)     # (drift of the whole stack: see test_ffn_mixnmatch_small)


def test_ffn_layer_pairs_gate_and_up_rows(mq, oracle):
    """One layer whose gate rows are the only non-constant ones: with gate row f next to up row f the
    output must follow the oracle, which reads the plane as (gate, up) pairs; the order inside a pair
    and the pairing itself would both show (GELU is not symmetric in its two factors)."""
    d, F, r = 256, 512, 8
    w_gu = _randn(5, 2 * F, d, scale=0.1)
    w_gu[1::2] = w_gu[1::2].abs() + 0.05          # up rows: positive weights
    w_dn = torch.eye(d, F) + _randn(6, d, F, scale=0.01)
    L = {"r": r}
    for name, w in (("gu", w_gu), ("dn", w_dn)):
        Q, a, z = mq.mq_quantize_int8(dev(w))
        L["alpha_" + name], L["zero_" + name] = mq.mq_params_to_bf16(a, z)
        L["gate_up" if name == "gu" else "down"] = mq.mq_slice(Q, r, packed=True)
    host = {k: (v if k == "r" else (bf16_bits(v) if v.dtype == torch.bfloat16 else v.cpu().numpy())) for k, v in L.items()}
    x = _randn(7, 2, d).abs().to(torch.bfloat16)
    y = mq.mq_ffn_mixnmatch(dev(x), [L], F)
    want = oracle.bf16_to_f64(oracle.ffn_mixnmatch(bf16_bits(x), [host], d, F)[0])
    assert_close(y.float().cpu().numpy(), want, c_rms=2.0 ** -6)


# --------------------------------------------------------------------------
# L2 reconstruction objective over the bit-widths (the step between forward and backward)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("M,N,nr,teacher,mix", [(16, 256, 3, None, False), (520, 1000, 3, (-1, 0, 0), False),
                                                (4096, 2304, 3, (-1, -1, 0), True), (33, 24, 2, (1, -1), False),
                                                (8, 8, 1, None, False), (0, 64, 3, None, False)])
def test_l2_loss(mq, oracle, M, N, nr, teacher, mix):
    lam = (0.1, 0.4, 1.0)[:nr]
    Ys = [(_randn(200 + i, M, N) * (1.0 + 0.1 * i)).to(torch.bfloat16) for i in range(nr)]
    T = _randn(210, M, N).to(torch.bfloat16)
    losses, dYs = mq.mq_matquant_l2_loss([dev(y) for y in Ys], dev(T), teacher, lam, mix)
    torch.cuda.synchronize()
    if M * N == 0:
        return
    want_l, want_d = oracle.matquant_l2_loss([bf16_bits(y) for y in Ys], bf16_bits(T), teacher, lam, mix)
    assert np.allclose(losses.cpu().numpy(), want_l, rtol=1e-4)         # fp32 sums of M N squares
    for i in range(nr):
        assert rel_l2(dYs[i].float().cpu().numpy(), want_d[i]) <= TOL    # one bf16 rounding: 2^-9 / sqrt(3)


FUSED_L2_CASES = [
    # M, N, K, rs, teacher, mix, ep
    (300, 264, 208, (8, 4, 2), None, False, False),
    (300, 264, 208, (8, 4, 2), (-1, 0, 0), False, True),
    (257, 136, 1040, (8, 4, 2), (-1, 0, 1), True, False),
    (16, 256, 256, (2, 8), (1, -1), False, False),      # r = 8 not first: the kernel's slot order differs
    (200, 136, 336, (4, 8, 2), (1, -1, 0), True, True),
    (200, 136, 336, (4, 2), None, False, False),
    (1, 8, 16, (2,), None, False, False),
    (520, 392, 64, (6, 3), (-1, 0), False, False),
    (72, 200, 96, (8, 4), (1, 0), False, False),        # every bit-width has a teacher: no target is read
    (96, 72, 80, (8, 4, 2), None, True, False),         # the mix flag without any teacher changes nothing
]


@pytest.mark.parametrize("M,N,K,rs,teacher,mix,ep", FUSED_L2_CASES)
def test_fwd_with_fused_l2_objective(mq, oracle, M, N, K, rs, teacher, mix, ep):
    # The target is the output of the unquantized layer plus noise of the size of the output, so that
    # Y_i - T is far above one bf16 step of Y_i: where the fp32 and the fp64 accumulation round a Y_i to
    # different neighbours (about one element in a thousand), dY_i moves by 2^-8 of it only.
    nr = len(rs)
    lam = (0.1, 0.4, 1.0)[:nr]
    W = _randn(M + N + K + 7, N, K, scale=0.02)
    X = _randn(M * 3 + 2, M, K).to(torch.bfloat16)
    Q, a, z, qo, ao, zo = _quantized(mq, oracle, W)
    clean = X.float() @ W.t()
    T = (clean + _randn(99, M, N) * clean.std()).to(torch.bfloat16)
    if not mix and teacher is not None and min(teacher) >= 0:
        T = None
    Yg = [torch.empty(M, N, dtype=torch.bfloat16, device="cuda") if i != 1 else None for i in range(nr)]
    losses, dYs = mq.mq_linear_fwd_multi_l2(dev(X), Q, a, z, rs, (dev(T) if T is not None else None), teacher, lam, mix, extra_precision=ep, Y=Yg)
    torch.cuda.synchronize()
    want_Y = [oracle.linear_fwd(bf16_bits(X), qo, ao, zo, r, ep=ep) for r in rs]
    want_l, want_d = oracle.matquant_l2_loss([oracle.bf16_round(y) for y in want_Y], (bf16_bits(T) if T is not None else None), teacher, lam, mix)
    assert np.allclose(losses.cpu().numpy(), want_l, rtol=1e-3)
    for i in range(nr):
        # dY_i = coef_i (Y_i - T_i): a bf16 step of Y_i, or of the output that serves as its teacher, moves it by
        # coef_i times that step, however small the difference itself is
        coef = lam[i] * 2.0 / (M * N)
        th = teacher[i] if teacher is not None else -1
        step = np.abs(want_Y[i]) + (np.abs(want_Y[th]) if th >= 0 else 0.0)
        assert_close(dYs[i].float().cpu().numpy(), want_d[i], c_rms=2.0 ** -6, what=(rs[i], "dY"), extra=coef * 2.0 ** -7 * step)
        if Yg[i] is not None:
            assert_close(Yg[i].float().cpu().numpy(), want_Y[i], what=(rs[i], "Y"))
    # the same arithmetic as the two calls in sequence: identical gradients, sums in another order
    Ys2 = mq.mq_linear_fwd_multi(dev(X), Q, a, z, rs, extra_precision=ep)
    l2, d2 = mq.mq_matquant_l2_loss(Ys2, (dev(T) if T is not None else None), teacher, lam, mix)
    torch.cuda.synchronize()
    for i in range(nr):
        assert torch.equal(dYs[i], d2[i]), rs[i]
        if Yg[i] is not None:
            assert torch.equal(Yg[i], Ys2[i]), rs[i]
    assert np.allclose(losses.cpu().numpy(), l2.cpu().numpy(), rtol=1e-5)
    # without any Y output
    l3, d3 = mq.mq_linear_fwd_multi_l2(dev(X), Q, a, z, rs, (dev(T) if T is not None else None), teacher, lam, mix, extra_precision=ep)
    torch.cuda.synchronize()
    assert torch.equal(l3, losses) and all(torch.equal(u, v) for u, v in zip(d3, dYs))


# --------------------------------------------------------------------------
# gradients with respect to the clip factors of the quantizer
# --------------------------------------------------------------------------
@pytest.mark.parametrize("M,N,K,rs,clip,ep", [(64, 48, 96, (8, 4, 2), True, False), (67, 48, 96, (8, 4, 2), True, False), (264, 272, 208, (8, 4, 2), True, True),
                                              (520, 400, 1040, (4, 2), False, False), (8, 16, 4112, (2,), True, False),
                                              (0, 32, 64, (8, 4, 2), False, False)])
def test_bwd_clip_factor_grads(mq, oracle, M, N, K, rs, clip, ep):
    nr = len(rs)
    lam = (0.3, 0.5, 1.0)[:nr]
    W = _randn(M + N + K + 3, N, K, scale=0.02)
    W[1] = 0.125                                  # constant row: no gradient unless gamma != beta
    W[2, 5] = 0.3                                 # outlier: the other weights of the row sit in few codes
    X = _randn(M * 7 + 1, M, K).to(torch.bfloat16)
    dYs = [(_randn(300 + i, M, N) * 1e-2).to(torch.bfloat16) for i in range(nr)]
    g = torch.rand(N, generator=torch.Generator().manual_seed(1)) * 0.4 + 0.5 if clip else None
    b = torch.rand(N, generator=torch.Generator().manual_seed(2)) * 0.4 + 0.5 if clip else None
    Wd = dev(W)
    Q, a, z = mq.mq_quantize_int8(Wd, dev(g) if clip else None, dev(b) if clip else None)
    qo, ao, zo = oracle.quantize_int8(W.numpy(), g.numpy() if clip else None, b.numpy() if clip else None)
    assert np.array_equal(Q.cpu().numpy(), qo)
    got = mq.mq_linear_bwd_clip(Wd, dev(X), Q, a, z, [dev(d) for d in dYs], lam, rs, dev(g) if clip else None,
                                dev(b) if clip else None, extra_precision=ep, want_dalpha_dzero=True)
    torch.cuda.synchronize()
    if M == 0:
        assert all(float(t.abs().max()) == 0.0 for t in got)
        return
    want = oracle.clip_factor_grads(W.numpy(), bf16_bits(X), [bf16_bits(d) for d in dYs], lam, rs,
                                    g.numpy() if clip else None, b.numpy() if clip else None, ep=ep)
    for name, mine, ref in zip(("dgamma", "dbeta", "dalpha", "dzero"), got, want):
        mine = mine.cpu().numpy().astype(np.float64)
        if np.abs(ref).max() == 0.0:              # e.g. d z without any clamp acting
            assert np.abs(mine).max() == 0.0, name
        else:
            assert rel_l2(mine, ref) <= TOL, (name, rel_l2(mine, ref))
    if not clip:                                  # (with gamma != beta the constant row has a range of its own)
        assert got[0][1].item() == 0.0 and got[1][1].item() == 0.0 and want[0][1] == 0.0


# --------------------------------------------------------------------------
# learnable affine re-parameterisation of a projection
# --------------------------------------------------------------------------
def _affine_case(seed, M, N, K):
    g = torch.Generator().manual_seed(seed)
    W = torch.randn(N, K, generator=g) * 0.02
    X = torch.randn(M, K, generator=g).to(torch.bfloat16)
    s = torch.rand(K, generator=g) * 1.5 + 0.5
    delta = torch.randn(K, generator=g) * 0.1
    b = torch.randn(N, generator=g) * 0.05
    return W, X, s, delta, b


@pytest.mark.parametrize("M,N,K", [(50, 48, 96), (520, 400, 1040), (1, 4, 8), (3, 7, 4100)])
def test_affine_weight_and_input(mq, oracle, M, N, K):
    W, X, s, delta, b = _affine_case(M + N + K, M, N, K)
    if K % 8 == 0:
        Xt = mq.mq_affine_input(dev(X), dev(s), dev(delta))
        want = oracle.affine_input(bf16_bits(X), s.numpy(), delta.numpy())
        got = bf16_bits(Xt.cpu())
        assert np.mean(got != want) <= 2e-3          # fp32 then bf16 against fp64 then bf16: rare double roundings
        assert rel_l2(Xt.float().cpu().numpy(), oracle.bf16_to_f64(want)) <= 1e-3
        assert torch.equal(mq.mq_affine_input(dev(X)), dev(X))
    Ws, c = mq.mq_affine_weight(dev(W), dev(s), dev(delta), dev(b))
    want_Ws, want_c = oracle.affine_weight(W.numpy(), s.numpy(), delta.numpy(), b.numpy())
    assert np.array_equal(Ws.cpu().numpy(), want_Ws)                     # the quantizer's input: bit for bit
    assert rel_l2(c.cpu().numpy().astype(np.float64), want_c) <= 1e-5    # fp32 products, fp64 across the workgroup
    wide = dev(torch.cat([W, W], dim=1))[:, :K]                          # a row stride
    Ws2, c2 = mq.mq_affine_weight(wide, dev(s), None, None)
    assert torch.equal(Ws2, Ws) and float(c2.abs().max()) == 0.0


@pytest.mark.parametrize("M,N,K", [(72, 48, 96), (264, 272, 208)])
def test_affine_layer_forward(mq, oracle, M, N, K):
    # the whole transformed layer: quantize W * s, forward on (X - delta) / s with the bias b + W delta
    rs = (8, 4, 2)
    W, X, s, delta, b = _affine_case(M * 3 + N, M, N, K)
    Ws, c = mq.mq_affine_weight(dev(W), dev(s), dev(delta), dev(b))
    Xt = mq.mq_affine_input(dev(X), dev(s), dev(delta))
    Q, a, z = mq.mq_quantize_int8(Ws)
    Ws_o, c_o = oracle.affine_weight(W.numpy(), s.numpy(), delta.numpy(), b.numpy())
    Xt_o = oracle.affine_input(bf16_bits(X), s.numpy(), delta.numpy())
    qo, ao, zo = oracle.quantize_int8(Ws_o)
    assert np.array_equal(Q.cpu().numpy(), qo)
    Y = [torch.empty(M, N, dtype=torch.bfloat16, device="cuda") for _ in rs]
    T = torch.zeros(M, N, dtype=torch.bfloat16, device="cuda")
    mq.mq_linear_fwd_multi_l2(Xt, Q, a, z, rs, T, Y=Y, bias=c)
    torch.cuda.synchronize()
    for r, y in zip(rs, Y):
        want = oracle.linear_fwd(Xt_o, qo, ao, zo, r) + c_o[None, :]
        assert_close(y.float().cpu().numpy(), want, what=r)
    # at 8 bits the transformed layer reproduces X W^T + b up to the quantization error
    plain = X.double().numpy() @ W.double().numpy().T + b.double().numpy()[None, :]
    assert rel_l2(Y[0].float().cpu().numpy(), plain) <= 3e-2


@pytest.mark.parametrize("M,N,K,nr", [(72, 48, 96, 3), (520, 400, 1040, 2), (5, 4, 8, 1), (4096, 256, 512, 3)])
def test_affine_bwd(mq, oracle, M, N, K, nr):
    W, X, s, delta, _ = _affine_case(M + 2 * N + K, M, N, K)
    lam = (0.2, 0.7, 1.0)[:nr]
    dXt = (_randn(41, M, K) * 1e-2).to(torch.bfloat16)
    dWs = _randn(42, N, K) * 1e-2
    dYs = [(_randn(43 + i, M, N) * 1e-2).to(torch.bfloat16) for i in range(nr)]
    dd, ds, dc = mq.mq_affine_bwd(dev(X), dev(dXt), dev(W), dev(dWs), [dev(d) for d in dYs], lam, dev(s), dev(delta))
    torch.cuda.synchronize()
    want = oracle.affine_bwd(bf16_bits(X), bf16_bits(dXt), W.numpy(), dWs.numpy(), [bf16_bits(d) for d in dYs], lam,
                             s.numpy(), delta.numpy())
    for name, mine, ref in zip(("ddelta", "ds", "dc"), (dd, ds, dc), want):
        assert rel_l2(mine.cpu().numpy().astype(np.float64), ref) <= 1e-4, name   # fp32 partial sums, fp64 across them


# --------------------------------------------------------------------------
# feed-forward block on the training path
# --------------------------------------------------------------------------
@pytest.mark.parametrize("M,F,nr,silu", [(40, 64, 3, False), (257, 1000, 2, True), (1, 8, 1, False), (0, 64, 3, False)])
def test_gated_unit_fwd_bwd(mq, oracle, M, F, nr, silu):
    GU = [(_randn(60 + i, M, 2 * F) * 2.0).to(torch.bfloat16) for i in range(nr)]
    dA = [_randn(70 + i, M, F).to(torch.bfloat16) for i in range(nr)]
    A = mq.mq_gated_unit_fwd([dev(t) for t in GU], silu)
    dGU = mq.mq_gated_unit_bwd([dev(t) for t in GU], [dev(t) for t in dA], silu)
    torch.cuda.synchronize()
    if M == 0:
        return
    for i in range(nr):
        want = oracle.bf16_to_f64(oracle.gated_unit(bf16_bits(GU[i]), silu))
        assert rel_l2(A[i].float().cpu().numpy(), want) <= 3e-3, i         # one bf16 rounding
        want = oracle.gated_unit_bwd(bf16_bits(GU[i]), bf16_bits(dA[i]), silu)
        assert rel_l2(dGU[i].float().cpu().numpy(), want) <= 3e-3, i


def test_ffn_block_training_step_composes(mq, oracle):
    """Forward and straight-through backward of a whole gated feed-forward block for r = 8, 4, 2 out of the
    library's calls (stacked gate/up layer -> gate -> one down layer per bit-width, and back), against the same
    composition of the oracle's functions."""
    M, d, F, rs, lam = 72, 96, 64, (8, 4, 2), (0.3, 0.6, 1.0)
    Wgu, Wd = _randn(1, 2 * F, d, scale=1.0 / d ** 0.5), _randn(2, d, F, scale=1.0 / F ** 0.5)
    X = _randn(3, M, d).to(torch.bfloat16)
    dYs = [(_randn(4 + i, M, d) * 1e-2).to(torch.bfloat16) for i in range(3)]
    Qg, ag, zg, qg, aog, zog = _quantized(mq, oracle, Wgu)
    Qd, ad, zd, qd, aod, zod = _quantized(mq, oracle, Wd)
    xb = bf16_bits(X)
    # ---- library
    GU = mq.mq_linear_fwd_multi(dev(X), Qg, ag, zg, rs)
    A = mq.mq_gated_unit_fwd(GU)
    Y = [mq.mq_linear_fwd_multi(A[i], Qd, ad, zd, (r,))[0] for i, r in enumerate(rs)]
    dA, dWd = [], torch.zeros(d, F, device="cuda")
    for i, r in enumerate(rs):
        dx, _ = mq.mq_linear_bwd(A[i], Qd, ad, zd, [dev(dYs[i])], (lam[i],), (r,), dW=dWd, accumulate_dW=True)
        dA.append(dx)
    dGU = mq.mq_gated_unit_bwd(GU, dA)
    dX, dWgu = mq.mq_linear_bwd(dev(X), Qg, ag, zg, dGU, None, rs)
    # the same two steps in one call: the gradients of the gated unit are formed inside the backward's first pass
    dX1, dWgu1 = mq.mq_linear_bwd_gated(dev(X), Qg, ag, zg, GU, dA, None, rs)
    torch.cuda.synchronize()
    assert torch.equal(dX1, dX) and torch.equal(dWgu1, dWgu)
    # ---- oracle
    ones = (1.0,) * 3
    GU_o = [oracle.bf16_round(oracle.linear_fwd(xb, qg, aog, zog, r)) for r in rs]
    A_o = [oracle.gated_unit(g) for g in GU_o]
    dA_o, dWd_o, dGU_o = [], np.zeros((d, F)), []
    for i, r in enumerate(rs):
        want = oracle.linear_fwd(A_o[i], qd, aod, zod, r)
        assert rel_l2(Y[i].float().cpu().numpy(), want) <= 2 * TOL, ("Y", r)
        dyb = bf16_bits(dYs[i])
        dA_o.append(oracle.bf16_round(oracle.linear_bwd_dx(qd, aod, zod, [dyb], (lam[i],), (r,))))
        dWd_o += oracle.linear_bwd_dw(A_o[i], [dyb], (lam[i],))
        dGU_o.append(oracle.bf16_round(oracle.gated_unit_bwd(GU_o[i], dA_o[i])))
    assert rel_l2(dWd.cpu().numpy().astype(np.float64), dWd_o) <= 2 * TOL
    assert rel_l2(dX.float().cpu().numpy(), oracle.linear_bwd_dx(qg, aog, zog, dGU_o, ones, rs)) <= 2 * TOL
    assert rel_l2(dWgu.cpu().numpy().astype(np.float64), oracle.linear_bwd_dw(xb, dGU_o, ones)) <= 2 * TOL


@pytest.mark.parametrize("M,F,K,rs,silu,ep", [(72, 64, 96, (8, 4, 2), False, False), (301, 136, 208, (4, 2), True, False),
                                              (520, 200, 320, (8, 6, 3), False, True), (1, 8, 16, (2,), True, False)])
def test_gated_backward_matches_the_two_calls_and_the_oracle(mq, oracle, M, F, K, rs, silu, ep):
    """mq_linear_bwd_gated = mq_gated_unit_bwd followed by mq_linear_bwd on the stacked gate / up layer: bit-identical to
    the two calls (lambda weights, accumulation into dW, dX only, dW only), and within the backward's bars of the oracle's
    composition of the same two steps."""
    nr = len(rs)
    lam = (0.25, 0.5, 1.0)[:nr]
    W = _randn(M + F + K, 2 * F, K, scale=1.0 / K ** 0.5)
    X = _randn(M + 1, M, K).to(torch.bfloat16)
    Q, a, z, qo, ao, zo = _quantized(mq, oracle, W)
    GU = mq.mq_linear_fwd_multi(dev(X), Q, a, z, rs, extra_precision=ep)
    # forward: the gated unit in the epilogue of the stacked layer = the two calls in sequence, bit for bit
    A0 = mq.mq_gated_unit_fwd(GU, silu=silu)
    GU1, A1 = mq.mq_linear_fwd_multi_gated(dev(X), Q, a, z, rs, silu=silu, extra_precision=ep)
    _, A2 = mq.mq_linear_fwd_multi_gated(dev(X), Q, a, z, rs, silu=silu, extra_precision=ep, store_GU=False)
    dA_host = [(_randn(40 + i, M, F) * 1e-2).to(torch.bfloat16) for i in range(nr)]
    dA = [dev(t) for t in dA_host]
    dGU = mq.mq_gated_unit_bwd(GU, dA, silu=silu)
    dX0, dW0 = mq.mq_linear_bwd(dev(X), Q, a, z, dGU, lam, rs, extra_precision=ep)
    dX1, dW1 = mq.mq_linear_bwd_gated(dev(X), Q, a, z, GU, dA, lam, rs, silu=silu, extra_precision=ep)
    assert torch.equal(dX1, dX0) and torch.equal(dW1, dW0)
    base = dev(_randn(41, 2 * F, K, scale=1e-2))
    acc0, acc1 = base.clone(), base.clone()
    mq.mq_linear_bwd(dev(X), Q, a, z, dGU, lam, rs, extra_precision=ep, need_dX=False, dW=acc0, accumulate_dW=True)
    none, _ = mq.mq_linear_bwd_gated(dev(X), Q, a, z, GU, dA, lam, rs, silu=silu, extra_precision=ep, need_dX=False, dW=acc1,
                                     accumulate_dW=True)
    assert none is None and torch.equal(acc0, acc1)
    dX2, none = mq.mq_linear_bwd_gated(dev(X), Q, a, z, GU, dA, lam, rs, silu=silu, extra_precision=ep, need_dW=False)
    assert none is None and torch.equal(dX2, dX0)
    # against the oracle's own chain (forward, rounding to bf16, gate, gate backward, linear backward): a GU that the
    # two sides round to different bf16 neighbours moves the gated values by one more step, hence the wider bars
    GU_o = [oracle.bf16_round(oracle.linear_fwd(bf16_bits(X), qo, ao, zo, r, ep=ep)) for r in rs]
    dGU_o = []
    for i in range(nr):
        assert torch.equal(GU1[i], GU[i]) and torch.equal(A1[i], A0[i]) and torch.equal(A2[i], A0[i]), rs[i]
        assert_close(GU1[i].float().cpu().numpy(), oracle.bf16_to_f64(GU_o[i]), what=("GU", rs[i]))
        assert_close(A1[i].float().cpu().numpy(), oracle.bf16_to_f64(oracle.gated_unit(GU_o[i], silu=silu)), c_rms=2.0 ** -5,
                     tol=2 * TOL, what=("A", rs[i]))
        dGU_o.append(oracle.bf16_round(oracle.gated_unit_bwd(GU_o[i], bf16_bits(dA_host[i]), silu=silu)))
    assert_close(dX1.float().cpu().numpy(), oracle.linear_bwd_dx(qo, ao, zo, dGU_o, lam, rs, ep=ep), c_rms=2.0 ** -5, tol=2 * TOL, what="dX")
    assert_close(dW1.cpu().numpy(), oracle.linear_bwd_dw(bf16_bits(X), dGU_o, lam), c_rms=2.0 ** -5, tol=2 * TOL, what="dW")

# --------------------------------------------------------------------------
# the whole step under HIP graph capture
# --------------------------------------------------------------------------
def test_step_replays_from_a_hip_graph(mq):
    """The library allocates nothing, never synchronises and records no memset: a whole step (quantize, slice with
    overflow list, forward with the objective, backward, clip-factor gradients, decode GEMV) is captured once and
    replayed on new inputs; every replay must reproduce the eager results bit for bit."""
    M, N, K, rs, lam = 136, 144, 256, (8, 4, 2), (0.2, 0.5, 1.0)
    W = dev(_randn(1, N, K, scale=0.02))
    X = dev(_randn(2, M, K).to(torch.bfloat16))
    T = dev(_randn(3, M, N).to(torch.bfloat16))
    xd = dev(_randn(4, 4, K).to(torch.bfloat16))
    u8 = dict(dtype=torch.uint8, device="cuda")
    Q, a, z = torch.empty(N, K, **u8), torch.empty(N, device="cuda"), torch.empty(N, device="cuda")
    a16, z16 = torch.empty(N, dtype=torch.bfloat16, device="cuda"), torch.empty(N, dtype=torch.bfloat16, device="cuda")
    p2 = torch.empty(N, K // 4, **u8)
    ovf = mq.Overflow(N, N * K // 4)
    dY = [torch.empty(M, N, dtype=torch.bfloat16, device="cuda") for _ in rs]
    losses = torch.empty(3, device="cuda")
    dX, dW = torch.empty(M, K, dtype=torch.bfloat16, device="cuda"), torch.empty(N, K, device="cuda")
    y = torch.empty(4, N, dtype=torch.bfloat16, device="cuda")
    ws_f = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_FWD_L2, M, N, K, 3), **u8)
    ws_b = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_BWD, M, N, K, 3), **u8)
    ws_c = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_BWD_CLIP, M, N, K, 3), **u8)
    def step():
        mq.mq_quantize_int8(W, Q=Q, alpha=a, zero=z)
        mq.mq_slice(Q, 2, packed=True, extra_precision=True, out=p2, ovf=ovf)
        mq.mq_params_to_bf16(a, z, a16, z16)
        mq.mq_linear_fwd_multi_l2(X, Q, a, z, rs, T, (-1, 0, 0), lam, dY=dY, losses=losses, ws=ws_f)
        mq.mq_linear_bwd(X, Q, a, z, dY, None, rs, dX=dX, dW=dW, ws=ws_b)
        grads = mq.mq_linear_bwd_clip(W, X, Q, a, z, dY, None, rs, ws=ws_c)     # (allocates its two outputs)
        mq.mq_gemv_sliced(xd, p2, a16, z16, 2, K, y=y, ovf=ovf)
        return list(grads)

    fixed = (Q, a, z, p2, ovf.row_ptr, losses, dX, dW, y, *dY)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream (kernel attributes are set here)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            captured = step()                    # the tensors the replays write their clip-factor gradients to
    for trial in range(3):
        W.copy_(dev(_randn(10 + trial, N, K, scale=0.02)))
        X.copy_(dev(_randn(20 + trial, M, K).to(torch.bfloat16)))
        torch.cuda.synchronize()
        eager = step()                           # eager, default stream
        torch.cuda.synchronize()
        want = [t.clone() for t in (*fixed, *eager)]
        for t in (Q, p2, losses, dX, dW, y, *dY, *captured):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (*fixed, *captured)]
        for i, (g_, w_) in enumerate(zip(got, want)):
            assert torch.equal(g_, w_), (trial, i)


def test_later_entry_points_replay_from_a_hip_graph(mq):
    """The same for the calls added later: mq_slice_multi, the forward with the gate in its epilogue, the backward with
    the gate gradient in its first pass (dW with a split last round needs no clearing between calls), the GEMV with a
    workspace in its K-split form and a Mix'n'Match stack at B = 16 whose down products run K-split.  Captured once,
    replayed on new inputs, compared bit for bit with eager calls."""
    M, F, K, rs, lam = 136, 72, 256, (8, 4, 2), (0.2, 0.5, 1.0)
    N = 2 * F
    u8 = dict(dtype=torch.uint8, device="cuda")
    bf = dict(dtype=torch.bfloat16, device="cuda")
    W = dev(_randn(1, N, K, scale=0.05))
    X = dev(_randn(2, M, K).to(torch.bfloat16))
    dA = [dev(_randn(30 + i, M, F, scale=1e-2).to(torch.bfloat16)) for i in range(3)]
    Q, a, z = torch.empty(N, K, **u8), torch.empty(N, device="cuda"), torch.empty(N, device="cuda")
    planes = [torch.empty(N, K // 2, **u8), torch.empty(N, K // 4, **u8)]
    ovf = mq.Overflow(N, N * K // 4)
    GU = [torch.empty(M, N, **bf) for _ in rs]
    A = [torch.empty(M, F, **bf) for _ in rs]
    dX, dW = torch.empty(M, K, **bf), torch.empty(N, K, device="cuda")
    ws_f = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_FWD, M, N, K, 3), **u8)
    ws_b = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_BWD, M, N, K, 3), **u8)
    # decode side: a long-row plane (K-split GEMV) and a two-layer stack with F = 7168
    Bd, Nd, Kd = 16, 96, 7168
    qd = dev(torch.randint(0, 256, (Nd, Kd), dtype=torch.int32, generator=torch.Generator().manual_seed(5)).to(torch.uint8))
    pd = mq.mq_slice(qd, 2, packed=True)
    ad = dev((torch.rand(Nd, generator=torch.Generator().manual_seed(6)) * 1e-3 + 1e-4).to(torch.bfloat16))
    zd = dev((torch.rand(Nd, generator=torch.Generator().manual_seed(7)) * 255).to(torch.bfloat16))
    xd = dev(_randn(8, Bd, Kd).to(torch.bfloat16))
    yd = torch.empty(Bd, Nd, **bf)
    ws_g = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_GEMV, Bd, Nd, Kd, 2), **u8)
    assert ws_g.numel() > 256                       # (the split form is what runs)
    d_, F_ = 128, 7168
    layers, _ = _ffn_stack(mq, None, 40, d_, F_, (2, 4), scale=1.5)
    xs = dev(_randn(9, Bd, d_).to(torch.bfloat16))
    ys = torch.empty(Bd, d_, **bf)
    ws_s = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_FFN_DECODE, Bd, F_, d_, 1), **u8)

    def step():
        mq.mq_quantize_int8(W, Q=Q, alpha=a, zero=z)
        mq.mq_slice_multi(Q, (4, 2), out=planes, ovf_r=2, ovf=ovf)
        mq.mq_linear_fwd_multi_gated(X, Q, a, z, rs, GU=GU, A=A, ws=ws_f)
        mq.mq_linear_bwd_gated(X, Q, a, z, GU, dA, lam, rs, dX=dX, dW=dW, ws=ws_b)
        mq.mq_gemv_sliced_ws(xd, pd, ad, zd, 2, Kd, y=yd, ws=ws_g)
        mq.mq_ffn_mixnmatch(xs, layers, F_, residual=True, y=ys, ws=ws_s)

    outs = (Q, *planes, ovf.row_ptr, *GU, *A, dX, dW, yd, ys)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    for trial in range(3):
        W.copy_(dev(_randn(50 + trial, N, K, scale=0.05)))
        X.copy_(dev(_randn(60 + trial, M, K).to(torch.bfloat16)))
        xd.copy_(dev(_randn(70 + trial, Bd, Kd).to(torch.bfloat16)))
        xs.copy_(dev(_randn(80 + trial, Bd, d_).to(torch.bfloat16)))
        torch.cuda.synchronize()
        step()
        torch.cuda.synchronize()
        want = [t.clone() for t in outs]
        for t in outs:
            t.zero_()
        ws_g.zero_(), ws_s.zero_(), ws_b.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (g_, w_) in enumerate(zip(outs, want)):
            assert torch.equal(g_, w_), (trial, i)


# --------------------------------------------------------------------------
# the calls as a training loop
# --------------------------------------------------------------------------
def test_cotraining_loop_reduces_every_loss(mq):
    """Quantization-aware training of one linear layer towards a teacher layer with the MatQuant objective
    (section 3.2): quantize -> forward for r = 8, 4, 2 with the L2 objective -> straight-through backward ->
    SGD on the fp32 master weights.  Signs and scales of the gradients are right if all three losses fall;
    the int2 loss cannot reach zero (four levels per row) but must fall well below its starting value."""
    M, N, K, rs, lam = 512, 64, 128, (8, 4, 2), (1.0, 1.0, 1.0)
    g = torch.Generator().manual_seed(0)
    W_teacher = torch.randn(N, K, generator=g) * 0.05
    W = (W_teacher + torch.randn(N, K, generator=g) * 0.05).cuda()       # start away from the teacher
    X = torch.randn(M, K, generator=g).to(torch.bfloat16).cuda()
    T = (X.float() @ W_teacher.cuda().t()).to(torch.bfloat16)
    first = last = None
    lr = 0.1 * N                                     # curvature of the summed mean losses: about 6 / N per weight
    for step in range(60):
        Q, a, z = mq.mq_quantize_int8(W)
        losses, dY = mq.mq_linear_fwd_multi_l2(X, Q, a, z, rs, T, None, lam)
        _, dW = mq.mq_linear_bwd(X, Q, a, z, dY, None, rs, need_dX=False)
        W -= lr * dW
        if step == 0:
            first = losses.cpu().numpy().copy()
        last = losses.cpu().numpy().copy()
    assert np.all(np.isfinite(last))
    assert last[0] < 0.05 * first[0] and last[1] < 0.1 * first[1] and last[2] < 0.7 * first[2], (first, last)


def test_clip_factor_calibration_reduces_the_int2_loss(mq):
    """OmniQuant-style calibration (section 3.1.2) with the library's calls: the weights stay fixed, the clip
    factors gamma, beta follow the sign of their gradients.  On heavy-tailed rows, clipping the range trades a
    few saturated outliers for finer steps everywhere else, so the int2 reconstruction loss must fall."""
    M, N, K, rs, lam = 512, 64, 256, (8, 4, 2), (0.1, 0.1, 1.0)
    g = torch.Generator().manual_seed(3)
    num, den = torch.randn(N, K, generator=g), torch.randn(N, K, 3, generator=g)
    W = (num / den.pow(2).mean(dim=2).sqrt() * 0.02).cuda()              # Student-t, 3 degrees of freedom
    X = torch.randn(M, K, generator=g).to(torch.bfloat16).cuda()
    T = (X.float() @ W.t()).to(torch.bfloat16)
    gamma, beta = torch.ones(N, device="cuda"), torch.ones(N, device="cuda")
    first = last = None
    for step in range(40):
        Q, a, z = mq.mq_quantize_int8(W, gamma, beta)
        losses, dY = mq.mq_linear_fwd_multi_l2(X, Q, a, z, rs, T, None, lam)
        dg, db = mq.mq_linear_bwd_clip(W, X, Q, a, z, dY, None, rs, gamma, beta)
        gamma = (gamma - 0.01 * torch.sign(dg)).clamp(0.3, 1.0)
        beta = (beta - 0.01 * torch.sign(db)).clamp(0.3, 1.0)
        if step == 0:
            first = losses.cpu().numpy().copy()
        last = losses.cpu().numpy().copy()
    assert np.all(np.isfinite(last))
    assert last[2] < 0.9 * first[2], (first, last)
    assert float(gamma.mean()) < 0.99 and float(beta.mean()) < 0.99      # the range was clipped


def test_measurement_probes_run():
    from paper_2502_06786_amd import bench_probes as mq
    ops = torch.randn(32768, generator=torch.Generator().manual_seed(3)).to(torch.bfloat16).cuda()
    sink = torch.zeros(65536, dtype=torch.float32, device="cuda")
    flops = mq.mq_probe_mfma(ops, 8, sink)
    assert flops == 256 * 4 * 8 * 12 * 32768
    torch.cuda.synchronize()
    assert torch.isfinite(sink).all() and sink.abs().sum() > 0
    sink16 = torch.zeros(131072, dtype=torch.float32, device="cuda")
    assert mq.mq_probe_mfma16(ops, 8, sink16) == 256 * 8 * 8 * 24 * 16384
    torch.cuda.synchronize()
    assert torch.isfinite(sink16).all() and sink16.abs().sum() > 0
    src = torch.arange(1 << 20, dtype=torch.int32).to(torch.uint8).cuda()
    assert mq.mq_probe_read(src) == src.numel()
    torch.cuda.synchronize()


# --------------------------------------------------------------------------
# argument checking (host side, nothing is launched)
# --------------------------------------------------------------------------
def test_error_codes(mq):
    Q = torch.zeros(8, 64, dtype=torch.uint8, device="cuda")
    with pytest.raises(mq.MqError) as e:
        mq.mq_slice(Q, 9)
    assert e.value.status == 3
    with pytest.raises(mq.MqError) as e:
        mq.mq_slice(Q, 5, packed=True)
    assert e.value.status == 3
    X = torch.zeros(4, 64, dtype=torch.bfloat16, device="cuda")
    a = torch.ones(8, device="cuda")
    with pytest.raises(mq.MqError) as e:
        mq.mq_linear_fwd_multi(X, Q, a, a, (8, 8))
    assert e.value.status == 3
    with pytest.raises(mq.MqError) as e:
        mq.mq_linear_fwd_multi(X, Q, a, a, (8, 4, 2), ws=torch.zeros(1, dtype=torch.uint8, device="cuda"))
    assert e.value.status in (4, 5)
    with pytest.raises(mq.MqError) as e:
        mq.mq_gemv_sliced(torch.zeros(17, 64, dtype=torch.bfloat16, device="cuda"), Q, a.bfloat16(), a.bfloat16(), 8, 64)
    assert e.value.status == 2
    # empty problems are no-ops
    assert mq.mq_linear_fwd_multi(X[:0], Q, a, a, (8,))[0].shape == (0, 8)
    assert mq.mq_slice(Q[:0], 4).shape == (0, 64)
