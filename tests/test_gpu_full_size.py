"""HIP path vs CPU oracle at the full sizes of configurations 2-5, in the launch configuration the
bench times.  Codes, packed planes and overflow lists are compared in full (bit-exact).  Y, dX, dW are
compared (a) on a stratified sample with one entry in every block of 32 tokens x 32 channels (Y), 32 tokens x
64 features (dX), 64 channels x 64 features (dW) - blocks that divide every output tile of the three
matrix-core kernels (forward 128 channels x 128 or 160 tokens with 32 channels per wave, dX 160 tokens x 256
features, dW 256 channels x 192 features), so no tile and no wave's part of a tile goes unsampled - and
(b) on 64 full rows and 64 full columns per tensor; every compared entry is a full-length fp64 dot product in
the oracle and has to meet the element bar of tests.util.assert_close next to the rel-L2 bar.  The decode
GEMV outputs are compared in full.
"""
import numpy as np
import pytest
import torch

from tests.util import accumulation_allowance, assert_close, bf16_bits, first_overflow_code, rel_l2

pytestmark = pytest.mark.gpu

TOL = 1e-2
NFULL = 64           # full rows and full columns per tensor
C_Y, C_GRAD = 2.0 ** -7, 2.0 ** -6   # absolute part of the element bar, in units of rms(want): see assert_close


@pytest.fixture(scope="module")
def mq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_06786_amd as mq_

    mq_.lib()
    return mq_


def _strata(seed, rows, cols, rb, cb):
    """One uniformly drawn entry in every rb x cb block of a rows x cols matrix (ragged last blocks included)."""
    rng = np.random.default_rng(seed)
    r0 = np.arange(0, rows, rb)
    c0 = np.arange(0, cols, cb)
    R0, C0 = np.meshgrid(r0, c0, indexing="ij")
    R0, C0 = R0.ravel(), C0.ravel()
    i = R0 + (rng.random(R0.size) * np.minimum(rb, rows - R0)).astype(np.int64)
    j = C0 + (rng.random(C0.size) * np.minimum(cb, cols - C0)).astype(np.int64)
    return i, j


def _lines(seed, n, count=NFULL):
    """`count` distinct indices below n, the first and the last always among them."""
    rng = np.random.default_rng(seed)
    pick = rng.choice(n, size=min(count, n), replace=False)
    pick[0], pick[-1] = 0, n - 1
    return np.unique(pick)


def _pick(t, i, j):
    return t[torch.from_numpy(i).cuda(), torch.from_numpy(j).cuda()].float().cpu().numpy().astype(np.float64)


def _rows(t, i):
    return t[torch.from_numpy(i).cuda()].float().cpu().numpy().astype(np.float64)


def _cols(t, j):
    return t[:, torch.from_numpy(j).cuda()].float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("config,name", [(2, "gate"), (2, "up"), (2, "down"), (3, "gate"), (3, "down"),
                                         (5, "gate"), (5, "down")])
def test_training_path_full_size(mq, oracle, config, name):
    from paper_2502_06786_amd import synth
    print(f"config {config} linear {name}", flush=True)
    case = synth.linear_case(config, name)
    M, N, K, rs, lam = case.M, case.N, case.K, case.rs, case.lambdas
    W = case.W.cuda()
    Q, alpha, zero = mq.mq_quantize_int8(W)
    del W
    qo, ao, zo = oracle.quantize_int8(case.W.numpy())
    assert np.array_equal(alpha.cpu().numpy(), ao) and np.array_equal(zero.cpu().numpy(), zo)
    assert np.array_equal(Q.cpu().numpy(), qo)

    # slice + pack, and the overflow list of the r = 2 slice; the oracle checks a slab of rows
    rows = np.r_[0:min(N, 2048), max(0, N - 512):N]
    for r in (4, 2):
        packed, ovf = mq.mq_slice(Q, r, packed=True, extra_precision=True, capacity=N * K // 8)
        torch.cuda.synchronize()
        assert np.array_equal(packed.cpu().numpy()[rows], oracle.pack(oracle.slice_codes(qo[rows], r), r))
        rp, ci = oracle.overflow_csr(qo, r)
        assert int(ovf.nnz.item()) == ci.size
        assert np.array_equal(ovf.row_ptr.cpu().numpy(), rp)
        assert np.array_equal(ovf.col_idx.cpu().numpy().view(np.uint16)[:ci.size], ci)
        del packed, ovf

    X = case.X.cuda()
    xb = bf16_bits(case.X)
    Ys = mq.mq_linear_fwd_multi(X, Q, alpha, zero, rs)
    ms, ns = _strata(config * 10 + 1, M, N, 32, 32)
    mrows, ncols = _lines(config * 10 + 6, M), _lines(config * 10 + 7, N)
    qc, ac, zc = np.ascontiguousarray(qo[ncols]), ao[ncols], zo[ncols]
    x_rms = float(case.X.float().pow(2).mean().sqrt())

    def allow_y(r, alpha_n):   # fp32 accumulation over K of 128 + code against x, in units of the output
        return accumulation_allowance(K, x_rms, alpha_n.astype(np.float64) * float(1 << (8 - r)))

    for r, Y in zip(rs, Ys):
        want = oracle.linear_fwd_sampled(xb, qo, ao, zo, r, ms, ns)
        err = assert_close(_pick(Y, ms, ns), want, C_Y, what=f"Y_{r} strata", extra=allow_y(r, ao[ns]))
        assert_close(_rows(Y, mrows), oracle.linear_fwd(xb[mrows], qo, ao, zo, r), C_Y, what=f"Y_{r} rows", extra=allow_y(r, ao)[None, :])
        assert_close(_cols(Y, ncols), oracle.linear_fwd(xb, qc, ac, zc, r), C_Y, what=f"Y_{r} columns", extra=allow_y(r, ac)[None, :])
        print(f"  Y_{r}: rel-L2 {err:.2e} on {ms.size} strata", flush=True)
    if config == 5:
        # extra precision vs plain at r = 2 (one bit-width per launch)
        for ep in (False, True):
            (Y2,) = mq.mq_linear_fwd_multi(X, Q, alpha, zero, (2,), extra_precision=ep)
            want = oracle.linear_fwd_sampled(xb, qo, ao, zo, 2, ms, ns, ep=ep)
            assert_close(_pick(Y2, ms, ns), want, C_Y, what=("r=2", ep), extra=allow_y(2, ao[ns]))
            assert_close(_rows(Y2, mrows[:16]), oracle.linear_fwd(xb[mrows[:16]], qo, ao, zo, 2, ep=ep), C_Y, what=("r=2 rows", ep),
                         extra=allow_y(2, ao)[None, :])
    del Ys
    if config in (2, 3):
        # the call the bench times: the same forward with the L2 objective in its epilogue (no Y stored).
        # Sampled gradients against the oracle; the losses, sums over all M N outputs, through what ties
        # them to the gradients at any size (loss_i = M N / (4 lambda_i^2) * mean(dY_i^2)) and against the
        # oracle's estimate from the sample.
        wants = [oracle.linear_fwd_sampled(xb, qo, ao, zo, r, ms, ns) for r in rs]
        scale = float(np.std(wants[0]))
        T = (torch.randn(M, N, generator=torch.Generator().manual_seed(config * 10 + 4)) * scale).to(torch.bfloat16)
        teacher = (-1, 0, 0)
        losses, dYs = mq.mq_linear_fwd_multi_l2(X, Q, alpha, zero, rs, T.cuda(), teacher, lam)
        torch.cuda.synchronize()
        tb = bf16_bits(T)[ms, ns].reshape(1, -1)
        est, want_d = oracle.matquant_l2_loss([oracle.bf16_round(w).reshape(1, -1) for w in wants], tb, teacher, lam)
        got_l = losses.cpu().numpy().astype(np.float64)
        for i, r in enumerate(rs):
            # dY_i = coef_i (Y_i - T_i): a bf16 step of Y_i or of its teacher output moves it by coef_i times that step
            coef = lam[i] * 2.0 / (M * N)
            step = np.abs(wants[i]) + (np.abs(wants[teacher[i]]) if teacher[i] >= 0 else 0.0)
            err = assert_close(_pick(dYs[i], ms, ns), want_d[i].ravel() * (ms.size / (M * N)), C_GRAD, what=f"fused dY_{r}",
                               extra=coef * (2.0 ** -7 * step + allow_y(r, ao[ns])))
            print(f"  fused dY_{r}: rel-L2 {err:.2e}  loss {got_l[i]:.4e} (sample estimate {est[i]:.4e})", flush=True)
            tied = float((dYs[i].double() ** 2).mean().item()) * (M * N) ** 2 / (4.0 * lam[i] ** 2)
            assert abs(got_l[i] - tied) <= TOL * tied, (r, got_l[i], tied)       # dY is rounded to bf16
            assert abs(got_l[i] - est[i]) <= 0.1 * est[i], (r, got_l[i], est[i])  # tens of thousands of samples: a few per cent
        del dYs, T

    dY = [d.cuda() for d in case.dY]
    dyb = [bf16_bits(d) for d in case.dY]
    if config == 2 and name == "gate":
        # gradients with respect to the clip factors: every row is an independent reduction, so the oracle
        # evaluates a sample of rows (its inputs restricted to them) in full
        Wd = case.W.cuda()
        dg, db = mq.mq_linear_bwd_clip(Wd, X, Q, alpha, zero, dY, lam, rs)
        rows_c = np.random.default_rng(config * 10 + 5).choice(N, 96, replace=False)
        want_g, want_b, _, _ = oracle.clip_factor_grads(case.W.numpy()[rows_c], xb, [d[:, rows_c] for d in dyb], lam, rs)
        for nm, mine, ref in (("dgamma", dg, want_g), ("dbeta", db, want_b)):
            err = rel_l2(mine.cpu().numpy().astype(np.float64)[rows_c], ref)
            print(f"  {nm}: rel-L2 {err:.2e}", flush=True)
            assert err <= TOL, (nm, err)
        del Wd
    dX, dW = mq.mq_linear_bwd(X, Q, alpha, zero, dY, lam, rs)
    # fp32 accumulation over the channels and bit-widths of 128 + code against lambda_r alpha_n 2^s dY_r
    dy_rms = float(case.dY[0].float().pow(2).mean().sqrt())
    op_rms = float(np.sqrt(np.mean([(l * (1 << (8 - r))) ** 2 for l, r in zip(lam, rs)]))) * float(np.sqrt(np.mean(ao.astype(np.float64) ** 2))) * dy_rms
    allow_dx = float(accumulation_allowance(N * len(rs), op_rms, 1.0))
    ms, ks = _strata(config * 10 + 2, M, K, 32, 64)
    want = oracle.linear_bwd_dx_sampled(qo, ao, zo, dyb, lam, rs, ms, ks)
    err = assert_close(_pick(dX, ms, ks), want, C_GRAD, what="dX strata", extra=allow_dx)
    print(f"  dX: rel-L2 {err:.2e} on {ms.size} strata", flush=True)
    mrows, kcols = _lines(config * 10 + 8, M), _lines(config * 10 + 9, K)
    assert_close(_rows(dX, mrows), oracle.linear_bwd_dx(qo, ao, zo, [d[mrows] for d in dyb], lam, rs), C_GRAD, what="dX rows", extra=allow_dx)
    assert_close(_cols(dX, kcols), oracle.linear_bwd_dx(np.ascontiguousarray(qo[:, kcols]), ao, zo, dyb, lam, rs), C_GRAD,
                 what="dX columns", extra=allow_dx)
    ns, ks = _strata(config * 10 + 3, N, K, 64, 64)
    want = oracle.linear_bwd_dw_sampled(xb, dyb, lam, ns, ks)
    err = assert_close(_pick(dW, ns, ks), want, C_GRAD, what="dW strata")
    print(f"  dW: rel-L2 {err:.2e} on {ns.size} strata", flush=True)
    nrows = _lines(config * 10 + 10, N)
    assert_close(_rows(dW, nrows), oracle.linear_bwd_dw(xb, [np.ascontiguousarray(d[:, nrows]) for d in dyb], lam), C_GRAD,
                 what="dW rows")
    assert_close(_cols(dW, kcols), oracle.linear_bwd_dw(np.ascontiguousarray(xb[:, kcols]), dyb, lam), C_GRAD, what="dW columns")


def test_training_block_full_size(mq, oracle):
    """The whole gated feed-forward block of configuration 2 on the training path (4096 tokens, d 2304, F 9216; r = 8/4/2):
    stacked gate / up layer with the gate in its epilogue, one down layer per bit-width, and the way back (down
    backward per bit-width, stacked backward with the gate gradient in its first pass), against the oracle's own
    chain of the same steps on 48 whole token rows (GU_r, A_r, Y_r, dA_r, dX) and on 32 whole (gate, up) channel
    pairs (the rows of dW of the stacked layer and the columns of dW of the down layer that belong to them)."""
    from paper_2502_06786_amd import synth
    shapes, M = synth.mlp_shapes(2)
    F, d = shapes["gate"]
    rs, lam = (8, 4, 2), (0.3, 0.6, 1.0)
    Wgu = torch.empty(2 * F, d)
    Wgu[0::2], Wgu[1::2] = synth.weight(2, "gate"), synth.weight(2, "up")
    Wd = synth.weight(2, "down") * 4.0        # (a down layer whose outputs are of order one)
    X = synth.activations(2, "gate", M, d)
    dYs = [(torch.randn(M, d, generator=torch.Generator().manual_seed(70 + i)) * 1e-2).to(torch.bfloat16) for i in range(3)]
    Qg, ag, zg = mq.mq_quantize_int8(Wgu.cuda())
    Qd, ad, zd = mq.mq_quantize_int8(Wd.cuda())
    qg, aog, zog = oracle.quantize_int8(Wgu.numpy())
    qd, aod, zod = oracle.quantize_int8(Wd.numpy())
    assert np.array_equal(Qg.cpu().numpy(), qg) and np.array_equal(Qd.cpu().numpy(), qd)
    # ---- library, in full
    Xd = X.cuda()
    GU, A = mq.mq_linear_fwd_multi_gated(Xd, Qg, ag, zg, rs)
    Y = [mq.mq_linear_fwd_multi(A[i], Qd, ad, zd, (r,))[0] for i, r in enumerate(rs)]
    dA, dWd = [], torch.zeros(d, F, device="cuda")
    for i, r in enumerate(rs):
        dx, _ = mq.mq_linear_bwd(A[i], Qd, ad, zd, [dYs[i].cuda()], (lam[i],), (r,), dW=dWd, accumulate_dW=True)
        dA.append(dx)
    dX, dWgu = mq.mq_linear_bwd_gated(Xd, Qg, ag, zg, GU, dA, None, rs)
    torch.cuda.synchronize()
    # ---- oracle on 48 token rows: every step of the chain is per token
    xb = bf16_bits(X)
    mrows = _lines(91, M, 48)
    ones = (1.0,) * 3
    wide = dict(c_rms=2.0 ** -5, tol=2 * TOL)   # a GU or dA rounded to the other bf16 neighbour moves what follows by a step
    GU_o, A_o, dA_o, dGU_o = [], [], [], []
    for i, r in enumerate(rs):
        GU_o.append(oracle.bf16_round(oracle.linear_fwd(xb[mrows], qg, aog, zog, r)))
        assert_close(_rows(GU[i], mrows), oracle.bf16_to_f64(GU_o[i]), C_Y, what=f"GU_{r} rows")
        A_o.append(oracle.gated_unit(GU_o[i]))
        assert_close(_rows(A[i], mrows), oracle.bf16_to_f64(A_o[i]), what=f"A_{r} rows", **wide)
        assert_close(_rows(Y[i], mrows), oracle.linear_fwd(A_o[i], qd, aod, zod, r), what=f"Y_{r} rows", **wide)
        dyb = bf16_bits(dYs[i][torch.from_numpy(mrows)])
        dA_o.append(oracle.bf16_round(oracle.linear_bwd_dx(qd, aod, zod, [dyb], (lam[i],), (r,))))
        assert_close(_rows(dA[i], mrows), oracle.bf16_to_f64(dA_o[i]), C_GRAD, what=f"dA_{r} rows")
        dGU_o.append(oracle.bf16_round(oracle.gated_unit_bwd(GU_o[i], dA_o[i])))
    assert_close(_rows(dX, mrows), oracle.linear_bwd_dx(qg, aog, zog, dGU_o, ones, rs), what="dX rows", **wide)
    print("  token rows ok", flush=True)
    # ---- oracle on 32 (gate, up) pairs, all tokens: the columns of GU, A, dA, dGU that belong to them
    fs = _lines(92, F, 32)
    cols = np.stack([2 * fs, 2 * fs + 1], axis=1).ravel()          # stacked channels of the pairs, pair by pair
    dWd_o, dGUc = np.zeros((d, fs.size)), []
    for i, r in enumerate(rs):
        GUc = oracle.bf16_round(oracle.linear_fwd(xb, np.ascontiguousarray(qg[cols]), aog[cols], zog[cols], r))     # [M, 64]
        Ac = oracle.gated_unit(GUc)                                                                                # [M, 32]
        dyb = bf16_bits(dYs[i])
        dAc = oracle.bf16_round(oracle.linear_bwd_dx(np.ascontiguousarray(qd[:, fs]), aod, zod, [dyb], (lam[i],), (r,)))   # [M, 32]
        dWd_o += oracle.linear_bwd_dw(Ac, [dyb], (lam[i],))                                                         # [d, 32]
        dGUc.append(oracle.bf16_round(oracle.gated_unit_bwd(GUc, dAc)))
    assert_close(_cols(dWd, fs), dWd_o, what="dW down columns", **wide)
    assert_close(_rows(dWgu, cols), oracle.linear_bwd_dw(xb, dGUc, ones), what="dW stacked rows", **wide)


@pytest.mark.parametrize("N", [3584, 896])
def test_attention_projection_shapes(mq, oracle, N):
    """The fused forward and the backward on attention-projection shapes of the 9B-shaped model (section 5 also quantizes
    attention weights): a square projection d -> d and a grouped-query key / value projection d -> d / 4, 8192 tokens;
    stratified samples as in test_training_path_full_size."""
    K, M, rs, lam = 3584, 8192, (8, 4, 2), (0.1, 0.1, 1.0)
    g = torch.Generator().manual_seed(N)
    W = torch.randn(N, K, generator=g) * 0.015
    X = torch.randn(M, K, generator=g).to(torch.bfloat16)
    dYs = [(torch.randn(M, N, generator=g) * 1e-3).to(torch.bfloat16) for _ in rs]
    Q, alpha, zero = mq.mq_quantize_int8(W.cuda())
    qo, ao, zo = oracle.quantize_int8(W.numpy())
    assert np.array_equal(Q.cpu().numpy(), qo)
    xb, dyb = bf16_bits(X), [bf16_bits(t) for t in dYs]
    Ys = mq.mq_linear_fwd_multi(X.cuda(), Q, alpha, zero, rs)
    ms, ns = _strata(N + 1, M, N, 32, 32)
    for r, Y in zip(rs, Ys):
        extra = accumulation_allowance(K, 1.0, ao[ns].astype(np.float64) * float(1 << (8 - r)))
        assert_close(_pick(Y, ms, ns), oracle.linear_fwd_sampled(xb, qo, ao, zo, r, ms, ns), C_Y, what=f"Y_{r}", extra=extra)
    dX, dW = mq.mq_linear_bwd(X.cuda(), Q, alpha, zero, [t.cuda() for t in dYs], lam, rs)
    ms, ks = _strata(N + 2, M, K, 32, 64)
    assert_close(_pick(dX, ms, ks), oracle.linear_bwd_dx_sampled(qo, ao, zo, dyb, lam, rs, ms, ks), C_GRAD, what="dX")
    ns, ks = _strata(N + 3, N, K, 64, 64)
    assert_close(_pick(dW, ns, ks), oracle.linear_bwd_dw_sampled(xb, dyb, lam, ns, ks), C_GRAD, what="dW")


@pytest.mark.parametrize("N,K", [(4096, 4096), (14336, 4096), (4096, 14336)])
def test_decode_gemv_7b_shapes(mq, oracle, N, K):
    from paper_2502_06786_amd import synth
    print(f"decode {K}->{N}", flush=True)
    W = synth.weight(4, f"{N}x{K}", (N, K))
    Q, alpha, zero = mq.mq_quantize_int8(W.cuda())
    a16, z16 = mq.mq_params_to_bf16(alpha, zero)
    ab, zb = bf16_bits(a16), bf16_bits(z16)
    for r in (4, 2, 6, 3):   # 6 and 3: the interpolated bit-widths, stored as bit streams
        packed = mq.mq_slice(Q, r, packed=True)
        pk = packed.cpu().numpy()
        assert np.array_equal(pk, oracle.pack(oracle.slice_codes(Q.cpu().numpy(), r), r))
        for B in synth.DECODE_BATCHES:
            x = synth.activations(4, f"x{B}:{N}x{K}", B, K)
            y = mq.mq_gemv_sliced(x.cuda(), packed, a16, z16, r, K)
            want = oracle.gemv_sliced(bf16_bits(x), pk, ab, zb, r, K)
            err = assert_close(y.float().cpu().numpy(), want, C_Y, what=(r, B))
            print(f"  int{r} B={B}: rel-L2 {err:.2e}", flush=True)


@pytest.mark.parametrize("name", ["gate", "down"])
def test_extra_precision_gemv_27b_shape(mq, oracle, name):
    """Configuration 5: int2 plain vs int2 + outlier bit on heavy-tailed weights, plus the same layer
    with codes planted at the paper's overflow density (about 5 % at r = 2, Table 7)."""
    from paper_2502_06786_amd import synth
    shapes, _ = synth.mlp_shapes(5)
    N, K = shapes[name]
    print(f"config 5 {name} {N}x{K}", flush=True)
    W = synth.weight(5, name)
    Q, alpha, zero = mq.mq_quantize_int8(W.cuda())
    del W
    a16, z16 = mq.mq_params_to_bf16(alpha, zero)
    ab, zb = bf16_bits(a16), bf16_bits(z16)
    for label, codes in (("minmax", Q), ("planted5pct", synth.planted_codes(55, N, K, first_overflow_code(2), 0.05).cuda())):
        packed, ovf = mq.mq_slice(codes, 2, packed=True, extra_precision=True, capacity=N * K // 8)
        torch.cuda.synchronize()
        qn = codes.cpu().numpy()
        rp, ci = oracle.overflow_csr(qn, 2)
        assert int(ovf.nnz.item()) == ci.size
        assert np.array_equal(ovf.col_idx.cpu().numpy().view(np.uint16)[:ci.size], ci)
        pk = packed.cpu().numpy()
        print(f"  {label}: overflow fraction {ci.size / qn.size:.4f}", flush=True)
        dense = mq.mq_slice(codes, 2, packed=True, extra_precision=True, dense_ep=True)
        dn = dense.cpu().numpy()
        assert np.array_equal(dn[:1024], oracle.pack(oracle.slice_codes(qn[:1024], 2, ep=True), 3))
        for B in synth.DECODE_BATCHES:
            x = synth.activations(5, f"x{B}:" + name, B, K)
            for use_ovf in (False, True):
                y = mq.mq_gemv_sliced(x.cuda(), packed, a16, z16, 2, K, ovf=ovf if use_ovf else None)
                want = oracle.gemv_sliced(bf16_bits(x), pk, ab, zb, 2, K, ovf=(rp, ci) if use_ovf else None)
                assert_close(y.float().cpu().numpy(), want, C_Y, what=(label, B, use_ovf))
                if use_ovf:   # the dense 3-bit plane holds the same weights
                    yd = mq.mq_gemv_sliced_dense_ep(x.cuda(), dense, a16, z16, 2, K)
                    assert_close(yd.float().cpu().numpy(), want, C_Y, what=(label, B, "dense"))
