"""HIP path vs CPU oracle at the full sizes of configurations 2-5, in the launch configuration the
bench times.  Codes, packed planes and overflow lists are compared in full (bit-exact); Y, dX, dW
are compared on >= 4096 randomly sampled outputs per tensor, each a full-length fp64 dot product in
the oracle; the decode GEMV outputs are compared in full.
"""
import numpy as np
import pytest
import torch

from tests.util import bf16_bits, first_overflow_code, rel_l2

pytestmark = pytest.mark.gpu

TOL = 1e-2
NSAMPLES = 4096


@pytest.fixture(scope="module")
def mq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_06786_amd as mq_

    mq_.lib()
    return mq_


def _samples(seed, rows, cols):
    rng = np.random.default_rng(seed)
    return rng.integers(0, rows, NSAMPLES), rng.integers(0, cols, NSAMPLES)


def _pick(t, i, j):
    return t[torch.from_numpy(i).cuda(), torch.from_numpy(j).cuda()].float().cpu().numpy().astype(np.float64)


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
    ms, ns = _samples(config * 10 + 1, M, N)
    for r, Y in zip(rs, Ys):
        want = oracle.linear_fwd_sampled(xb, qo, ao, zo, r, ms, ns)
        err = rel_l2(_pick(Y, ms, ns), want)
        print(f"  Y_{r}: rel-L2 {err:.2e}", flush=True)
        assert err <= TOL, (r, err)
    if config == 5:
        # extra precision vs plain at r = 2 (one bit-width per launch)
        for ep in (False, True):
            (Y2,) = mq.mq_linear_fwd_multi(X, Q, alpha, zero, (2,), extra_precision=ep)
            want = oracle.linear_fwd_sampled(xb, qo, ao, zo, 2, ms, ns, ep=ep)
            assert rel_l2(_pick(Y2, ms, ns), want) <= TOL, ("r=2", ep)
    del Ys
    if config == 2:
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
            err = rel_l2(_pick(dYs[i], ms, ns), want_d[i].ravel() * (NSAMPLES / (M * N)))
            print(f"  fused dY_{r}: rel-L2 {err:.2e}  loss {got_l[i]:.4e} (sample estimate {est[i]:.4e})", flush=True)
            assert err <= TOL, (r, err)
            tied = float((dYs[i].double() ** 2).mean().item()) * (M * N) ** 2 / (4.0 * lam[i] ** 2)
            assert abs(got_l[i] - tied) <= TOL * tied, (r, got_l[i], tied)       # dY is rounded to bf16
            assert abs(got_l[i] - est[i]) <= 0.1 * est[i], (r, got_l[i], est[i])  # 4096 samples: a few per cent
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
    ms, ks = _samples(config * 10 + 2, M, K)
    want = oracle.linear_bwd_dx_sampled(qo, ao, zo, dyb, lam, rs, ms, ks)
    err = rel_l2(_pick(dX, ms, ks), want)
    print(f"  dX: rel-L2 {err:.2e}", flush=True)
    assert err <= TOL, ("dX", err)
    ns, ks = _samples(config * 10 + 3, N, K)
    want = oracle.linear_bwd_dw_sampled(xb, dyb, lam, ns, ks)
    err = rel_l2(_pick(dW, ns, ks), want)
    print(f"  dW: rel-L2 {err:.2e}", flush=True)
    assert err <= TOL, ("dW", err)


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
            err = rel_l2(y.float().cpu().numpy(), want)
            print(f"  int{r} B={B}: rel-L2 {err:.2e}", flush=True)
            assert err <= TOL, (r, B, err)


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
                err = rel_l2(y.float().cpu().numpy(), want)
                assert err <= TOL, (label, B, use_ovf, err)
                if use_ovf:   # the dense 3-bit plane holds the same weights
                    yd = mq.mq_gemv_sliced_dense_ep(x.cuda(), dense, a16, z16, 2, K)
                    assert rel_l2(yd.float().cpu().numpy(), want) <= TOL, (label, B, "dense")
