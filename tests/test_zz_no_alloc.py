"""The forward entry point that allocates nothing (built-in scratch) against mq_linear_fwd_multi, through the C ABI:
two calls in a row, the second with a smaller input; outputs must be bit-identical to the workspace entry point's
(the same kernels run on the same operands)."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _randn(seed, *shape, scale=1.0):
    return torch.randn(*shape, generator=torch.Generator().manual_seed(seed)) * scale


def test_noalloc_forward_matches_workspace_forward():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_06786_amd as mq
    lib = mq.lib()
    vp = ctypes.c_void_p
    rs = (8, 4, 2)
    c_rs = (ctypes.c_int * 3)(*rs)
    stream = vp(torch.cuda.current_stream().cuda_stream)
    for seed, (M, N, K) in enumerate([(600, 392, 464), (130, 136, 208)]):      # the second call is the smaller one
        print(f"no-alloc forward M={M} N={N} K={K}", flush=True)
        W = _randn(10 + seed, N, K, scale=0.02).cuda()
        X = _randn(20 + seed, M, K).to(torch.bfloat16).cuda()
        Q, a, z = mq.mq_quantize_int8(W)
        want = mq.mq_linear_fwd_multi(X, Q, a, z, rs)
        got = [torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in rs]
        ptrs = (vp * 3)(*[t.data_ptr() for t in got])
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        st = lib.mq_linear_fwd_multi_noalloc(vp(X.data_ptr()), vp(Q.data_ptr()), vp(a.data_ptr()), vp(z.data_ptr()),
                                             M, N, K, c_rs, 3, 0, ptrs, stream)
        assert st == 0, mq.status_string(st)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before        # no device memory was taken
        for r, g, w in zip(rs, got, want):
            assert torch.equal(g.view(torch.int16), w.view(torch.int16)), r
    # beyond the built-in scratch: refused before anything is launched
    st = lib.mq_linear_fwd_multi_noalloc(vp(X.data_ptr()), vp(Q.data_ptr()), vp(a.data_ptr()), vp(z.data_ptr()),
                                         (1 << 18) + 1, N, K, c_rs, 3, 0, ptrs, stream)
    assert st == 2
