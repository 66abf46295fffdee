"""The no-allocation variant of tlq_x_stat (partial sums in the library's fixed device
array) against the workspace variant: same kernels, so the results must be bit-identical.
Two calls in a row share the array; the second uses a smaller input."""
import ctypes as C

import numpy as np
import pytest

from paper_2602_07899_amd import tlq

pytestmark = pytest.mark.gpu


def _both(torch, gpu, n_tok, c_in, ld, kind, dtype, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    Xfull = (torch.randn((n_tok, ld), generator=g, dtype=torch.float32) * 3.0).to(dtype).to(gpu)
    X = Xfull[:, :c_in]
    p = tlq.params(xstat_kind=kind, x_dtype=tlq.BF16 if dtype == torch.bfloat16 else tlq.F16)
    tlq.profile_enable(False)   # an earlier test may have left per-kernel timing on
    want = torch.full((c_in,), -1.0, dtype=torch.float32, device=gpu)
    got = torch.full((c_in,), -2.0, dtype=torch.float32, device=gpu)
    tlq.x_stat(X, p, want)
    # raw C ABI call: pointers and sizes only
    st = tlq.lib().tlq_x_stat_static(C.c_void_p(X.data_ptr()), n_tok, c_in, X.stride(0), C.byref(p),
                                     C.c_void_p(got.data_ptr()),
                                     C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == tlq.OK, tlq.status_string(st)
    torch.cuda.synchronize()
    return want.cpu().numpy(), got.cpu().numpy(), X


def test_x_stat_static_matches_workspace_variant_two_calls(gpu):
    import torch
    from oracle import tlq_oracle as orc
    # first call: several row chunks, ragged channel tail, strided rows; second call: smaller input
    for (n_tok, c_in, ld, kind, dtype, seed) in ((20000, 1288, 1296, 0, torch.float16, 1),
                                                 (777, 520, 520, 0, torch.float16, 2),
                                                 (5000, 2048, 2048, 1, torch.bfloat16, 3),
                                                 (130, 64, 72, 1, torch.bfloat16, 4)):
        want, got, X = _both(torch, gpu, n_tok, c_in, ld, kind, dtype, seed)
        assert np.array_equal(want.view(np.uint32), got.view(np.uint32)), (n_tok, c_in, kind)
        ref = (orc.x_stat_mean if kind == 0 else orc.x_stat_max)(X.float().cpu().numpy())
        assert np.array_equal(got, ref), (n_tok, c_in, kind)


def test_x_stat_static_limits(gpu):
    import torch
    p = tlq.params()
    c_big = 16384 + 8
    X = torch.zeros((4, c_big), dtype=torch.float16, device=gpu)
    out = torch.zeros(c_big, dtype=torch.float32, device=gpu)
    with pytest.raises(tlq.TlqError) as e:
        tlq.x_stat_static(X, p, out)
    assert e.value.status == tlq.ERR_WORKSPACE
    X = torch.ones((4, 16384), dtype=torch.float16, device=gpu)
    tlq.x_stat_static(X, p, out[:16384])
    torch.cuda.synchronize()
    assert bool((out[:16384] == 1.0).all())
    # per-kernel timing creates HIP events: refused while it is on
    tlq.profile_enable(True)
    try:
        with pytest.raises(tlq.TlqError) as e:
            tlq.x_stat_static(X, p, out[:16384])
        assert e.value.status == tlq.ERR_UNSUPPORTED
    finally:
        tlq.profile_enable(False)
