"""Gradient-guided token selection on the GPU (Sec. 3.1.2) against the oracle:
gradient statistic, Top-K set, masked channel maximum, and a search that uses
the resulting x_stat."""
import numpy as np
import pytest

from oracle import tlq_oracle as orc
from paper_2602_07899_amd import tlq
from paper_2602_07899_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _grads(rng, B, N, C, n_vis):
    # most visual tokens carry near-zero gradient, text tokens and a few visual ones matter
    g = rng.standard_normal((B, N, C)).astype(np.float32)
    amp = np.where(np.arange(N) < n_vis, rng.lognormal(-4.0, 1.5, N), rng.lognormal(0.0, 0.5, N))
    return (g * amp[None, :, None]).reshape(B * N, C).astype(np.float16)


@pytest.mark.parametrize("B,N,C,n_vis,l2", [(4, 128, 512, 96, False), (3, 1200, 1000, 1152, True), (128, 37, 64, 30, False)])
def test_selection_pipeline(gpu, B, N, C, n_vis, l2):
    import torch
    rng = np.random.default_rng(B * N + C)
    G = _grads(rng, B, N, C, n_vis)
    X = (rng.standard_normal((B * N, C)) * rng.uniform(0.2, 5, C)).astype(np.float16)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu)
    p = tlq.params()
    sum_n = torch.empty(N, dtype=torch.float64, device=gpu)
    tlq.token_importance(t(G), B, p, sum_n, l2=l2)
    ref = orc.token_importance(G, B, l2=l2)
    np.testing.assert_allclose(sum_n.cpu().numpy(), ref, rtol=1e-12)
    k = N // 2
    mask = torch.empty(N, dtype=torch.uint8, device=gpu)
    tlq.topk_mask(sum_n, k, mask)
    m = mask.cpu().numpy().astype(bool)
    rm = orc.top_fraction_mask(ref, k)
    assert m.sum() == k
    if not np.array_equal(m, rm):       # only positions whose statistics agree to rounding may swap
        diff = np.flatnonzero(m != rm)
        assert np.ptp(ref[diff]) <= 1e-12 * np.abs(ref[diff]).max()
    # the oracle's own mask feeds the masked maximum on both sides
    xs = torch.empty(C, dtype=torch.float32, device=gpu)
    tlq.x_stat_masked(t(X), t(rm.astype(np.uint8)), p, xs)
    assert np.array_equal(xs.cpu().numpy(), orc.x_stat_topk_max(X, rm))


def test_search_with_topk_x_stat(gpu):
    import torch
    c = wl.CONFIGS["cfg3_mini_w3"]
    X, W, w = wl.make_tokens(c, 0), wl.make_weight(c, 0), wl.make_token_weights(c, 0)
    N = c.n_vis + c.n_txt
    rng = np.random.default_rng(0)
    G = _grads(rng, c.n_samples, N, X.shape[1], c.n_vis)
    mask = orc.top_fraction_mask(orc.token_importance(G, c.n_samples), N // 2)
    xs = orc.x_stat_topk_max(X, mask)
    al = wl.alpha_grid(8)
    Y = orc.ref_output(X, W).astype(np.float16)
    ref = orc.scale_search(X, W, Y, w, 4, 128, al, x_stat=xs, act_bits=8)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu)
    p = tlq.params(bits=4, group=128, act_bits=8)
    gm = torch.empty(N, dtype=torch.uint8, device=gpu)
    sn = torch.empty(N, dtype=torch.float64, device=gpu)
    tlq.token_importance(t(G), c.n_samples, p, sn)
    tlq.topk_mask(sn, N // 2, gm)
    gxs = torch.empty(X.shape[1], dtype=torch.float32, device=gpu)
    tlq.x_stat_masked(t(X), gm, p, gxs)
    assert np.array_equal(gxs.cpu().numpy(), xs)
    best = torch.empty(X.shape[1], dtype=torch.float32, device=gpu)
    idx = torch.empty(1, dtype=torch.int32, device=gpu)
    losses = torch.empty(al.size, dtype=torch.float32, device=gpu)
    tlq.scale_search(t(X), t(W), t(Y), t(w), t(al), p, best, idx, losses, x_stat_in=gxs)
    rel = np.abs(losses.cpu().numpy() - ref["losses"]) / ref["losses"]
    assert rel.max() < 1e-3 and int(idx.item()) == ref["best_idx"]
