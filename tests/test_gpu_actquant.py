"""GPU parity of the activation-quantised candidate evaluation (the paper's
W4A8 / W4A6 setting: f_q = Q_w(W*scale) Q_a(x/scale), Sec. 3.2.1) against the
oracle: integer codes and per-token steps bit-exact, losses within 1e-3."""
import numpy as np
import pytest

from oracle import tlq_oracle as orc
from paper_2602_07899_amd import tlq
from paper_2602_07899_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _t(a, gpu, bf16=False):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    return (t.to(torch.bfloat16) if bf16 else t).to(gpu)


@pytest.mark.parametrize("n,c,abits,bf16", [(256, 512, 8, False), (300, 1096, 6, False), (5, 8, 4, False),
                                            (130, 11008, 8, False), (77, 13824, 8, True), (64, 4096, 2, True)])
def test_act_fake_quant_bit_exact(gpu, n, c, abits, bf16):
    import torch
    rng = np.random.default_rng(n + c)
    X = rng.standard_normal((n, c)).astype(np.float32)
    X[:, rng.choice(c, max(1, c // 100), replace=False)] *= 30.0
    X[0] = 0.0                                                # an all-zero token takes the floored step
    X = orc.round_to_bf16(X) if bf16 else X.astype(np.float16)
    s = rng.lognormal(0, 0.6, c).astype(np.float32)
    p = tlq.params(act_bits=abits, x_dtype=tlq.BF16 if bf16 else tlq.F16)
    for inv in (orc.recip_scale(s), None):
        codes = torch.empty((n, c), dtype=torch.float16, device=gpu)
        sigma = torch.empty(n, dtype=torch.float32, device=gpu)
        tlq.act_fake_quant(_t(X, gpu, bf16), None if inv is None else _t(inv, gpu), p, codes, sigma)
        rc, rs = orc.act_quant(X, inv, abits)
        assert np.array_equal(sigma.cpu().numpy().view(np.uint32), rs.view(np.uint32))
        assert np.array_equal(codes.cpu().numpy().astype(np.int16), rc)


def _search(gpu, X, W, Y, w, al, p, bf16=False):
    import torch
    n, ci = X.shape
    best = torch.empty(ci, dtype=torch.float32, device=gpu)
    idx = torch.empty(1, dtype=torch.int32, device=gpu)
    losses = torch.empty(al.size, dtype=torch.float32, device=gpu)
    tlq.scale_search(_t(X, gpu, bf16), _t(W, gpu, bf16), _t(Y, gpu), _t(w, gpu), _t(al, gpu), p, best, idx, losses)
    return best.cpu().numpy(), int(idx.item()), losses.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("abits", [8, 6, 4])
def test_scale_search_w4ax_cfg1(gpu, abits):
    c = wl.CONFIGS["cfg1_small"]
    X, W, w = wl.make_tokens(c, 0), wl.make_weight(c, 0), wl.make_token_weights(c, 0)
    al = wl.alpha_grid(c.n_alpha)
    Y = orc.ref_output(X, W).astype(np.float16)
    p = tlq.params(bits=4, group=128, act_bits=abits)
    best, idx, L = _search(gpu, X, W, Y, w, al, p)
    ref = orc.scale_search(X, W, Y, w, 4, 128, al, act_bits=abits)
    rel = np.abs(L - ref["losses"]) / ref["losses"]
    print(f"W4A{abits}: max rel loss error {rel.max():.2e}, best {idx} (oracle {ref['best_idx']})")
    assert rel.max() < 1e-3
    if idx != ref["best_idx"]:
        srt = np.sort(ref["losses"])
        assert (srt[1] - srt[0]) / srt[0] < 1e-3
    assert np.array_equal(best, ref["s_table"][idx])


@pytest.mark.parametrize("n,ci,co,bits,group,sym,abits,bf16", [
    (1000, 1024, 777, 4, 128, 0, 8, False), (515, 384, 300, 4, 0, 1, 6, False), (640, 1408, 512, 3, 64, 0, 8, True)])
def test_scale_search_act_ragged(gpu, n, ci, co, bits, group, sym, abits, bf16):
    """Includes the paper's own setting: per-channel symmetric weights (group = whole row,
    symmetric) with per-token symmetric activations."""
    rng = np.random.default_rng(n + ci + abits)
    X = rng.standard_normal((n, ci)).astype(np.float32)
    X[n // 2:, rng.choice(ci, max(1, ci // 100), replace=False)] *= 25.0
    W = (rng.standard_normal((co, ci)) * 0.02).astype(np.float32)
    X, W = (orc.round_to_bf16(X), orc.round_to_bf16(W)) if bf16 else (X.astype(np.float16), W.astype(np.float16))
    w = rng.lognormal(0, 1, n)
    w = (w / w.sum()).astype(np.float32)
    Y = orc.ref_output(X, W).astype(np.float32)
    al = wl.alpha_grid(10)
    p = tlq.params(bits=bits, group=group, symmetric=sym, act_bits=abits, x_dtype=tlq.BF16 if bf16 else tlq.F16,
                   yref_dtype=tlq.F32)
    import torch
    Yp = torch.zeros((n, (co + 7) // 8 * 8), dtype=torch.float32, device=gpu)
    Yp[:, :co] = _t(Y, gpu)
    best = torch.empty(ci, dtype=torch.float32, device=gpu)
    idx = torch.empty(1, dtype=torch.int32, device=gpu)
    losses = torch.empty(al.size, dtype=torch.float32, device=gpu)
    tlq.scale_search(_t(X, gpu, bf16), _t(W, gpu, bf16), Yp[:, :co], _t(w, gpu), _t(al, gpu), p, best, idx, losses)
    L = losses.cpu().numpy().astype(np.float64)
    ref = orc.scale_search(X, W, Y, w, bits, group, al, symmetric=bool(sym), act_bits=abits)
    rel = np.abs(L - ref["losses"]) / ref["losses"]
    print(f"{n}x{ci}x{co} W{bits}A{abits} sym={sym} bf16={bf16}: max rel loss error {rel.max():.2e}")
    assert rel.max() < 1e-3
    gi = int(idx.item())
    if gi != ref["best_idx"]:
        srt = np.sort(ref["losses"])
        assert (srt[1] - srt[0]) / srt[0] < 1e-3


def test_act_single_candidate_paths(gpu):
    """tlq_weighted_layer_err and tlq_apply_best with Q_a against the oracle."""
    import torch
    rng = np.random.default_rng(9)
    n, ci, co = 300, 512, 264
    X = rng.standard_normal((n, ci)).astype(np.float16)
    W = (rng.standard_normal((co, ci)) * 0.02).astype(np.float16)
    w = rng.uniform(0.1, 1, n).astype(np.float32)
    s = rng.lognormal(0, 0.5, ci).astype(np.float32)
    Y = orc.ref_output(X, W).astype(np.float16)
    p = tlq.params(bits=4, group=128, act_bits=8)
    _, _, _, deq = orc.fake_quant(W, s, 4, 128)
    wdq = deq.astype(np.float16)
    loss = torch.empty(1, dtype=torch.float32, device=gpu)
    pte = torch.empty(n, dtype=torch.float32, device=gpu)
    tlq.weighted_layer_err(_t(X, gpu), _t(wdq, gpu), _t(orc.recip_scale(s), gpu), _t(Y, gpu), _t(w, gpu), p, loss, pte)
    e = orc.per_token_err(Y, orc.quantised_output_aq(X, wdq, s, 8))
    np.testing.assert_allclose(pte.cpu().numpy(), e, rtol=1e-3)
    assert abs(loss.item() - float((w.astype(np.float64) * e).sum())) / float((w * e).sum()) < 1e-3
    out = torch.empty((n, co), dtype=torch.float16, device=gpu)
    tlq.apply_best(_t(X, gpu), _t(W, gpu), _t(s, gpu), p, out)
    ref = orc.apply_best(X, W, s, 4, 128, act_bits=8)
    codes, sigma = orc.act_quant(X, orc.recip_scale(s), 8)
    mag = (np.abs(codes.astype(np.float64)) @ np.abs(deq.astype(np.float64)).T) * sigma[:, None]
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2.0 ** -11 * (0.6 * mag + 1.01 * np.abs(ref)) + 1e-6)
