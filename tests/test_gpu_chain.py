"""Quantisation-exposed sequential calibration (PassAct2 chain, W3) on the GPU
against the oracle chain.  Per linear, both sides get the ORACLE's exposed
input (so a one-ulp difference upstream cannot hide or fake a mismatch); the
free-running GPU chain is then checked against the same oracle records."""
import numpy as np
import pytest

from oracle import chain as ochain
from oracle import tlq_oracle as orc
from paper_2602_07899_amd import chain as gchain
from paper_2602_07899_amd import tlq
from paper_2602_07899_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _setup(gpu):
    import torch
    c = wl.CONFIGS["cfg3_mini_w3"]
    X0 = wl.make_tokens(c, 0)
    Ws = [wl.make_weight(c, li) for li in range(7)]
    w = wl.make_token_weights(c, 0)
    al = wl.alpha_grid(c.n_alpha)
    mults = [wl.chain_multipliers(c, li) for li in range(7)]
    period, split = c.n_vis + c.n_txt, c.n_vis
    recs = ochain.run_chain(X0, Ws, w, c.bits, c.group, al, mults, period, split)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu)
    return c, X0, Ws, w, al, mults, period, split, recs, t


def test_chain_teacher_forced_parity(gpu):
    import torch
    c, X0, Ws, w, al, mults, period, split, recs, t = _setup(gpu)
    p = tlq.params(bits=c.bits, group=c.group)
    for li, (W, r) in enumerate(zip(Ws, recs)):
        X, Y = r["X"], r["Y_ref"]
        co, ci = W.shape
        best = torch.empty(ci, dtype=torch.float32, device=gpu)
        idx = torch.empty(1, dtype=torch.int32, device=gpu)
        losses = torch.empty(al.size, dtype=torch.float32, device=gpu)
        tlq.scale_search(t(X), t(W), t(Y), t(w), t(al), p, best, idx, losses)
        gl, ol = losses.cpu().numpy().astype(np.float64), r["res"]["losses"]
        rel = np.abs(gl - ol) / ol
        assert rel.max() < 1e-3, (li, rel.max())
        gi, oi = int(idx.item()), r["res"]["best_idx"]
        if gi != oi:
            srt = np.sort(ol)
            assert (srt[1] - srt[0]) / srt[0] < 1e-3
        # S6 with the oracle's chosen scales: quantised output to storage precision
        Zg = torch.empty((X.shape[0], co), dtype=torch.float16, device=gpu)
        tlq.apply_best(t(X), t(W), t(r["res"]["best_scales"]), p, Zg)
        zd = orc.apply_best(X, W, r["res"]["best_scales"], c.bits, c.group)
        _, _, _, deq = orc.fake_quant(W, r["res"]["best_scales"], c.bits, c.group)
        mag = np.abs(X.astype(np.float64) / r["res"]["best_scales"]) @ np.abs(deq.astype(np.float64)).T
        err = np.abs(Zg.cpu().numpy().astype(np.float64) - zd)
        assert np.all(err <= 2.0 ** -11 * (0.6 * mag + 1.01 * np.abs(zd)) + 1e-6), li
        # glue of the next stage on the oracle's quantised outputs
        if li in (0, 1, 2, 3, 5):
            nxt = li + 1
            Zb = t(recs[4]["Z"]) if nxt == 6 else None
            Za = t(recs[5]["Z"]) if nxt == 6 else t(r["Z"])
            out = torch.empty((X.shape[0], Ws[nxt].shape[1]), dtype=torch.float16, device=gpu)
            tlq.rmsnorm_mul(Za, p, out, Zb=Zb, m_a=t(mults[nxt][0]), m_b=t(mults[nxt][1]), period=period,
                            split=split)
            exp = ochain.glue(recs[5]["Z"] if nxt == 6 else r["Z"], recs[4]["Z"] if nxt == 6 else None,
                              mults[nxt][0], mults[nxt][1], period, split)
            got = out.cpu().numpy().astype(np.float64)
            assert np.all(np.abs(got - exp) <= 2.0 ** -10 * np.abs(exp) + 1e-6), li
        print(f"linear {li}: max rel loss error {rel.max():.2e}, best {gi} (oracle {oi})")


def test_chain_free_running(gpu):
    c, X0, Ws, w, al, mults, period, split, recs, t = _setup(gpu)
    p = tlq.params(bits=c.bits, group=c.group)
    g = gchain.run_chain(t(X0), [t(W) for W in Ws], t(w), t(al), p,
                         [(t(a), t(b)) for a, b in mults], period, split, keep=True)
    same_so_far = True
    for li, (gr, r) in enumerate(zip(g, recs)):
        ol = r["res"]["losses"]
        gl = gr["losses"].cpu().numpy().astype(np.float64)
        gi, oi = int(gr["best_idx"].item()), r["res"]["best_idx"]
        x = gr["X"].cpu().numpy().astype(np.float64)
        xo = r["X"].astype(np.float64)
        assert np.isfinite(x).all() and np.isfinite(gl).all() and gi == int(np.argmin(gl))
        relx = np.linalg.norm(x - xo) / np.linalg.norm(xo)
        rell = float(np.max(np.abs(gl - ol) / ol))
        print(f"linear {li}: best {gi} (oracle {oi}), |dX|/|X| {relx:.2e}, max rel loss diff {rell:.2e}")
        if same_so_far:
            # until a (near-tied) choice differs upstream, the exposed inputs differ only by
            # storage rounding and the few quantisation codes it can flip
            assert relx < 2e-2 and rell < 5e-2, li
        if gi != oi:
            srt = np.sort(ol)
            assert (srt[1] - srt[0]) / srt[0] < 5e-2, (li, gi, oi)
            same_so_far = False


def test_chain_full_size_7b_w3(gpu):
    """The 7B-class chain at its real size (64 x 640 = 40,960 tokens, W3 g128, 20
    alphas).  A full oracle is out of reach, so (a) what holds at any size is checked -
    finite positive losses, first-minimum selection, normalised exposed inputs, the
    search's alpha = 0 loss equal to plain round-to-nearest evaluated through the two
    single-purpose entry points - and (b) for two late linears (o_proj after three
    quantised predecessors, down_proj at the end of the chain) the oracle evaluates 56
    sampled tokens of the exposed input the chain actually produced: scale table from the
    oracle's own statistic of that input, per-token errors of three candidates, and the
    chain's recorded losses tied to the entry point that produced those errors."""
    import torch
    c = wl.CONFIGS["cfg3_7b_w3"]
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu)
    X0 = t(wl.make_tokens(c, 0))
    Ws = [t(wl.make_weight(c, li)) for li in range(7)]
    w = t(wl.make_token_weights(c, 0))
    al = t(wl.alpha_grid(c.n_alpha))
    mults = [tuple(t(m) for m in wl.chain_multipliers(c, li)) for li in range(7)]
    p = tlq.params(bits=c.bits, group=c.group)
    period, split = c.n_vis + c.n_txt, c.n_vis
    g = gchain.run_chain(X0, Ws, w, al, p, mults, period, split, keep=True)
    torch.cuda.synchronize()
    for li, r in enumerate(g):
        L = r["losses"].cpu().numpy()
        assert np.all(np.isfinite(L)) and np.all(L > 0), li
        assert int(r["best_idx"].item()) == int(np.argmin(L)), li
        assert torch.isfinite(r["Z"].float()).all()
        if li > 0 and li != 5:
            # rows of a glued input have unit mean square before the outlier multipliers
            X = r["X"][:2048].float()
            mv, mt = mults[li]
            rows = torch.arange(2048, device=gpu) % period
            m = torch.where((rows < split)[:, None], mv[None, :], mt[None, :])
            ms = ((X / m) ** 2).mean(dim=1)
            assert torch.all((ms - 1).abs() < 2e-2), li
        print(f"linear {li}: best alpha index {int(r['best_idx'].item())}, loss range "
              f"{L.min():.3e} .. {L.max():.3e}")
    # alpha = 0 is plain RTN: fake_quant (unit scales) -> weighted_layer_err on the same exposed input
    r = g[3]
    W = Ws[3]
    wdq = torch.empty_like(W)
    tlq.fake_quant(W, None, p, Wdq=wdq)
    Y = torch.empty((X0.shape[0], W.shape[0]), dtype=torch.float16, device=gpu)
    tlq.ref_output(r["X"], W, Y, p)
    loss = torch.empty(1, dtype=torch.float32, device=gpu)
    tlq.weighted_layer_err(r["X"], wdq, None, Y, w, p, loss)
    assert loss.item() == r["losses"][0].item()
    # (b) sampled-token parity against the oracle on the exposed inputs of o_proj and down_proj
    wh = wl.make_token_weights(c, 0)
    alh = wl.alpha_grid(c.n_alpha)
    for li in (3, 6):
        r, W = g[li], Ws[li]
        Wh = W.cpu().numpy()
        n_tok, c_in = r["X"].shape
        xsum = np.zeros(c_in, np.float64)
        for i in range(0, n_tok, 8192):       # the oracle's x_stat of the exposed input, streamed
            xsum += np.abs(r["X"][i:i + 8192].cpu().numpy().astype(np.float64)).sum(axis=0)
        ost = orc.scale_table((xsum / n_tok).astype(np.float32), alh)
        st = torch.empty((c.n_alpha, c_in), dtype=torch.float32, device=gpu)
        xs = torch.empty(c_in, dtype=torch.float32, device=gpu)
        tlq.x_stat(r["X"], p, xs)
        tlq.scale_table(xs, al, st)
        ulp = np.abs(st.cpu().numpy().view(np.int32).astype(np.int64) - ost.view(np.int32))
        assert ulp.max() <= 1, li
        Y = torch.empty((n_tok, W.shape[0]), dtype=torch.float16, device=gpu)
        tlq.ref_output(r["X"], W, Y, p)
        rows = np.sort(np.random.default_rng(30 + li).choice(n_tok, 56, replace=False))
        trows = torch.from_numpy(rows).to(gpu)
        Xr, Yr = r["X"][trows].cpu().numpy(), Y[trows].cpu().numpy()
        Yo = orc.ref_output(Xr, Wh)
        assert np.all(np.abs(Yr.astype(np.float64) - Yo) <= 2.0 ** -10 * np.abs(Yo) + 1e-4), li
        wdq = torch.empty_like(W)
        pte = torch.empty(n_tok, dtype=torch.float32, device=gpu)
        L = r["losses"].cpu().numpy().astype(np.float64)
        bi = int(r["best_idx"].item())
        for k in sorted({0, bi, 19}):
            tlq.fake_quant(W, t(ost[k]), p, Wdq=wdq)
            inv = (1.0 / ost[k].astype(np.float64)).astype(np.float32)
            tlq.weighted_layer_err(r["X"], wdq, t(inv), Y, w, p, loss, pte)
            _, _, _, deq = orc.fake_quant(Wh, ost[k], c.bits, c.group)
            e = orc.per_token_err(Yr, orc.quantised_output(Xr, deq.astype(np.float16), inv_s=inv))
            np.testing.assert_allclose(pte[trows].cpu().numpy(), e, rtol=1e-3)
            e_pure = orc.per_token_err(Yr, orc.quantised_output(Xr, deq, s=ost[k]))
            np.testing.assert_allclose(pte[trows].cpu().numpy(), e_pure, rtol=2e-3)
            assert abs(loss.item() - L[k]) / L[k] < 2e-4, (li, k)
        # the quantised output the chain propagated = f_q of the chosen scales on those rows
        zo = orc.apply_best(Xr, Wh, r["best_scales"].cpu().numpy(), c.bits, c.group)
        zg = r["Z"][trows].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(zg - zo) <= 2.0 ** -9 * np.abs(zo) + 2e-3 * np.abs(zo).mean()), li
        print(f"linear {li}: sampled-token parity on the exposed input ok (best {bi})")
