"""Pins of the sequential-chain oracle (oracle/chain.py) against things other than
itself: explicit Python loops, closed forms and the structural facts that define the
quantisation-exposed propagation of Sec. 3.2.1 (PassAct2) on the synthetic layer."""
import math

import numpy as np

from oracle import chain as och
from oracle import tlq_oracle as orc
from paper_2602_07899_amd import workloads as wl


def _brute_glue(Z, Zb, m_a, m_b, period, split):
    out = []
    for t, row in enumerate(Z):
        v = [float(a) for a in row]
        if Zb is not None:
            v = [a * float(b) for a, b in zip(v, Zb[t])]
        ms = sum(a * a for a in v) / len(v)
        inv = 1.0 / math.sqrt(ms + 1e-6)
        m = m_a if (t % period) < split else m_b
        out.append([a * inv * float(mc) for a, mc in zip(v, m)])
    return np.array(out)


def test_glue_matches_explicit_loops():
    g = np.random.default_rng(11)
    Z = g.standard_normal((13, 6)) * 3.0
    Zb = g.standard_normal((13, 6))
    m_a = g.uniform(0.5, 4.0, 6)
    m_b = g.uniform(5.0, 30.0, 6)
    for zb in (None, Zb):
        got = och.glue(Z, zb, m_a, m_b, period=5, split=3)
        want = _brute_glue(Z.tolist(), None if zb is None else zb.tolist(), m_a.tolist(), m_b.tolist(), 5, 3)
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=0)


def test_glue_closed_forms():
    g = np.random.default_rng(12)
    Z = g.standard_normal((24, 32)) * 7.0
    ones = np.ones(32)
    # unit multipliers: every row leaves with unit mean square (up to the 1e-6 inside the root)
    out = och.glue(Z, None, ones, ones, period=6, split=4)
    np.testing.assert_allclose((out * out).mean(axis=1), 1.0, rtol=1e-6)
    # a positive rescale of a row is removed by the normalisation
    out2 = och.glue(Z * 16.0, None, ones, ones, period=6, split=4)
    np.testing.assert_allclose(out2, out, rtol=1e-6)
    # a constant row of value v gives v/sqrt(v^2 + 1e-6) exactly
    c = och.glue(np.full((1, 8), 3.0), None, np.ones(8), np.ones(8), period=1, split=1)
    np.testing.assert_allclose(c, 3.0 / math.sqrt(9.0 + 1e-6), rtol=1e-15)
    # the eps sits inside the square root, added to the mean square: a zero row stays zero and finite
    z = och.glue(np.zeros((2, 8)), None, np.ones(8), np.ones(8), period=1, split=1)
    assert np.array_equal(z, np.zeros((2, 8)))
    tiny = och.glue(np.full((1, 4), 1e-4), None, np.ones(4), np.ones(4), period=1, split=1)
    np.testing.assert_allclose(tiny, 1e-4 / math.sqrt(1e-8 + 1e-6), rtol=1e-14)


def test_glue_visual_text_split():
    g = np.random.default_rng(13)
    period, split, n = 7, 5, 21
    Z = g.standard_normal((n, 10))
    m_vis = np.ones(10); m_vis[3] = 5.0
    m_txt = np.ones(10); m_txt[3] = 30.0
    base = och.glue(Z, None, np.ones(10), np.ones(10), period, split)
    out = och.glue(Z, None, m_vis, m_txt, period, split)
    pos = np.arange(n) % period
    vis, txt = pos < split, pos >= split
    # rows before `split` inside each sample take the first multiplier, the rest the second
    np.testing.assert_allclose(out[vis, 3], 5.0 * base[vis, 3], rtol=1e-15)
    np.testing.assert_allclose(out[txt, 3], 30.0 * base[txt, 3], rtol=1e-15)
    other = np.arange(10) != 3
    np.testing.assert_array_equal(out[:, other], base[:, other])
    # swapping the two multipliers must change the result (guards a swapped argument)
    swapped = och.glue(Z, None, m_txt, m_vis, period, split)
    assert not np.allclose(swapped, out)
    # the product branch normalises the PRODUCT, not each factor
    Zb = g.standard_normal((n, 10))
    prod = och.glue(Z, Zb, m_vis, m_txt, period, split)
    np.testing.assert_allclose(prod, och.glue(Z * Zb, None, m_vis, m_txt, period, split), rtol=1e-15)


def _mini():
    c = wl.CONFIGS["cfg3_mini_w3"]
    Ws = [wl.make_weight(c, li) for li in range(7)]
    X0 = wl.make_tokens(c, 0)
    w = wl.make_token_weights(c, 0)
    mults = [wl.chain_multipliers(c, li) for li in range(7)]
    return c, X0, Ws, w, mults


def test_run_chain_wiring():
    c, X0, Ws, w, mults = _mini()
    al = wl.alpha_grid(c.n_alpha)[:3]
    period, split = c.n_vis + c.n_txt, c.n_vis
    recs = och.run_chain(X0, Ws, w, c.bits, c.group, al, mults, period, split)
    assert len(recs) == 7
    # the first linear sees the given tokens; `up` sees exactly `gate`'s exposed input
    assert np.array_equal(recs[0]["X"], X0)
    assert recs[5]["X"] is recs[4]["X"] or np.array_equal(recs[5]["X"], recs[4]["X"])
    for li, r in enumerate(recs):
        W = Ws[li]
        assert r["X"].shape == (c.n_tok, W.shape[1]) and r["X"].dtype == np.float16
        # the target is the full-precision linear on the SAME exposed input (PassAct2 objective)
        np.testing.assert_array_equal(r["Y_ref"], (r["X"].astype(np.float64) @ W.astype(np.float64).T).astype(np.float16))
        # the recorded search is the search on that input and target
        again = orc.scale_search(r["X"], W, r["Y_ref"], w, c.bits, c.group, al)
        np.testing.assert_array_equal(again["losses"], r["res"]["losses"])
        assert again["best_idx"] == r["res"]["best_idx"]
        # Z is f_q of the chosen scales on the exposed input, rounded to storage
        _, _, _, deq = orc.fake_quant(W, r["res"]["best_scales"], c.bits, c.group)
        Zq = ((r["X"].astype(np.float64) / r["res"]["best_scales"].astype(np.float64)[None, :])
              @ deq.astype(np.float64).T).astype(np.float16)
        np.testing.assert_array_equal(r["Z"], Zq)
    # propagation: linear li (1..4) sees the glue of linear li-1's QUANTISED output, with ITS OWN multipliers
    for li in (1, 2, 3, 4):
        want = _brute_rows(recs[li - 1]["Z"], None, mults[li], period, split)
        np.testing.assert_array_equal(recs[li]["X"][ROWS], want)
    # down sees the glue of the product of the two quantised MLP branches
    want = _brute_rows(recs[4]["Z"], recs[5]["Z"], mults[6], period, split)
    np.testing.assert_array_equal(recs[6]["X"][ROWS], want)
    # and not of the full-precision outputs: quantisation must be visible downstream
    fp_next = och.glue(recs[0]["Y_ref"], None, mults[1][0], mults[1][1], period, split).astype(np.float16)
    assert not np.array_equal(fp_next, recs[1]["X"])


ROWS = np.array([0, 1, 95, 96, 127, 128, 500, 639])


def _brute_rows(Z, Zb, mult, period, split):
    Zs = Z[ROWS].astype(np.float64)
    out = np.empty_like(Zs)
    for i, t in enumerate(ROWS):
        v = Zs[i] if Zb is None else Zs[i] * Zb[t].astype(np.float64)
        m = mult[0] if (t % period) < split else mult[1]
        out[i] = v / math.sqrt(float((v * v).sum()) / v.size + 1e-6) * m.astype(np.float64)
    return out.astype(np.float16)


def test_run_chain_with_identity_quantiser_reproduces_fp_chain():
    """With 8 bits the quantiser is close to the identity: every exposed input of the chain
    must then agree with the full-precision chain (same glue, no quantiser) to a few
    storage ulps, and every loss must be tiny against the energy of the target."""
    c, X0, Ws, w, mults = _mini()
    period, split = c.n_vis + c.n_txt, c.n_vis
    al = wl.alpha_grid(c.n_alpha)[:2]
    recs = och.run_chain(X0, Ws, w, 8, c.group, al, mults, period, split)
    X = X0
    outs = {}
    for li in range(7):
        if li == 5:
            X = Xg
        elif li == 6:
            X = och.glue(outs[4], outs[5], mults[6][0], mults[6][1], period, split).astype(np.float16)
        elif li > 0:
            X = och.glue(outs[li - 1], None, mults[li][0], mults[li][1], period, split).astype(np.float16)
        if li == 4:
            Xg = X
        outs[li] = (X.astype(np.float64) @ Ws[li].astype(np.float64).T).astype(np.float16)
        a, b = recs[li]["X"].astype(np.float64), X.astype(np.float64)
        assert np.linalg.norm(a - b) <= 2e-2 * np.linalg.norm(b), li
        energy = float((w.astype(np.float64) * (recs[li]["Y_ref"].astype(np.float64) ** 2).mean(axis=1)).sum())
        assert recs[li]["res"]["losses"].min() < 1e-3 * energy, li
