"""Pins for the CPU oracle: everything here runs without a GPU.

Each test ties the oracle to something other than itself: a hand-worked
example (tests/golden), brute force on tiny layers, closed forms, invariants
that the paper's equations imply, or a library routine the definition
reduces to.  A companion test plants typical mistakes in copies of the
definition and checks that the pins would catch them.
"""
import json
import os

import numpy as np
import pytest

from oracle import brute
from oracle import tlq_oracle as orc
from paper_2602_07899_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _load_hand():
    with open(os.path.join(GOLD, "hand_worked_w2_g4.json")) as f:
        return json.load(f)


# ---------------------------------------------------------------- golden
def test_hand_worked_example():
    g = _load_hand()
    X = np.array(g["X"], np.float16)
    W = np.array(g["W"], np.float16)
    w = np.array(g["token_w"], np.float32)
    al = np.array(g["alpha_grid"], np.float32)
    xs = orc.x_stat_mean(X)
    assert xs.tolist() == g["x_stat"]
    Y = orc.ref_output(X, W)
    assert Y.tolist() == g["Y_ref"]
    st = orc.scale_table(xs, al)
    for k, cand in enumerate(g["candidates"]):
        assert st[k].tolist() == cand["s"]
        codes, zp, delta, deq = orc.fake_quant(W, st[k], g["bits"], g["group"])
        assert codes.tolist() == cand["codes"]
        assert zp.tolist() == cand["zp"]
        assert delta.tolist() == cand["delta"]
        assert deq.tolist() == cand["deq"]
        L, e = orc.weighted_layer_err(X, deq, Y, w, s=st[k])
        assert e.tolist() == cand["per_token_err"]
        assert L == cand["loss"]
    res = orc.scale_search(X, W, Y, w, g["bits"], g["group"], al)
    assert res["best_idx"] == g["best_idx"]
    assert res["losses"].tolist() == [c["loss"] for c in g["candidates"]]
    assert res["best_scales"].tolist() == g["candidates"][g["best_idx"]]["s"]


# ------------------------------------------------------------ brute force
@pytest.mark.parametrize("seed,n,ci,co,bits,group", [
    (1, 5, 8, 3, 4, 4), (2, 7, 8, 6, 3, 2), (3, 4, 6, 5, 2, 2), (4, 8, 8, 8, 4, 0),
    (5, 3, 4, 7, 3, 4),
])
def test_brute_force_tiny(seed, n, ci, co, bits, group):
    X, W, w = wl.tiny_layer(seed, n, ci, co)
    Y = orc.ref_output(X, W).astype(np.float32)  # rounded once, same array to both
    alphas = [0.0, 0.25, 0.5, 0.8]
    xs_b, losses_b, best_b = brute.brute_search(X.tolist(), W.tolist(), Y.tolist(), w.tolist(),
                                                bits, group, alphas)
    res = orc.scale_search(X, W, Y, w, bits, group, np.array(alphas, np.float32))
    assert [float(v) for v in xs_b] == res["x_stat"].tolist()
    np.testing.assert_allclose(res["losses"], losses_b, rtol=1e-12, atol=0)
    assert res["best_idx"] == best_b
    # codes / zero points / steps, candidate by candidate
    for k, a in enumerate(alphas):
        s_b = brute.brute_scale(xs_b, a)
        assert [float(v) for v in s_b] == res["s_table"][k].tolist()
        codes, zp, delta, deq = orc.fake_quant(W, res["s_table"][k], bits, group)
        for o in range(co):
            cb, zb, db, qb = brute.brute_fake_quant_row(W[o].tolist(), s_b, bits, group)
            assert cb == codes[o].tolist()
            assert zb == zp[o].tolist()
            assert [float(v) for v in db] == delta[o].tolist()
            assert [float(v) for v in qb] == deq[o].tolist()


# ------------------------------------------------------- scale closed forms
def test_alpha_zero_unit_scales_and_alpha_one_identity():
    X = wl.make_tokens(wl.CONFIGS["cfg1_small"], 0)
    xs = orc.x_stat_mean(X)
    st = orc.scale_table(xs, np.array([0.0, 1.0], np.float32))
    assert np.all(st[0] == np.float32(1.0))
    assert np.array_equal(st[1], np.maximum(xs, np.float32(2.0 ** -14)))
    # dead channel: floored, finite, alpha=0 still exactly one
    st0 = orc.scale_table(np.array([0.0, 1.0], np.float32), np.array([0.0, 0.5], np.float32))
    assert st0[0].tolist() == [1.0, 1.0]
    assert st0[1].tolist() == [2.0 ** -7, 1.0]


def test_scale_monotone_in_alpha():
    xs = np.array([0.01, 0.5, 1.0, 3.0, 40.0], np.float32)
    st = orc.scale_table(xs, wl.alpha_grid(20)).astype(np.float64)
    d = np.diff(st, axis=0)
    assert np.all(d[:, xs > 1] > 0) and np.all(d[:, xs < 1] < 0) and np.all(d[:, xs == 1] == 0)


def test_x_stat_reduces_to_library_mean():
    X = wl.make_tokens(wl.CONFIGS["cfg1_small"], 0)
    ref = np.mean(np.abs(X.astype(np.float64)), axis=0)
    np.testing.assert_allclose(orc.x_stat_mean(X).astype(np.float64), ref, rtol=2 ** -24)
    # exactness claim: fp16 magnitudes sum exactly in float64 -> order independent
    perm = np.random.default_rng(0).permutation(X.shape[0])
    assert np.array_equal(orc.x_stat_mean(X), orc.x_stat_mean(X[perm]))


# ------------------------------------------------------------- quantiser
def _gauss_w(c_out=64, c_in=512, seed=0):
    return (np.random.default_rng(seed).standard_normal((c_out, c_in)) * 0.02).astype(np.float16)


@pytest.mark.parametrize("bits", [3, 4, 8])
def test_quantiser_grid_properties(bits):
    W = _gauss_w()
    s = (np.random.default_rng(1).uniform(0.5, 4.0, W.shape[1])).astype(np.float32)
    codes, zp, delta, deq = orc.fake_quant(W, s, bits, 128)
    qmax = 2 ** bits - 1
    ws = (W.astype(np.float32) * s[None, :]).reshape(W.shape[0], -1, 128)
    # every random Gaussian group straddles zero: min -> code 0, max -> code qmax
    c3 = codes.reshape(ws.shape)
    assert np.all(np.take_along_axis(c3, ws.argmin(2)[..., None], 2) == 0)
    assert np.all(np.take_along_axis(c3, ws.argmax(2)[..., None], 2) == qmax)
    # round-to-nearest: error at most half a step
    err = np.abs(ws.astype(np.float64) - deq.reshape(ws.shape).astype(np.float64))
    assert np.all(err <= 0.5 * delta[..., None].astype(np.float64) * (1 + 1e-5))
    # idempotent on its own grid
    again = orc.requantise_on_grid(deq, delta, zp, bits, 128)
    assert np.array_equal(again, codes)
    assert codes.dtype == np.uint8 and codes.max() <= qmax


def test_rounding_error_energy_is_delta_sq_over_12():
    # Sec. 2.2: uniform rounding error, variance Delta^2/12
    W = _gauss_w(256, 1024, seed=3)
    codes, zp, delta, deq = orc.fake_quant(W, None, 4, 128)
    err2 = ((W.astype(np.float64) - deq.astype(np.float64)) ** 2).mean()
    pred = (delta.astype(np.float64) ** 2).mean() / 12.0
    assert abs(err2 / pred - 1.0) < 0.05


def test_power_of_two_scale_invariance():
    W = _gauss_w()
    s = (np.random.default_rng(2).uniform(0.5, 4.0, W.shape[1])).astype(np.float32)
    c1, z1, d1, q1 = orc.fake_quant(W, s, 4, 128)
    c2, z2, d2, q2 = orc.fake_quant(W, s * np.float32(8.0), 4, 128)
    assert np.array_equal(c1, c2) and np.array_equal(z1, z2)
    assert np.array_equal(d1 * np.float32(8.0), d2)
    assert np.array_equal(q1 * np.float32(8.0), q2)


def test_constant_and_same_sign_groups():
    # constant group: range floored, everything maps to one code, deq == value up to delta
    W = np.full((1, 8), 0.5, np.float16)
    codes, zp, delta, deq = orc.fake_quant(W, None, 4, 8)
    assert delta[0, 0] == np.float32(1e-5) / np.float32(15)
    assert len(set(codes[0].tolist())) == 1
    # all-positive group: zero point saturates at 0 and small values clip at code 0
    W = np.array([[1.0, 2.0, 3.0, 4.0]], np.float16)
    codes, zp, delta, deq = orc.fake_quant(W, None, 2, 4)
    assert zp[0, 0] == 0 and delta[0, 0] == 1.0
    assert codes[0].tolist() == [1, 2, 3, 3] and deq[0].tolist() == [1.0, 2.0, 3.0, 3.0]


def test_symmetric_variant_closed_form():
    # Sec. 2.2: s_i = max|x| / (2^(n-1) - 1): the row maximum lands on the top code
    W = _gauss_w(16, 256, seed=5)
    for bits in (4, 8):
        codes, zp, delta, deq = orc.fake_quant(W, None, bits, 0, symmetric=True)
        half = 2 ** (bits - 1)
        am = np.abs(W.astype(np.float32)).max(axis=1)
        assert np.array_equal(delta[:, 0], am / np.float32(half - 1))
        q = codes.astype(np.int32) - half
        assert np.all(np.abs(q).max(axis=1) == half - 1)
        assert q.min() >= -half and q.max() <= half - 1
        idx = np.abs(W.astype(np.float32)).argmax(axis=1)
        np.testing.assert_allclose(np.abs(deq[np.arange(16), idx]), am, rtol=1e-6)


# ------------------------------------------------------- contraction / loss
def _cfg1():
    c = wl.CONFIGS["cfg1_small"]
    X = wl.make_tokens(c, 0)
    W = wl.make_weight(c, 0)
    w = wl.make_token_weights(c, 0)
    return c, X, W, w


def test_smoothing_identity_without_quantisation():
    # Sec. 2.2 smoothing equation: exact when nothing is quantised
    c, X, W, w = _cfg1()
    Y = orc.ref_output(X, W)
    st = orc.scale_table(orc.x_stat_mean(X), wl.alpha_grid(20))
    for k in (0, 7, 19):
        ws = W.astype(np.float64) * st[k].astype(np.float64)[None, :]
        L, e = orc.weighted_layer_err(X, ws, Y, w, s=st[k])
        assert L < 1e-24 * float((Y ** 2).mean()) or L < 1e-26


def test_uniform_weights_reduce_to_mse_and_library_matmul():
    c, X, W, w = _cfg1()
    Y = orc.ref_output(X, W)
    s = orc.scale_table(orc.x_stat_mean(X), np.array([0.5], np.float32))[0]
    _, _, _, deq = orc.fake_quant(W, s, 4, 128)
    n = X.shape[0]
    L, e = orc.weighted_layer_err(X, deq, Y, np.full(n, 1.0 / n), s=s)
    # independent evaluation through einsum on explicitly scaled operands
    Xs = X.astype(np.float64) / s.astype(np.float64)
    Yq = np.einsum("tc,oc->to", Xs, deq.astype(np.float64))
    np.testing.assert_allclose(L, np.mean((Y - Yq) ** 2), rtol=1e-12)
    # not transposed: a non-square problem has the right output shape
    Xr, Wr, wr = wl.tiny_layer(11, 5, 8, 3)
    assert orc.quantised_output(Xr, Wr.astype(np.float32)).shape == (5, 3)
    np.testing.assert_allclose(orc.ref_output(Xr, Wr),
                               np.einsum("tc,oc->to", Xr.astype(np.float64), Wr.astype(np.float64)),
                               rtol=1e-13, atol=1e-15)


def test_loss_linear_in_token_weights_and_one_hot():
    c, X, W, w = _cfg1()
    Y = orc.ref_output(X, W)
    _, _, _, deq = orc.fake_quant(W, None, 4, 128)
    rng = np.random.default_rng(7)
    w1, w2 = rng.uniform(0, 1, X.shape[0]), rng.uniform(0, 1, X.shape[0])
    L1, e = orc.weighted_layer_err(X, deq, Y, w1)
    L2, _ = orc.weighted_layer_err(X, deq, Y, w2)
    L12, _ = orc.weighted_layer_err(X, deq, Y, w1 + w2)
    np.testing.assert_allclose(L12, L1 + L2, rtol=1e-12)
    hot = np.zeros(X.shape[0]); hot[17] = 1.0
    Lh, _ = orc.weighted_layer_err(X, deq, Y, hot)
    assert Lh == e[17]
    # that token's error from first principles
    d = Y[17] - X[17].astype(np.float64) @ deq.astype(np.float64).T
    np.testing.assert_allclose(e[17], (d ** 2).mean(), rtol=1e-12)


def test_inv_s_and_s_agree():
    c, X, W, w = _cfg1()
    Y = orc.ref_output(X, W)
    s = np.exp2(np.random.default_rng(3).integers(-2, 3, X.shape[1])).astype(np.float32)
    _, _, _, deq = orc.fake_quant(W, s, 4, 128)
    La, _ = orc.weighted_layer_err(X, deq, Y, w, s=s)
    Lb, _ = orc.weighted_layer_err(X, deq, Y, w, inv_s=(1.0 / s).astype(np.float32))
    assert La == Lb  # powers of two: both forms exact


def test_search_alpha0_is_plain_rtn_and_selects_first_minimum():
    c, X, W, w = _cfg1()
    Y = orc.ref_output(X, W)
    res = orc.scale_search(X, W, Y, w, 4, 128, wl.alpha_grid(20))
    _, _, _, deq = orc.fake_quant(W, None, 4, 128)
    L0, _ = orc.weighted_layer_err(X, deq, Y, w)
    assert res["losses"][0] == L0
    assert res["best_idx"] == int(np.argmin(res["losses"]))
    # outlier channels make smoothing pay off: some alpha > 0 must beat RTN
    assert res["best_idx"] > 0 and res["losses"][res["best_idx"]] < L0
    assert np.array_equal(res["best_scales"], res["s_table"][res["best_idx"]])
    # selection rules
    assert orc.select_best([3.0, 1.0, 1.0, 2.0]) == 1
    assert orc.select_best([np.inf, np.nan, 5.0]) == 2
    assert orc.select_best([np.nan, np.inf]) == -1


def test_apply_best_is_fq_output():
    # PassAct2: next input equals the quantised layer's output for the chosen scale
    X, W, w = wl.tiny_layer(21, 6, 8, 4)
    s = np.array([2, 1, 0.5, 1, 4, 1, 1, 2], np.float32)
    out = orc.apply_best(X, W, s, 4, 4)
    _, _, _, deq = orc.fake_quant(W, s, 4, 4)
    exp = np.zeros((6, 4))
    for t in range(6):
        for o in range(4):
            exp[t, o] = sum(float(X[t, c]) / float(s[c]) * float(deq[o, c]) for c in range(8))
    np.testing.assert_allclose(out, exp, rtol=1e-13, atol=1e-15)


def test_bf16_rounding_helper():
    a = np.array([1.0, 1.00390625, 1.01171875, 3.0e-39, -2.5], np.float32)
    r = orc.round_to_bf16(a)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.015625) and r[4] == -2.5
    try:
        import torch
        t = torch.from_numpy(np.random.default_rng(0).standard_normal(4096).astype(np.float32))
        assert np.array_equal(orc.round_to_bf16(t.numpy()), t.to(torch.bfloat16).float().numpy())
    except ImportError:
        pass


# ---------------------------------------------- the pins catch planted mistakes
def test_pins_catch_planted_mistakes():
    """Plant typical mistakes in copies of the definition (on the CPU) and check
    that the hand-worked example tells them apart from the correct result."""
    g = _load_hand()
    X = np.array(g["X"], np.float64)
    W = np.array(g["W"], np.float32)
    w = np.array(g["token_w"], np.float64)
    Y = np.array(g["Y_ref"], np.float64)
    s = np.array(g["candidates"][1]["s"], np.float32)
    good = g["candidates"][1]["loss"]

    def loss(deq, xs):
        d = Y - xs @ deq.astype(np.float64).T
        return float((w * (d * d).mean(axis=1)).sum())

    def quant(ws, rnd=np.rint, zp_sign=-1.0, clip=True):
        mx, mn = ws.max(1, keepdims=True), ws.min(1, keepdims=True)
        delta = (mx - mn) / np.float32(3)
        zp = np.clip(rnd(zp_sign * mn / delta), 0, 3)
        q = rnd(ws / delta) + zp
        if clip:
            q = np.clip(q, 0, 3)
        return (q - zp) * delta

    xs_ok = X / s.astype(np.float64)
    assert loss(quant(W * s), xs_ok) == good                      # the copy itself is right
    assert loss(quant(W * s, rnd=lambda v: np.floor(v + 0.5)), xs_ok) != good   # half-up rounding
    assert loss(quant(W * s, zp_sign=1.0), xs_ok) != good          # wrong zero-point sign
    # no clipping: on this example the weighted loss happens to coincide, the
    # dequantised values (and the per-token errors) do not
    assert not np.array_equal(quant(W * s, clip=False), quant(W * s))
    assert quant(W * s).tolist() == g["candidates"][1]["deq"]
    assert loss(quant(W * s), X) != good                           # forgot to divide X by s
    assert loss(quant(W / s), xs_ok) != good                       # scaled W the wrong way
    assert loss(quant(W * s), X * s.astype(np.float64)) != good    # multiplied X instead
    d = Y - xs_ok @ quant(W * s).astype(np.float64).T
    assert float((w[::-1] * (d * d).mean(axis=1)).sum()) != good   # weights on wrong tokens
    assert float((w * (d * d).sum(axis=1)).sum()) != good          # dropped the 1/C_out


# ------------------------------------------------- activation quantisation (Q_a)
def test_act_quant_closed_forms():
    # Sec. 2.2: s_i = max_j |X_ij| / (2^(n-1) - 1), codes in [-2^(n-1), 2^(n-1) - 1]
    X = wl.make_tokens(wl.CONFIGS["cfg1_small"], 0)
    for bits in (8, 6, 4):
        half = 2 ** (bits - 1)
        codes, sigma = orc.act_quant(X, None, bits)
        am = np.abs(X.astype(np.float32)).max(axis=1)
        assert np.array_equal(sigma, am / np.float32(half - 1))
        assert codes.min() >= -half and codes.max() <= half - 1
        assert np.all(np.abs(codes).max(axis=1) == half - 1)        # the row maximum lands on the top code
        xhat = codes.astype(np.float64) * sigma.astype(np.float64)[:, None]
        assert np.all(np.abs(xhat - X.astype(np.float64)) <= 0.5 * sigma[:, None] * (1 + 1e-4))
        # idempotent: quantising the dequantised row again gives the same codes and step
        c2, s2 = orc.act_quant(xhat.astype(np.float32), None, bits)
        assert np.array_equal(c2, codes) and np.allclose(s2, sigma, rtol=1e-6)
    # int8 example worked by hand: row [1.27, -0.635, 0.0049, 0.02] -> step 0.01, codes 127, -64 (tie to even), 0, 2
    Xh = np.array([[1.27, -0.64, 0.0049, 0.02]], np.float32)
    c, sg = orc.act_quant(Xh, None, 8)
    assert np.isclose(sg[0], 0.01, rtol=1e-6) and c[0].tolist() == [127, -64, 0, 2]
    # a constant zero row takes the floored step and all-zero codes
    c, sg = orc.act_quant(np.zeros((1, 8), np.float32), None, 8)
    assert sg[0] == np.float32(1e-5) / np.float32(127) and not c.any()


@pytest.mark.parametrize("seed,n,ci,co,bits,group,abits", [(1, 5, 8, 3, 4, 4, 8), (2, 6, 8, 4, 3, 2, 6),
                                                          (3, 4, 4, 5, 4, 0, 4)])
def test_act_quant_search_matches_brute_force(seed, n, ci, co, bits, group, abits):
    X, W, w = wl.tiny_layer(seed, n, ci, co)
    Y = orc.ref_output(X, W).astype(np.float32)
    alphas = [0.0, 0.3, 0.6]
    res = orc.scale_search(X, W, Y, w, bits, group, np.array(alphas, np.float32), act_bits=abits)
    xs = brute.brute_x_stat(X.tolist())
    for k, a in enumerate(alphas):
        s_b = brute.brute_scale(xs, a)
        Lb = brute.brute_loss_aq(X.tolist(), W.tolist(), Y.tolist(), w.tolist(), s_b, bits, group, abits)
        np.testing.assert_allclose(res["losses"][k], Lb, rtol=1e-12)
        codes, sigma = orc.act_quant(X, orc.recip_scale(res["s_table"][k]), abits)
        for t in range(n):
            cb, sb = brute.brute_act_quant_row(X[t].tolist(), s_b, abits)
            assert cb == codes[t].tolist() and float(sb) == float(sigma[t])


def test_act_quant_limits():
    # many activation bits on a narrow row: Q_a is nearly the identity, so the loss approaches
    # the weight-only loss; and the activation error adds to it at low bits
    c = wl.CONFIGS["cfg1_small"]
    X, W, w = wl.make_tokens(c, 0), wl.make_weight(c, 0), wl.make_token_weights(c, 0)
    Y = orc.ref_output(X, W)
    al = np.array([0.0, 0.5], np.float32)
    base = orc.scale_search(X, W, Y, w, 4, 128, al)["losses"]
    a8 = orc.scale_search(X, W, Y, w, 4, 128, al, act_bits=8)["losses"]
    a4 = orc.scale_search(X, W, Y, w, 4, 128, al, act_bits=4)["losses"]
    assert np.all(a8 > base * 0.98) and np.all(a4 > a8)
    # smoothing (alpha = 0.5) shrinks the per-token range of the outlier rows: it helps A4 far more than A16
    assert a4[1] / a4[0] < base[1] / base[0]
    # exact representability: an integer-valued row whose max is 127 survives A8 unchanged
    Xi = np.random.default_rng(0).integers(-127, 128, (4, 16)).astype(np.float32)
    Xi[:, 0] = 127
    codes, sigma = orc.act_quant(Xi, None, 8)
    assert np.all(sigma == 1.0) and np.array_equal(codes, Xi.astype(np.int16))


# ------------------------------------------- gradient-guided token selection
def test_token_importance_and_topk_selection():
    rng = np.random.default_rng(4)
    B, N, C = 3, 10, 6
    G = rng.standard_normal((B * N, C)).astype(np.float32)
    s1 = orc.token_importance(G, B)
    s2 = orc.token_importance(G, B, l2=True)
    for n in range(N):                                  # written out from the definition
        a = sum(sum(abs(float(G[b * N + n, c])) for c in range(C)) / C for b in range(B))
        e = sum(sum(float(G[b * N + n, c]) ** 2 for c in range(C)) ** 0.5 for b in range(B))
        assert abs(s1[n] - a) < 1e-12 and abs(s2[n] - e) < 1e-12
    m = orc.top_fraction_mask(s1, N // 2)
    assert m.sum() == N // 2 and s1[m].min() >= s1[~m].max()
    assert orc.top_fraction_mask(np.array([1.0, 3.0, 3.0, 0.5]), 2).tolist() == [False, True, True, False]
    assert orc.top_fraction_mask(np.array([2.0, 2.0, 2.0, 2.0]), 2).tolist() == [True, True, False, False]
    # masked channel maximum over the selected positions of every sample
    X = rng.standard_normal((B * N, C)).astype(np.float16)
    xs = orc.x_stat_topk_max(X, m)
    ref = np.zeros(C)
    for r in range(B * N):
        if m[r % N]:
            ref = np.maximum(ref, np.abs(X[r].astype(np.float64)))
    assert np.array_equal(xs, ref.astype(np.float32))
    assert np.array_equal(orc.x_stat_topk_max(X, np.ones(N, bool)), orc.x_stat_max(X))


# ------------------------------------------- brute force, randomised shapes
def test_brute_force_random_tiny_layers():
    """The fixed brute-force cases above, widened: random tiny shapes, group sizes, bit widths,
    outlier strengths and alpha grids (hypothesis, derandomised), oracle against the pure-Python
    loops - losses to 1e-12, codes, zero points and steps exactly."""
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=60, deadline=None, derandomize=True)
    @given(seed=st.integers(0, 10_000), n=st.integers(1, 6), groups=st.integers(1, 3), g=st.sampled_from([2, 4]),
           co=st.integers(1, 5), bits=st.integers(2, 5), whole_row=st.booleans(), mult=st.sampled_from([1.0, 8.0, 60.0]),
           abits=st.sampled_from([0, 0, 2, 4, 8]))
    def run(seed, n, groups, g, co, bits, whole_row, mult, abits):
        ci = g * groups
        X, W, w = wl.tiny_layer(seed, n, ci, co, mult=mult)
        Y = orc.ref_output(X, W).astype(np.float32)
        group = 0 if whole_row else g
        alphas = [0.0, 0.3, 0.65, 0.95]
        res = orc.scale_search(X, W, Y, w, bits, group, np.array(alphas, np.float32), act_bits=abits)
        xs_b = brute.brute_x_stat(X.tolist())
        assert [float(v) for v in xs_b] == res["x_stat"].tolist()
        for k, a in enumerate(alphas):
            s_b = brute.brute_scale(xs_b, a)
            assert [float(v) for v in s_b] == res["s_table"][k].tolist()
            if abits:
                Lb = brute.brute_loss_aq(X.tolist(), W.tolist(), Y.tolist(), w.tolist(), s_b, bits, group, abits)
            else:
                Lb = brute.brute_loss(X.tolist(), W.tolist(), Y.tolist(), w.tolist(), s_b, bits, group)
            assert abs(res["losses"][k] - Lb) <= 1e-12 * abs(Lb) + 1e-300
            codes, zp, delta, deq = orc.fake_quant(W, res["s_table"][k], bits, group)
            for o in range(co):
                cb, zb, db, qb = brute.brute_fake_quant_row(W[o].tolist(), s_b, bits, group)
                assert cb == codes[o].tolist() and zb == zp[o].tolist()
                assert [float(v) for v in db] == delta[o].tolist()
        assert res["best_idx"] == int(np.argmin(res["losses"]))

    run()


def test_token_second_moment_pins():
    """The second-moment matrix against what fixes it: explicit loops on a tiny case, symmetry and
    positive semi-definiteness, the closed form for one-hot tokens, and the identity that ties it
    to the (brute-force pinned) weighted layer error - the loss of f_q(x) = What x against
    f_fp(x) = W x is the quadratic form of W - What in it."""
    rng = np.random.default_rng(11)
    n, ci, co = 13, 6, 5
    X = rng.standard_normal((n, ci)).astype(np.float16)
    w = rng.uniform(0.1, 1.0, n)
    w = (w / w.sum()).astype(np.float32)
    G = orc.token_second_moment(X, w)
    loops = np.zeros((ci, ci))
    for t in range(n):
        for i in range(ci):
            for j in range(ci):
                loops[i, j] += float(w[t]) * float(X[t, i]) * float(X[t, j])
    np.testing.assert_allclose(G, loops, rtol=1e-13, atol=1e-15)
    assert np.array_equal(G, G.T) or np.allclose(G, G.T, rtol=1e-15)
    assert np.linalg.eigvalsh(G).min() > -1e-12
    np.testing.assert_allclose(orc.token_second_moment(X, w, rows=[4, 1], cols=[0, 5, 2]), G[np.ix_([4, 1], [0, 5, 2])],
                               rtol=1e-13)
    # one-hot tokens: G is diagonal with the weight mass of each channel
    E = np.eye(ci, dtype=np.float16)[rng.integers(0, ci, n)]
    Gd = orc.token_second_moment(E, w)
    want = np.zeros(ci)
    for t in range(n):
        want[int(np.argmax(E[t]))] += float(w[t])
    np.testing.assert_allclose(Gd, np.diag(want), rtol=1e-13, atol=0)
    # quadratic-form identity with the layer error (asymmetric in rows/columns and in the sign of
    # the difference's cross terms, so a transposed or mis-weighted G fails it)
    W = (rng.standard_normal((co, ci)) * 0.05).astype(np.float16)
    s = orc.scale_table(orc.x_stat_mean(X), np.array([0.45], np.float32))[0]
    _, _, _, deq = orc.fake_quant(W.astype(np.float32), s, 3, 2)
    L, _ = orc.weighted_layer_err(X, deq, orc.ref_output(X, W), w, s=s)
    D = W.astype(np.float64) - deq.astype(np.float64) / s.astype(np.float64)
    np.testing.assert_allclose(np.einsum("oi,ij,oj->", D, G, D) / co, L, rtol=1e-11)
    # and it does not hold for the transposed weighting (rows weighted instead of tokens)
    Gbad = (X.astype(np.float64).T @ X.astype(np.float64)) / n
    assert abs(np.einsum("oi,ij,oj->", D, Gbad, D) / co - L) > 1e-6 * L
