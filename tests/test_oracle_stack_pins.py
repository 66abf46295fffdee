"""Pins of the decoder-stack oracle (oracle/stack.py) against things other than
itself: brute-force loops, closed forms, library routines and the structural
facts that define the three propagation modes of Sec. 3.2.1."""
import math

import numpy as np
import scipy.special

from oracle import stack as ost
from oracle import tlq_oracle as orc

F16 = lambda a: np.asarray(a, np.float64).astype(np.float16)


def _brute_attention(q, k, v, n_heads, seq_len):
    n, width = len(q), len(q[0])
    dh = width // n_heads
    out = [[0.0] * width for _ in range(n)]
    for t in range(n):
        b0 = (t // seq_len) * seq_len
        for h in range(n_heads):
            cs = range(h * dh, (h + 1) * dh)
            sc = [sum(q[t][c] * k[j][c] for c in cs) / math.sqrt(dh) for j in range(b0, t + 1)]
            m = max(sc)
            e = [math.exp(x - m) for x in sc]
            z = sum(e)
            for c in cs:
                out[t][c] = sum(e[j - b0] * v[j][c] for j in range(b0, t + 1)) / z
    return np.array(out)


def test_attention_matches_brute_force():
    g = np.random.default_rng(3)
    q, k, v = (g.standard_normal((10, 6)) * 2.0 for _ in range(3))
    got = ost.causal_attention(q, k, v, n_heads=2, seq_len=5)
    want = _brute_attention(q.tolist(), k.tolist(), v.tolist(), 2, 5)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)


def test_attention_closed_forms():
    g = np.random.default_rng(4)
    S, H, dh = 7, 3, 4
    q, k, v = (g.standard_normal((3 * S, H * dh)) for _ in range(3))
    out = ost.causal_attention(q, k, v, H, S)
    # the first token of every sample can only attend to itself
    np.testing.assert_allclose(out[::S], v[::S], rtol=1e-13)
    # zero keys: uniform attention over the prefix = running mean of v within the sample
    out0 = ost.causal_attention(q, np.zeros_like(k), v, H, S)
    run = np.cumsum(v.reshape(3, S, -1), axis=1) / np.arange(1, S + 1)[None, :, None]
    np.testing.assert_allclose(out0, run.reshape(3 * S, -1), rtol=1e-12)
    # samples do not see each other; heads do not see each other
    v2 = v.copy()
    v2[S:] += 5.0
    np.testing.assert_array_equal(ost.causal_attention(q, k, v2, H, S)[:S], out[:S])
    k2 = k.copy()
    k2[:, dh:] *= -3.0
    np.testing.assert_array_equal(ost.causal_attention(q, k2, v, H, S)[:, :dh], out[:, :dh])
    # a key that dominates: with a huge score on key j every later query copies v[j]
    qd, kd = np.zeros((S, dh)), np.zeros((S, dh))
    qd[:, 0] = 1.0
    kd[2, 0] = 1e4
    od = ost.causal_attention(qd, kd, v[:S, :dh], 1, S)
    np.testing.assert_allclose(od[2:], np.broadcast_to(v[2, :dh], (S - 2, dh)), rtol=1e-12)
    # causality: changing a later token leaves earlier outputs untouched
    q3, k3, v3 = q.copy(), k.copy(), v.copy()
    q3[4], k3[4], v3[4] = 9.0, -9.0, 7.0
    np.testing.assert_array_equal(ost.causal_attention(q3, k3, v3, H, S)[:4], out[:4])


def test_silu_and_rmsnorm_closed_forms():
    g = np.random.default_rng(5)
    a, u = g.standard_normal((5, 9)) * 4.0, g.standard_normal((5, 9))
    np.testing.assert_allclose(ost.silu_mul(a, u), a * scipy.special.expit(a) * u, rtol=1e-13)
    one = np.ones_like(a)
    np.testing.assert_allclose(ost.silu_mul(a, one) - ost.silu_mul(-a, one), a, rtol=1e-12, atol=1e-14)
    assert ost.silu_mul(np.zeros(3), np.ones(3)).tolist() == [0.0, 0.0, 0.0]
    np.testing.assert_allclose(ost.silu_mul(np.array([50.0, -800.0]), np.array([2.0, 1.0])), [100.0, 0.0], atol=1e-18)
    r = ost.rmsnorm(a * 100.0)
    np.testing.assert_allclose((r * r).mean(axis=1), 1.0, rtol=1e-9)
    np.testing.assert_allclose(ost.rmsnorm(3.0 * a, eps=0.0), ost.rmsnorm(a, eps=0.0), rtol=1e-13)
    np.testing.assert_allclose(ost.rmsnorm(np.array([[3.0, 4.0]]), eps=0.0), [[3.0 / math.sqrt(12.5), 4.0 / math.sqrt(12.5)]])


def _tiny_stack(seed=0, layers=2, d=16, ffn=24, n_samples=2, seq=6):
    g = np.random.default_rng(seed)
    h0 = g.standard_normal((n_samples * seq, d))
    h0[:, 3] *= 8.0
    shapes = [(d, d)] * 4 + [(ffn, d)] * 2 + [(d, ffn)]
    Ws = [[(g.standard_normal(s) * 0.3).astype(np.float16) for s in shapes] for _ in range(layers)]
    w = g.uniform(0.1, 1.0, n_samples * seq)
    al = np.array([0.0, 0.25, 0.5, 0.75], np.float32)
    return F16(h0), Ws, (w / w.sum()).astype(np.float32), al


def test_modes_structure():
    h0, Ws, w, al = _tiny_stack()
    run = lambda mode, bits=3: ost.run_stack(h0, Ws, w, bits, 8, al, n_heads=2, seq_len=6, rnd=F16, mode=mode)
    none, p1, p2 = run("none"), run("passact1"), run("passact2")
    # nothing is quantised before the first group: identical in all modes
    for n in ("q_proj", "k_proj", "v_proj"):
        for r in (p1, p2):
            np.testing.assert_array_equal(r[0][n]["X"], none[0][n]["X"])
            np.testing.assert_array_equal(r[0][n]["res"]["losses"], none[0][n]["res"]["losses"])
    differs = 0
    for l in range(2):
        for n in ost.LINEARS:
            # PassAct1's targets are the full-precision model's outputs, i.e. the "none" run's
            np.testing.assert_array_equal(p1[l][n]["Y_ref"], none[l][n]["Y_ref"])
            # "none" and PassAct2 compare against the full-precision linear on the SAME input
            for r in (none, p2):
                np.testing.assert_array_equal(r[l][n]["Y_ref"], F16(orc.ref_output(r[l][n]["X"], Ws[l][ost.LINEARS.index(n)])))
            # both quantised streams see the same kind of input up to the choice of scales:
            # PassAct1 and PassAct2 expose the same inputs while their chosen scales agree
            differs += int(not np.array_equal(p2[l][n]["X"], none[l][n]["X"]))
    assert differs >= 8           # the quantised stream really is fed forward
    np.testing.assert_array_equal(p1[1]["h_out_fp"], none[1]["h_out"])
    # the quantised stream of PassAct1 is propagated with its own chosen scales
    r = p1[0]["o_proj"]
    z = orc.apply_best(r["X"], Ws[0][3], r["res"]["best_scales"], 3, 8)
    np.testing.assert_array_equal(r["Z"], F16(z))
    # at 8 bits the quantised stream stays close to the full-precision one
    n8, q8 = run("none", 8), run("passact2", 8)
    d = np.abs(q8[1]["h_out"].astype(np.float64) - n8[1]["h_out"].astype(np.float64)).max()
    assert d < 0.05 * np.abs(n8[1]["h_out"].astype(np.float64)).max()
    d3 = np.abs(p2[1]["h_out"].astype(np.float64) - none[1]["h_out"].astype(np.float64)).max()
    assert d3 > 4 * d


def test_block_wiring_against_direct_formulas():
    h0, Ws, w, al = _tiny_stack(seed=1, layers=1)
    r = ost.run_stack(h0, Ws, w, 4, 8, al, n_heads=2, seq_len=6, rnd=F16, mode="passact2")[0]
    f = lambda a: np.asarray(a, np.float64)
    x1 = f(h0) / np.sqrt((f(h0) ** 2).mean(1, keepdims=True) + 1e-6)
    np.testing.assert_array_equal(r["q_proj"]["X"], F16(x1))
    np.testing.assert_array_equal(r["k_proj"]["X"], r["q_proj"]["X"])
    att = _brute_attention(f(r["q_proj"]["Z"]).tolist(), f(r["k_proj"]["Z"]).tolist(), f(r["v_proj"]["Z"]).tolist(), 2, 6)
    np.testing.assert_allclose(f(r["o_proj"]["X"]), att, rtol=2e-3, atol=1e-6)      # fp16 storage
    h1 = F16(f(h0) + f(r["o_proj"]["Z"]))
    x2 = f(h1) / np.sqrt((f(h1) ** 2).mean(1, keepdims=True) + 1e-6)
    np.testing.assert_array_equal(r["gate_proj"]["X"], F16(x2))
    np.testing.assert_array_equal(r["up_proj"]["X"], r["gate_proj"]["X"])
    m = f(r["gate_proj"]["Z"]) * scipy.special.expit(f(r["gate_proj"]["Z"])) * f(r["up_proj"]["Z"])
    np.testing.assert_allclose(f(r["down_proj"]["X"]), m, rtol=2e-3, atol=1e-7)
    np.testing.assert_array_equal(r["h_out"], F16(f(h1) + f(r["down_proj"]["Z"])))


def test_joint_search_is_the_width_weighted_mean_of_the_separate_losses():
    h0, Ws, w, al = _tiny_stack(seed=2, layers=1)
    kw = dict(n_heads=2, seq_len=6, rnd=F16, mode="passact2")
    sep = ost.run_stack(h0, Ws, w, 3, 8, al, **kw)[0]
    jnt = ost.run_stack(h0, Ws, w, 3, 8, al, joint=True, **kw)[0]
    # q/k/v share the input and x_stat, so per alpha the joint loss is the mean of the three (equal widths)
    lj = jnt["q_proj"]["res"]["losses"]
    ls = np.mean([sep[n]["res"]["losses"] for n in ("q_proj", "k_proj", "v_proj")], axis=0)
    np.testing.assert_allclose(lj, ls, rtol=1e-12)
    assert jnt["k_proj"]["res"]["best_idx"] == jnt["q_proj"]["res"]["best_idx"] == int(np.argmin(ls))
    np.testing.assert_array_equal(jnt["v_proj"]["res"]["best_scales"], jnt["q_proj"]["res"]["best_scales"])
    # every member is then quantised with the shared scale
    z = orc.apply_best(jnt["k_proj"]["X"], Ws[0][1], jnt["q_proj"]["res"]["best_scales"], 3, 8)
    np.testing.assert_array_equal(jnt["k_proj"]["Z"], F16(z))
