"""Oracle of the sequential calibration of a stack of synthetic decoder blocks
(test infrastructure; numpy, float64; imports nothing from the GPU package).

Sec. 3.2.1 describes three ways to feed a linear layer during its search:
  "none"     every linear sees the full-precision model's activations;
  "passact1" two activation streams are kept, x_fp through the full-precision
             linears and x_q through the already quantised ones; the scale is
             searched on x_q against the full-precision output f_fp(x_fp);
  "passact2" one stream: the input of every linear is the output of the
             quantised linears before it, and the target is the full-precision
             linear applied to that same exposed input.
What sits between the linears is the workload's decoder block, not the paper's
method:  h -> RMSNorm -> q, k, v -> causal attention per calibration sample
-> o -> + residual -> RMSNorm -> gate, up -> SiLU(gate) * up -> down ->
+ residual.  Linears that share an input (q/k/v, gate/up) can be searched
jointly: one scale vector for the row-wise concatenation of their weights
(the scale is folded into the one normalisation that precedes them, Sec. 2.2).
Every tensor the device path stores in the activation type is rounded to that
type here too (`rnd`).
"""
from __future__ import annotations

import numpy as np

from oracle import tlq_oracle as orc

LINEARS = ("q_proj", "k_proj", "v_proj", "o_proj", "gate_proj", "up_proj", "down_proj")


def rmsnorm(h, eps=1e-6):
    """Row-wise h / sqrt(mean(h^2) + eps), float64."""
    v = np.asarray(h, np.float64)
    return v / np.sqrt((v * v).mean(axis=1, keepdims=True) + eps)


def causal_attention(q, k, v, n_heads, seq_len):
    """softmax(q k^T / sqrt(d_head) + causal mask) v, per block of `seq_len`
    consecutive rows (one calibration sample) and per head; float64.
    q, k, v: [n_tok, n_heads * d_head]."""
    q, k, v = (np.asarray(a, np.float64) for a in (q, k, v))
    n_tok, width = q.shape
    assert n_tok % seq_len == 0 and width % n_heads == 0
    dh = width // n_heads
    out = np.empty_like(q)
    mask = np.triu(np.ones((seq_len, seq_len), bool), k=1)          # key index > query index
    for b in range(n_tok // seq_len):
        r = slice(b * seq_len, (b + 1) * seq_len)
        for h in range(n_heads):
            c = slice(h * dh, (h + 1) * dh)
            s = q[r, c] @ k[r, c].T / np.sqrt(float(dh))
            s[mask] = -np.inf
            s -= s.max(axis=1, keepdims=True)
            p = np.exp(s)
            p /= p.sum(axis=1, keepdims=True)
            out[r, c] = p @ v[r, c]
    return out


def silu_mul(g, u):
    """SiLU(g) * u = g / (1 + exp(-g)) * u, float64."""
    g, u = np.asarray(g, np.float64), np.asarray(u, np.float64)
    with np.errstate(over="ignore"):
        return g / (1.0 + np.exp(-g)) * u


def _search_group(Xq, Xfp, Ws, token_w, bits, group, alphas, joint, rnd, kw, x_stat=None):
    """Search the linears `Ws` that share the exposed input Xq; the target is
    computed from Xfp (== Xq unless two streams are kept).  Returns per-linear
    records and the quantised / full-precision outputs."""
    recs, Zq, Zfp = [], [], []
    Ys = [rnd(orc.ref_output(Xfp, W)) for W in Ws]
    if joint and len(Ws) > 1:
        Wc, Yc = np.concatenate(Ws, axis=0), np.concatenate(Ys, axis=1)
        res = orc.scale_search(Xq, Wc, Yc, token_w, bits, group, alphas, x_stat=x_stat, **kw)
        results = [res] * len(Ws)
    else:
        results = [orc.scale_search(Xq, W, Y, token_w, bits, group, alphas, x_stat=x_stat, **kw) for W, Y in zip(Ws, Ys)]
    for W, Y, res in zip(Ws, Ys, results):
        with np.errstate(over="ignore"):
            Zq.append(rnd(orc.apply_best(Xq, W, res["best_scales"], bits, group, **kw)))
        Zfp.append(Y)
        recs.append({"X": Xq, "Y_ref": Y, "res": res, "Z": Zq[-1]})
    return recs, Zq, Zfp


def run_stack(h0, layer_weights, token_w, bits, group, alphas, n_heads, seq_len, rnd,
              mode="passact2", joint=False, symmetric=False, act_bits=0, xstat_fn=None):
    """h0 [n_tok, d] (already in the activation type); layer_weights: one list of
    7 weight matrices per decoder block, in LINEARS order; rnd(a) rounds a float64
    array to the activation type (returned as an array numpy can compute with).
    xstat_fn(layer, names, X) may supply the per-channel statistic of a group's exposed
    input (e.g. the gradient-guided Top-K maximum of Sec. 3.1.2); None = mean |x|.
    Returns records[layer][linear] with the exposed input X, the target Y_ref, the
    search result and the quantised output Z."""
    assert mode in ("none", "passact1", "passact2")
    kw = {"symmetric": symmetric, "act_bits": act_bits}
    two = mode == "passact1"
    hq = np.asarray(h0)
    hf = hq
    out = []
    for layer, Ws in enumerate(layer_weights):
        recs = {}

        def block(xq, xf, names):
            idx = [LINEARS.index(n) for n in names]
            xs = xstat_fn(layer, names, xq) if xstat_fn is not None else None
            r, zq, zf = _search_group(xq, xf, [Ws[i] for i in idx], token_w, bits, group, alphas, joint, rnd, kw, xs)
            for n, rec in zip(names, r):
                recs[n] = rec
            if mode == "none":              # the quantised outputs are never fed forward
                return zf, zf
            return zq, (zf if two else zq)

        x1q = rnd(rmsnorm(hq))
        x1f = rnd(rmsnorm(hf)) if two else x1q
        zq, zf = block(x1q, x1f, ("q_proj", "k_proj", "v_proj"))
        aq = rnd(causal_attention(zq[0], zq[1], zq[2], n_heads, seq_len))
        af = rnd(causal_attention(zf[0], zf[1], zf[2], n_heads, seq_len)) if two else aq
        zq, zf = block(aq, af, ("o_proj",))
        hq = rnd(np.asarray(hq, np.float64) + np.asarray(zq[0], np.float64))
        hf = rnd(np.asarray(hf, np.float64) + np.asarray(zf[0], np.float64)) if two else hq
        x2q = rnd(rmsnorm(hq))
        x2f = rnd(rmsnorm(hf)) if two else x2q
        zq, zf = block(x2q, x2f, ("gate_proj", "up_proj"))
        mq = rnd(silu_mul(zq[0], zq[1]))
        mf = rnd(silu_mul(zf[0], zf[1])) if two else mq
        zq, zf = block(mq, mf, ("down_proj",))
        hq = rnd(np.asarray(hq, np.float64) + np.asarray(zq[0], np.float64))
        hf = rnd(np.asarray(hf, np.float64) + np.asarray(zf[0], np.float64)) if two else hq
        recs["h_out"] = hq
        recs["h_out_fp"] = hf
        out.append(recs)
    return out
