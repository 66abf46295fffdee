"""Brute-force cross-check of the oracle on tiny layers (test infrastructure).

Pure-Python triple loops over Python floats (IEEE double).  The quantiser's
float32 steps go through numpy.float32 *scalars*, one operation at a time, so
each step rounds exactly once.  Nothing here is vectorised and nothing is
imported from the oracle: the two are written independently from the same
definitions (Sec. 2.2 quantiser, Sec. 3.1.2 scale, Sec. 3.2.1 objective) and
a test asserts that they agree.
"""
from __future__ import annotations

import math

import numpy as np

f32 = np.float32


def _rne(x: float) -> float:
    """Round half to even on a Python float."""
    fl = math.floor(x)
    d = x - fl
    if d > 0.5:
        return fl + 1.0
    if d < 0.5:
        return float(fl)
    return float(fl) if (fl % 2 == 0) else fl + 1.0


def brute_x_stat(X):
    n, c = len(X), len(X[0])
    out = []
    for j in range(c):
        acc = 0.0
        for t in range(n):
            acc += abs(float(X[t][j]))
        out.append(f32(acc / n))
    return out


def brute_scale(x_stat, alpha):
    out = []
    for v in x_stat:
        base = float(v)
        if base < 2.0 ** -14:
            base = 2.0 ** -14
        out.append(f32(math.pow(base, float(f32(alpha)))))
    return out


def brute_fake_quant_row(wrow, s, bits, group):
    """One output row.  Returns (codes, zps, deltas, deq) as Python lists."""
    c_in = len(wrow)
    g = c_in if group == 0 else group
    qmax = f32((1 << bits) - 1)
    codes, zps, deltas, deq = [], [], [], []
    for g0 in range(0, c_in, g):
        ws = [f32(f32(wrow[c]) * f32(s[c])) for c in range(g0, g0 + g)]
        mx = ws[0]
        mn = ws[0]
        for v in ws[1:]:
            if v > mx:
                mx = v
            if v < mn:
                mn = v
        rng = f32(mx - mn)
        if rng < f32(1e-5):
            rng = f32(1e-5)
        delta = f32(rng / qmax)
        z = _rne(float(f32(f32(-mn) / delta)))
        z = min(max(z, 0.0), float(qmax))
        for v in ws:
            q = _rne(float(f32(v / delta))) + z
            q = min(max(q, 0.0), float(qmax))
            codes.append(int(q))
            deq.append(f32(f32(q - z) * delta))
        zps.append(int(z))
        deltas.append(delta)
    return codes, zps, deltas, deq


def brute_loss(X, W, Y_ref, token_w, s, bits, group):
    """sum_t w_t * (1/C_out) * sum_o (Y_ref[t][o] - sum_c (X[t][c]/s[c]) deq[o][c])^2"""
    n, c_in, c_out = len(X), len(X[0]), len(W)
    deq_rows = [brute_fake_quant_row(W[o], s, bits, group)[3] for o in range(c_out)]
    total = 0.0
    for t in range(n):
        row = 0.0
        for o in range(c_out):
            y = 0.0
            for c in range(c_in):
                y += (float(X[t][c]) / float(s[c])) * float(deq_rows[o][c])
            d = float(Y_ref[t][o]) - y
            row += d * d
        total += float(token_w[t]) * (row / c_out)
    return total


def brute_search(X, W, Y_ref, token_w, bits, group, alphas):
    xs = brute_x_stat(X)
    losses = []
    for a in alphas:
        s = brute_scale(xs, a)
        losses.append(brute_loss(X, W, Y_ref, token_w, s, bits, group))
    best = 0
    for k in range(1, len(losses)):
        if losses[k] < losses[best]:
            best = k
    return xs, losses, best


def brute_act_quant_row(xrow, s, act_bits):
    """Per-token symmetric quantiser on x/s (Sec. 2.2 first two equations applied to one
    activation row; Sec. 3.2.1 Q_a).  Returns (codes, sigma)."""
    half = 1 << (act_bits - 1)
    xt = [f32(f32(xrow[c]) * f32(1.0 / float(f32(s[c])))) for c in range(len(xrow))]
    amax = f32(0.0)
    for v in xt:
        a = f32(abs(v))
        if a > amax:
            amax = a
    if amax < f32(1e-5):
        amax = f32(1e-5)
    sigma = f32(amax / f32(half - 1))
    codes = []
    for v in xt:
        q = _rne(float(f32(v / sigma)))
        codes.append(int(min(max(q, -half), half - 1)))
    return codes, sigma


def brute_loss_aq(X, W, Y_ref, token_w, s, bits, group, act_bits):
    n, c_in, c_out = len(X), len(X[0]), len(W)
    deq_rows = [brute_fake_quant_row(W[o], s, bits, group)[3] for o in range(c_out)]
    total = 0.0
    for t in range(n):
        codes, sigma = brute_act_quant_row(X[t], s, act_bits)
        row = 0.0
        for o in range(c_out):
            y = 0.0
            for c in range(c_in):
                y += codes[c] * float(deq_rows[o][c])
            d = float(Y_ref[t][o]) - float(sigma) * y
            row += d * d
        total += float(token_w[t]) * (row / c_out)
    return total
