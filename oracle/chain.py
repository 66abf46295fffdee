"""Oracle of the quantisation-exposed sequential calibration of one synthetic
decoder layer (test infrastructure; numpy, float64).

Sec. 3.2.1, PassAct2: every linear is searched on the output of the already
quantised linears before it.  Order q, k, v, o, gate, up, down.  Between two
linears the synthetic chain applies a row-wise RMS normalisation and a fixed
per-channel multiplier (the workload recipe, not the paper's method); `up`
shares `gate`'s input and `down` sees the normalised product of their
quantised outputs.  Each exposed input is rounded to the activation type, as
it would be stored.
"""
from __future__ import annotations

import numpy as np

from oracle import tlq_oracle as orc


def glue(Z, Zb, m_vis, m_txt, period, split):
    """v = Z (* Zb); out = v / sqrt(mean(v^2) + 1e-6) * m(row), float64."""
    v = np.asarray(Z, np.float64)
    if Zb is not None:
        v = v * np.asarray(Zb, np.float64)
    inv = 1.0 / np.sqrt((v * v).mean(axis=1, keepdims=True) + 1e-6)
    rows = np.arange(v.shape[0]) % period
    m = np.where((rows < split)[:, None], np.asarray(m_vis, np.float64)[None, :],
                 np.asarray(m_txt, np.float64)[None, :])
    return v * inv * m


def run_chain(X0, Ws, token_w, bits, group, alphas, mults, period, split, act=np.float16):
    """Returns one record per linear: exposed input X, Y_ref (rounded to `act`),
    search result, and the quantised output Z (rounded to `act`)."""
    recs = []
    X = np.asarray(X0)
    Z = {}
    for li, W in enumerate(Ws):
        if li == 5:                      # up shares gate's exposed input
            X = recs[4]["X"]
        elif li == 6:                    # down: normalised product of the two quantised branches
            X = glue(Z[4], Z[5], mults[6][0], mults[6][1], period, split).astype(act)
        elif li > 0:
            X = glue(Z[li - 1], None, mults[li][0], mults[li][1], period, split).astype(act)
        Y = orc.ref_output(X, W).astype(act)
        res = orc.scale_search(X, W, Y, token_w, bits, group, alphas)
        with np.errstate(over="ignore"):
            Z[li] = orc.apply_best(X, W, res["best_scales"], bits, group).astype(act)
        recs.append({"X": X, "Y_ref": Y, "res": res, "Z": Z[li]})
    return recs
