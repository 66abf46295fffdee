"""Quantisation-exposed sequential calibration of one synthetic decoder layer
through libtlq (Sec. 3.2.1, PassAct2): each linear is searched on the output
of the already quantised linears before it.  Host-side sequencing only - every
tensor operation is a library kernel (`tlq_ref_output`, `tlq_scale_search`,
`tlq_apply_best`, `tlq_rmsnorm_mul`); torch supplies device memory.

Order q, k, v, o, gate, up, down; `up` shares `gate`'s input; `down` sees the
normalised product of the two quantised branches.
"""
from __future__ import annotations

from . import tlq


def run_chain(X0, Ws, token_w, alpha_grid, p, mults, period, split, keep=False):
    """X0 [n_tok, c_in0], Ws: list of 7 weight tensors, mults[li] = (m_vis, m_txt)
    device float vectors for the input of linear li (li >= 1).  Returns a list of
    dicts with best_idx, losses, best_scales (device tensors) per linear, plus the
    exposed input X and quantised output Z when keep=True."""
    import torch
    dev, act = X0.device, X0.dtype
    n_tok = X0.shape[0]
    y_dt = {tlq.F16: torch.float16, tlq.BF16: torch.bfloat16, tlq.F32: torch.float32}[p.yref_dtype]
    ws_bytes = max(max(tlq.scale_search_workspace_bytes(n_tok, W.shape[1], W.shape[0], alpha_grid.numel(), p),
                       tlq.apply_best_workspace_bytes(n_tok, W.shape[1], W.shape[0], p)) for W in Ws)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    recs, Z, X = [], {}, X0
    for li, W in enumerate(Ws):
        c_out, c_in = W.shape
        if li == 5:
            X = recs[4]["_X"]
        elif li == 6:
            Xn = torch.empty((n_tok, c_in), dtype=act, device=dev)
            X = tlq.rmsnorm_mul(Z[4], p, Xn, Zb=Z[5], m_a=mults[6][0], m_b=mults[6][1], period=period, split=split)
        elif li > 0:
            Xn = torch.empty((n_tok, c_in), dtype=act, device=dev)
            X = tlq.rmsnorm_mul(Z[li - 1], p, Xn, m_a=mults[li][0], m_b=mults[li][1], period=period, split=split)
        Y = torch.empty((n_tok, c_out), dtype=y_dt, device=dev)
        tlq.ref_output(X, W, Y, p)
        best = torch.empty(c_in, dtype=torch.float32, device=dev)
        idx = torch.empty(1, dtype=torch.int32, device=dev)
        losses = torch.empty(alpha_grid.numel(), dtype=torch.float32, device=dev)
        tlq.scale_search(X, W, Y, token_w, alpha_grid, p, best, idx, losses, workspace=ws)
        Zl = torch.empty((n_tok, c_out), dtype=act, device=dev)
        tlq.apply_best(X, W, best, p, Zl, workspace=ws)
        Z[li] = Zl
        rec = {"best_idx": idx, "losses": losses, "best_scales": best, "_X": X}
        if keep:
            rec["X"], rec["Z"] = X, Zl
        recs.append(rec)
        if not keep and li - 1 in Z and li - 1 != 4:      # gate's output is needed again by down
            del Z[li - 1]
    return recs
