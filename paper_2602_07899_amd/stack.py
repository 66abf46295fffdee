"""Sequential calibration of a stack of synthetic decoder blocks through libtlq
(Sec. 3.2.1).  Host-side sequencing only: every tensor operation is a library
kernel; torch supplies device memory and the concatenation of weight rows for a
joint search.

Propagation modes (Sec. 3.2.1):
  "none"      every linear is searched on the full-precision model's activations;
  "passact1"  two activation streams: x_fp through the full-precision linears,
              x_q through the quantised ones; searched on x_q against f_fp(x_fp);
  "passact2"  one stream: each linear sees the output of the quantised linears
              before it and is compared with the full-precision linear on that input.
Block: h -> RMSNorm -> q, k, v -> causal attention per sample -> o -> +residual
-> RMSNorm -> gate, up -> SiLU(gate)*up -> down -> +residual.
`joint=True` searches linears that share an input (q/k/v, gate/up) with one
scale vector over their row-concatenated weights.
A journal (JSON lines, one record per searched group) makes a run resumable:
groups found in it are not searched again - their recorded grid index is turned
back into scales (same x_stat and scale-table kernels, so the same bits) and
only the propagation is redone.
"""
from __future__ import annotations

import json
import os

from . import tlq

LINEARS = ("q_proj", "k_proj", "v_proj", "o_proj", "gate_proj", "up_proj", "down_proj")
GROUPS = (("q_proj", "k_proj", "v_proj"), ("o_proj",), ("gate_proj", "up_proj"), ("down_proj",))


class Journal:
    """Append-only JSON-lines record of finished searches, keyed by (layer, linear).  The first
    line of the file is a header holding the run's configuration (quantiser, grid, propagation
    mode, statistic, seed - whatever the caller passes as `config`); a journal whose header
    differs from the current configuration belongs to another run and is refused."""

    def __init__(self, path, config=None):
        self.path = path
        self.done = {}
        self.config = config
        self.header_written = False
        if path and os.path.exists(path) and os.path.getsize(path) > 0:
            with open(path, "rb") as f:
                first = f.readline()
            try:
                head = json.loads(first.decode()) if first.endswith(b"\n") else None
            except ValueError:
                head = None
            if isinstance(head, dict) and "journal_config" in head:
                self.header_written = True
                if config is not None and head["journal_config"] != config:
                    raise ValueError(f"journal {path} was written with another configuration: "
                                     f"{head['journal_config']} != {config}")
            elif config is not None:
                raise ValueError(f"journal {path} has no configuration header; refusing to resume from it")
        if path and os.path.exists(path):
            good = 0
            with open(path, "rb") as f:
                for raw in f:
                    try:
                        r = json.loads(raw.decode()) if raw.endswith(b"\n") else None
                    except ValueError:
                        r = None
                    if r is None and raw.strip():   # a line cut short by an interrupted run
                        break
                    good += len(raw)
                    if r is not None and "journal_config" not in r:
                        self.done[(r["layer"], r["linear"])] = r
            if good != os.path.getsize(path):       # drop the damaged tail so that appends stay line-aligned
                with open(path, "r+b") as f:
                    f.truncate(good)

    def get(self, layer, name):
        return self.done.get((layer, name))

    def put(self, rec):
        self.done[(rec["layer"], rec["linear"])] = rec
        if self.path:
            with open(self.path, "a") as f:
                if not self.header_written and self.config is not None:
                    f.write(json.dumps({"journal_config": self.config}) + "\n")
                    self.header_written = True
                f.write(json.dumps(rec) + "\n")
                f.flush()
                os.fsync(f.fileno())


def second_moment_pays(n_tok, c_in, widths, n_alpha):
    """Flop model behind strategy="auto": contracting the tokens with every candidate costs
    2 N C_in C_out per candidate; the second-moment form N C_in^2 once per group (symmetric
    product) plus C_out C_in^2 per candidate (symmetric contraction).  Its contractions run at
    about three quarters of the token form's rate (short launches, tiles of unequal length), so it is
    chosen when its flop count is under half of the token form's."""
    c_out = sum(widths)
    tokens = 2.0 * n_alpha * n_tok * c_in * c_out
    moment = float(n_tok) * c_in * c_in + float(n_alpha) * c_out * c_in * c_in
    return moment < 0.5 * tokens


def run_stack(h0, weights_fn, n_layers, token_w, alpha_grid, p, n_heads, seq_len, mode="passact2",
              joint=False, journal=None, keep=False, on_layer=None, xstat_fn=None, strategy="tokens"):
    """h0 [n_tok, n_heads*128] device tensor in the activation type; weights_fn(layer)
    returns the 7 device weight matrices of one block (LINEARS order).  Returns
    (records, h_q, h_fp): records[layer][linear] holds device tensors best_idx, losses,
    best_scales (plus X, Y_ref, Z when keep=True); h_q / h_fp are the final hidden
    states of the quantised / full-precision streams (the same tensor unless
    mode == "passact1").  xstat_fn(layer, names, X) may return a device float vector with the
    per-channel statistic of a group's exposed input (e.g. the gradient-guided Top-K maximum,
    Sec. 3.1.2, built with tlq.token_importance / topk_mask / x_stat_masked); None = the
    statistic p.xstat_kind names.  strategy "gram" evaluates the candidates through the weighted
    second-moment matrix of each group's exposed input (tlq.token_gram / scale_search_gram): weight-only
    settings whose target is f_fp of that same input, i.e. not PassAct1; the target then is the exact
    product and, under PassAct2, the full-precision outputs are not formed at all.  strategy "auto"
    decides per group of linears with `second_moment_pays`."""
    import torch
    assert mode in ("none", "passact1", "passact2")
    assert strategy in ("tokens", "gram", "auto")
    gram_ok = mode != "passact1" and p.act_bits == 0
    assert strategy != "gram" or gram_ok, "the second-moment form needs f_q linear in the searched input"
    gram_any = strategy == "gram" or (strategy == "auto" and gram_ok)     # some group may use it
    dev, act = h0.device, h0.dtype
    n_tok, d = h0.shape
    assert d == n_heads * 128 and n_tok % seq_len == 0
    two = mode == "passact1"
    y_dt = {tlq.F16: torch.float16, tlq.BF16: torch.bfloat16, tlq.F32: torch.float32}[p.yref_dtype]
    assert y_dt == act, "the full-precision stream is propagated in the activation type"
    na = alpha_grid.numel()
    new = lambda cols, dt=act: torch.empty((n_tok, cols), dtype=dt, device=dev)
    ws_cache = {}

    def workspace(c_in, c_out):
        need = max(tlq.scale_search_gram_workspace_bytes(c_in, c_out, na, p) if gram_any else 0,
                   tlq.scale_search_workspace_bytes(n_tok, c_in, c_out, na, p) if strategy != "gram" else 0,
                   tlq.token_gram_workspace_bytes(n_tok, c_in) if gram_any else 0,
                   tlq.apply_best_workspace_bytes(n_tok, c_in, c_out, p), tlq.x_stat_workspace_bytes(n_tok, c_in))
        if ws_cache.get("n", 0) < need:
            ws_cache["t"] = None
            ws_cache["t"] = torch.empty(need, dtype=torch.uint8, device=dev)
            ws_cache["n"] = need
        return ws_cache["t"]

    def prepared_buffer(nbytes):
        if ws_cache.get("pn", 0) < nbytes:
            ws_cache["p"] = None
            ws_cache["p"] = torch.empty(nbytes, dtype=torch.uint8, device=dev)
            ws_cache["pn"] = nbytes
        return ws_cache["p"][:nbytes]

    def search_group(layer, names, Ws, Xq, Xfp, recs):
        """Returns (Zq list, Zfp list): per-member quantised and full-precision outputs
        (column slices of one matrix each)."""
        widths = [W.shape[0] for W in Ws]
        c_in, tot = Ws[0].shape[1], sum(widths)
        offs = [sum(widths[:i]) for i in range(len(Ws))]
        gram = strategy == "gram" or (strategy == "auto" and gram_ok and second_moment_pays(n_tok, c_in, widths, na))
        need_y = not (gram and mode == "passact2")       # the target enters only through the matrix there
        Y = new(tot, y_dt) if need_y else None
        Ys = [Y[:, o:o + w] for o, w in zip(offs, widths)] if need_y else [None] * len(Ws)
        for W, Yi in zip(Ws, Ys):
            if need_y:
                tlq.ref_output(Xfp, W, Yi, p)
        Z = None if mode == "none" else new(tot)
        # once per distinct exposed input: the channel statistic and (bf16) the fp16 re-expression
        xs_in = xstat_fn(layer, names, Xq) if xstat_fn is not None else None
        if xs_in is None:
            xs_in = torch.empty(c_in, dtype=torch.float32, device=dev)
            tlq.x_stat(Xq, p, xs_in, workspace=workspace(c_in, max(widths)))
        pb = tlq.prepared_tokens_bytes(n_tok, c_in, p)
        prep = None
        if pb:
            prep = prepared_buffer(pb)
            tlq.prepare_tokens(Xq, p, prep)
        gm = []

        def group_gram():      # once per distinct exposed input as well, and only if a member is searched
            if not gm:
                gb = tlq.token_gram_bytes(c_in)
                if ws_cache.get("gn", 0) < gb:
                    ws_cache["g"] = None
                    ws_cache["g"] = torch.empty(gb, dtype=torch.uint8, device=dev)
                    ws_cache["gn"] = gb
                gm.append(tlq.token_gram(Xq, token_w, p, ws_cache["g"][:gb], workspace=workspace(c_in, max(widths))))
            return gm[0]
        units = [(names, torch.cat(Ws, dim=0) if len(Ws) > 1 else Ws[0], Y, Z)] if joint else \
                [((n,), W, Yi, None if Z is None else Z[:, o:o + w]) for n, W, Yi, o, w in zip(names, Ws, Ys, offs, widths)]
        for unames, W, Yu, Zu in units:
            ws = workspace(c_in, W.shape[0])
            best = torch.empty(c_in, dtype=torch.float32, device=dev)
            idx = torch.empty(1, dtype=torch.int32, device=dev)
            losses = torch.empty(na, dtype=torch.float32, device=dev)
            old = journal.get(layer, unames[0]) if journal is not None else None
            want_joint = list(unames) if len(unames) > 1 else None
            if old is not None and (old.get("joint") != want_joint or not (0 <= old["best_idx"] < na)):
                old = None      # recorded for another grouping, or no candidate was finite: search again
            if old is not None:                                   # resume: rebuild the chosen scales
                tlq.scale_table(xs_in, alpha_grid[old["best_idx"]:old["best_idx"] + 1], best)
                idx.fill_(old["best_idx"])
                losses.copy_(torch.tensor(old["losses"], dtype=torch.float32))
            else:
                if gram:
                    g_in = group_gram()          # (may regrow the shared workspace: fetch `ws` after it)
                    ws = workspace(c_in, W.shape[0])
                    tlq.scale_search_gram(g_in, W, alpha_grid, p, xs_in, best, idx, losses, workspace=ws)
                else:
                    tlq.scale_search(Xq, W, Yu, token_w, alpha_grid, p, best, idx, losses, x_stat_in=xs_in,
                                     workspace=ws, prepared=prep)
                if journal is not None:
                    li, ll = int(idx.item()), [float(v) for v in losses.tolist()]
                    for n in unames:
                        journal.put({"layer": layer, "linear": n, "best_idx": li,
                                     "alpha": float(alpha_grid[li].item()) if li >= 0 else None, "losses": ll,
                                     "joint": list(unames) if len(unames) > 1 else None})
            if Zu is not None:
                tlq.apply_best(Xq, W, best, p, Zu, workspace=ws, prepared=prep)
            for n in unames:
                rec = {"best_idx": idx, "losses": losses, "best_scales": best}
                if keep:
                    k = names.index(n)
                    rec.update(X=Xq, Y_ref=Ys[k], Z=None if Z is None else Z[:, offs[k]:offs[k] + widths[k]])
                recs[n] = rec
        Zfp = Ys
        Zq = Zfp if Z is None else [Z[:, o:o + w] for o, w in zip(offs, widths)]
        return Zq, (Zfp if (two or mode == "none") else Zq)

    hq = h0
    hf = h0
    out = []
    for layer in range(n_layers):
        Wl = dict(zip(LINEARS, weights_fn(layer)))
        recs = {}
        grp = lambda names, xq, xf: search_group(layer, names, [Wl[n] for n in names], xq, xf, recs)

        x1q = tlq.rmsnorm_mul(hq, p, new(d))
        x1f = tlq.rmsnorm_mul(hf, p, new(d)) if two else x1q
        zq, zf = grp(GROUPS[0], x1q, x1f)
        aq = tlq.causal_attention(zq[0], zq[1], zq[2], n_heads, seq_len, p, new(d))
        af = tlq.causal_attention(zf[0], zf[1], zf[2], n_heads, seq_len, p, new(d)) if two else aq
        del zq, zf
        zq, zf = grp(GROUPS[1], aq, af)
        hq_new = tlq.residual_add(hq, zq[0], p, new(d))
        hf = tlq.residual_add(hf, zf[0], p, new(d)) if two else hq_new
        hq = hq_new
        del zq, zf, aq, af
        x2q = tlq.rmsnorm_mul(hq, p, new(d))
        x2f = tlq.rmsnorm_mul(hf, p, new(d)) if two else x2q
        zq, zf = grp(GROUPS[2], x2q, x2f)
        f = Wl["gate_proj"].shape[0]
        mq = tlq.silu_mul(zq[0], zq[1], p, new(f))
        mf = tlq.silu_mul(zf[0], zf[1], p, new(f)) if two else mq
        del zq, zf
        zq, zf = grp(GROUPS[3], mq, mf)
        hq_new = tlq.residual_add(hq, zq[0], p, new(d))
        hf = tlq.residual_add(hf, zf[0], p, new(d)) if two else hq_new
        hq = hq_new
        del zq, zf, mq, mf
        if keep:
            recs["h_out"], recs["h_out_fp"] = hq, hf
        out.append(recs)
        if on_layer is not None:
            on_layer(layer, recs)
    return out, hq, hf
