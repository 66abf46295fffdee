"""Run the sequential calibration of a synthetic decoder stack on one GPU and
report wall time, split into search and glue.

    python -m paper_2602_07899_amd.run_stack --stack cfg5_13b_stack --bits 4

Inputs are drawn on the device (torch's counter-based generator, seeded per
stack and per block), with the same structure as the host recipe of
`workloads.py`: N(0,1) embeddings with a fixed 1 % of outlier channels scaled
x5 on visual rows and x30 on text rows, N(0, w_std^2) weights, heavy-tailed
token weights.  One progress line per block; the last line is a JSON summary.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

from . import stack as gstack
from . import tlq
from . import workloads as wl

SEARCH_KERNELS = ("xstat_partial", "xstat_final", "scale_table", "fake_quant", "gemm_loss", "finalize", "bf16_to_f16",
                  "act_quant", "gram_operand", "gemm_gram", "gram_scale", "gemm_gram_loss")
BLOCK_KERNELS = ("rmsnorm_mul", "causal_attention", "silu_mul", "residual_add")
SELECT_KERNELS = ("token_importance", "topk_mask")


def device_inputs(sw, dev, dtype, n_samples=None):
    """h0 [n_tok, hidden] and token weights [n_tok] on the device."""
    import torch
    ns = n_samples or sw.n_samples
    per, d = sw.seq_len, sw.hidden
    g = torch.Generator(device=dev)
    g.manual_seed(sw.seed * 1000 + 999)
    h = torch.randn((ns * per, d), generator=g, device=dev, dtype=torch.float32)
    oc = torch.from_numpy(wl.outlier_channels(sw.as_workload(), 0)).to(dev)
    is_txt = (torch.arange(ns * per, device=dev) % per) >= sw.n_vis
    mult = torch.where(is_txt, sw.txt_mult, sw.vis_mult).to(torch.float32)
    h[:, oc] *= mult[:, None]
    w = torch.exp(torch.randn(ns * per, generator=g, device=dev, dtype=torch.float32))
    w = torch.where(is_txt, 4.0 * w, w).double()
    return h.to(dtype), (w / w.sum()).float()


def device_weights(sw, dev, dtype):
    import torch

    def fn(layer):
        g = torch.Generator(device=dev)
        g.manual_seed(sw.seed * 1000 + layer)
        return [(torch.randn(s, generator=g, device=dev, dtype=torch.float32) * sw.w_std).to(dtype)
                for s in sw.shapes()]
    return fn


def topk_xstat_fn(sw, n_samples, p, dev, dtype, frac=0.5):
    """x_stat = max over the Top-(frac) positions by accumulated gradient norm (Sec. 3.1.2).  The
    gradients are synthetic stand-ins (they need the trained model and its loss): N(0,1) scaled
    per position so that most visual positions carry almost no gradient."""
    import torch
    per = sw.seq_len
    g = torch.Generator(device=dev)
    g.manual_seed(sw.seed * 1000 + 777)
    amp_vis = torch.exp(torch.randn(sw.n_vis, generator=g, device=dev) * 1.5 - 4.0)
    amp_txt = torch.exp(torch.randn(sw.n_txt, generator=g, device=dev) * 0.5)
    amp = torch.cat([amp_vis, amp_txt]).repeat(n_samples)[:, None]

    def fn(layer, names, X):
        c = X.shape[1]
        g.manual_seed((sw.seed * 1000 + layer) * 16 + gstack.GROUPS.index(tuple(names)))
        G = (torch.randn((n_samples * per, c), generator=g, device=dev, dtype=torch.float32) * amp).to(dtype)
        sum_n = torch.empty(per, dtype=torch.float64, device=dev)
        tlq.token_importance(G, n_samples, p, sum_n)
        mask = torch.empty(per, dtype=torch.uint8, device=dev)
        tlq.topk_mask(sum_n, max(1, int(per * frac)), mask)
        xs = torch.empty(c, dtype=torch.float32, device=dev)
        tlq.x_stat_masked(X, mask, p, xs)
        return xs
    return fn


def run(stack_name, bits, mode="passact2", joint=False, n_layers=None, n_samples=None, journal_path=None,
        act_bits=0, log=print, group=None, symmetric=False, xstat="mean", strategy="tokens"):
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("run_stack needs a GPU")
    dev = torch.device("cuda:0")
    sw = wl.STACKS[stack_name]
    bf16 = sw.act_dtype == "bf16"
    dtype = torch.bfloat16 if bf16 else torch.float16
    code = tlq.BF16 if bf16 else tlq.F16
    p = tlq.params(bits=bits, group=sw.group if group is None else group, symmetric=1 if symmetric else 0,
                   x_dtype=code, yref_dtype=code, act_bits=act_bits)
    layers = n_layers or sw.n_layers
    h0, w = device_inputs(sw, dev, dtype, n_samples)
    al = torch.from_numpy(wl.alpha_grid(sw.n_alpha)).to(dev)
    jcfg = {"stack": stack_name, "seed": sw.seed, "bits": bits, "group": p.group, "symmetric": int(p.symmetric),
            "act_bits": act_bits, "mode": mode, "joint": bool(joint), "x_stat": xstat, "xstat_kind": int(p.xstat_kind),
            "n_samples": int(n_samples or sw.n_samples), "n_alpha": sw.n_alpha, "dtype": sw.act_dtype,
            "strategy": strategy}
    journal = gstack.Journal(journal_path, config=jcfg) if journal_path else None
    tlq.profile_reset()
    tlq.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.time()
    summary = []

    def on_layer(layer, recs):
        # one small device-to-host read per block: it is the progress line
        idx = [int(recs[n]["best_idx"].item()) for n in gstack.LINEARS]
        ls = [recs[n]["losses"].tolist() for n in gstack.LINEARS]
        summary.append({"layer": layer, "best_idx": idx, "losses": ls})
        log(f"[run_stack] W{bits} {mode} block {layer + 1}/{layers} done at {time.time() - t0:7.2f} s  best_idx={idx}")
        sys.stdout.flush()

    xfn = topk_xstat_fn(sw, n_samples or sw.n_samples, p, dev, dtype) if xstat == "topk" else None
    _, hq, hf = gstack.run_stack(h0, device_weights(sw, dev, dtype), layers, w, al, p, sw.n_heads, sw.seq_len,
                                 mode=mode, joint=joint, journal=journal, on_layer=on_layer, xstat_fn=xfn,
                                 strategy=strategy)
    torch.cuda.synchronize()
    wall = time.time() - t0
    tlq.profile_enable(False)
    prof = {k.name: k for k in tlq.profile_read()}
    search_ms = sum(k.total_ms for n, k in prof.items() if n in SEARCH_KERNELS or n in SELECT_KERNELS)
    block_ms = sum(k.total_ms for n, k in prof.items() if n in BLOCK_KERNELS)
    prop_ms = sum(k.total_ms for n, k in prof.items()
                  if n not in SEARCH_KERNELS and n not in BLOCK_KERNELS and n not in SELECT_KERNELS)
    gl = prof.get("gemm_loss") or prof.get("gemm_gram_loss")
    out = {
        "stack": stack_name, "bits": bits, "group": p.group, "symmetric": bool(p.symmetric), "mode": mode,
        "joint": joint, "act_bits": act_bits, "x_stat": xstat, "strategy": strategy, "layers": layers,
        "n_tok": int(h0.shape[0]), "hidden": sw.hidden, "ffn": sw.ffn, "dtype": sw.act_dtype,
        # search = S0..S5; propagate = full-precision targets and the quantised outputs fed forward (S6);
        # block = the decoder block between the linears; the rest is weight generation and host time
        "wall_s": wall, "search_kernels_s": search_ms / 1e3, "propagate_kernels_s": prop_ms / 1e3,
        "block_kernels_s": block_ms / 1e3, "other_s": wall - (search_ms + prop_ms + block_ms) / 1e3,
        "evals": 7 * layers * sw.n_alpha,
        "evals_per_s": (7 * layers * sw.n_alpha) / wall,
        "gemm_loss_tflops": (gl.total_work / (gl.total_ms * 1e-3) / 1e12) if gl and gl.total_ms > 0 else None,
        "kernels": {n: {"launches": k.launches, "ms": round(k.total_ms, 3)} for n, k in prof.items()},
        "peak_hbm_bytes": int(torch.cuda.max_memory_allocated()),
        "h_finite": bool(torch.isfinite(hq.float()).all().item()),
        "h_rms": float(hq.float().pow(2).mean().sqrt().item()),
        "stream_gap_rel": float(((hq.float() - hf.float()).norm() / hf.float().norm()).item()),
        "blocks": summary,
    }
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--stack", default="cfg5_13b_stack", choices=sorted(wl.STACKS))
    ap.add_argument("--bits", type=int, default=4)
    ap.add_argument("--mode", default="passact2", choices=("none", "passact1", "passact2"))
    ap.add_argument("--joint", action="store_true")
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--samples", type=int, default=None)
    ap.add_argument("--act-bits", type=int, default=0)
    ap.add_argument("--group", type=int, default=None, help="quantisation group (0 = whole row); default: the stack's")
    ap.add_argument("--symmetric", action="store_true")
    ap.add_argument("--xstat", default="mean", choices=("mean", "topk"),
                    help="mean |x| (default) or the maximum over the Top-50%% positions by synthetic gradient norm")
    ap.add_argument("--strategy", default="tokens", choices=("tokens", "gram", "auto"),
                    help="tokens: every candidate contracts the tokens; gram: candidates are evaluated through the "
                         "weighted second-moment matrix of the exposed input (weight-only, not passact1); auto: per "
                         "group of linears, whichever the flop model favours")
    ap.add_argument("--journal", default=None)
    ap.add_argument("--brief", action="store_true", help="leave the per-block records out of the summary")
    a = ap.parse_args()
    out = run(a.stack, a.bits, a.mode, a.joint, a.layers, a.samples, a.journal, a.act_bits, group=a.group,
              symmetric=a.symmetric, xstat=a.xstat, strategy=a.strategy)
    if a.brief:
        out.pop("blocks")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
