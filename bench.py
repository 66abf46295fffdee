"""Benchmark of the TLQ scale-search hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the whole hot path (x_stat, scale table, fake
quantisation of every candidate, fused contraction + weighted loss, final
combine and selection) over the seven linears of one decoder layer with a
20-point alpha grid: 7 x 20 = 140 candidate evaluations.  The headline
workload is the largest one-GPU layer configuration, the 13B-class layer
with 128 x 1200 = 153,600 synthetic calibration tokens (cfg4_13b_w4); the
7B-class layer with 16 x 640 tokens (cfg2_7b_w4) is timed in the same run and
reported under "secondary".  Inputs (X, W, Y_ref, token weights) are resident
in HBM before the timed region.  Prints ONE JSON line.

Outside the timed region the CPU oracle is timed on a bounded sample of each
workload ("cpu_baseline") and its losses on that sample are compared with the
library's losses on the same inputs ("parity_max_rel").
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "candidate-scale evals/sec per layer + fused-kernel TFLOP/s (% fp16 MFMA peak)"
PEAK_FP16_TFLOPS = 2500.0      # MI355X dense fp16 MFMA peak (published)
HOST_THREADS = 16              # the GPU machine's CPU share


def log(msg):
    print(f"bench.py: {msg}", file=sys.stderr, flush=True)


def source_fingerprint():
    """sha256 over the sources of the contraction kernels (the kernel the stored counter
    readings describe): those readings are only quoted for the build they were taken from."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2602_07899_amd", "csrc")
    files = [os.path.join(csrc, "gemm.hip"), os.path.join(csrc, "common.h")]
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic(workload_name):
    """Bytes per gemm_loss launch that cross the L2/fabric boundary, from the rocprofv3 --pmc
    runs summarised in profiles/traffic.json (written by paper_2602_07899_amd/record_traffic.py);
    None unless that record was taken from exactly this source tree."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path))
    if rec.get("source_fingerprint") != source_fingerprint():
        return None
    return rec.get("gemm_loss_bytes_per_launch", {}).get(workload_name)


def host_cores():
    try:
        from threadpoolctl import threadpool_info
        return int(max([i.get("num_threads", 1) for i in threadpool_info()] or [os.cpu_count() or 1]))
    except Exception:
        return int(os.cpu_count() or 1)


def resident_inputs(wl, tlq, torch, workload, dev, p, want_abs_sum_of=None):
    """Draw every linear's inputs from the seeded per-sample generators (host threads), place
    them in HBM and form Y_ref with the library's own f_fp GEMM.  Returns the per-linear
    tuples and, for linear `want_abs_sum_of`, the float64 column sums of |X| (the oracle's
    x_stat numerator, accumulated while the samples pass through the host)."""
    import numpy as np
    per = workload.n_vis + workload.n_txt
    layers, abs_sum = [], None
    for li, spec in enumerate(workload.linears):
        X = torch.empty((workload.n_tok, spec.c_in), dtype=torch.float16, device=dev)
        keep = li == want_abs_sum_of
        if keep:
            abs_sum = np.zeros(spec.c_in, np.float64)

        def one(b):
            xb = wl.make_sample_tokens(workload, li, b).astype(np.float16)
            return b, xb, (np.abs(xb.astype(np.float64)).sum(axis=0) if keep else None)

        with cf.ThreadPoolExecutor(HOST_THREADS) as ex:
            for b, xb, s in ex.map(one, range(workload.n_samples)):
                X[b * per:(b + 1) * per].copy_(torch.from_numpy(xb))
                if keep:
                    abs_sum += s
        W = torch.from_numpy(wl.make_weight(workload, li)).to(dev)
        w = torch.from_numpy(wl.make_token_weights(workload, li)).to(dev)
        Y = torch.empty((workload.n_tok, spec.c_out), dtype=torch.float16, device=dev)
        tlq.ref_output(X, W, Y, p)
        out = (torch.empty(spec.c_in, dtype=torch.float32, device=dev),
               torch.empty(1, dtype=torch.int32, device=dev),
               torch.empty(workload.n_alpha, dtype=torch.float32, device=dev))
        layers.append((spec, X, W, Y, w, out))
        log(f"{workload.name}: inputs of {spec.name} resident")
    return layers, abs_sum


def timed_workload(wl, tlq, torch, workload, layers, p, al, workspace, steps, warmup, act_bits):
    """W warm-up steps, then exactly K timed steps bracketed by device synchronisation; HIP
    events around every kernel on the launch stream give the per-kernel figures."""
    def step():
        for spec, X, W, Y, w, (best, idx, losses) in layers:
            tlq.scale_search(X, W, Y, w, al, p, best, idx, losses, workspace=workspace)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    tlq.profile_reset()
    tlq.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tlq.profile_enable(False)
    kernels = {k.name: k for k in tlq.profile_read()}

    per_linear = []
    for spec, X, W, Y, w, (best, idx, losses) in layers:
        ms = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            tlq.scale_search(X, W, Y, w, al, p, best, idx, losses, workspace=workspace)
            e1.record()
            e1.synchronize()
            ms.append(e0.elapsed_time(e1))
        m = sorted(ms)[1]
        per_linear.append({"linear": f"{spec.name}:{spec.c_out}x{spec.c_in}", "ms_per_search": round(m, 4),
                           "evals_per_s": workload.n_alpha / (m * 1e-3),
                           "search_tflops": 2.0 * workload.n_tok * spec.c_in * spec.c_out * workload.n_alpha
                                            / (m * 1e-3) / 1e12})
    evals = len(layers) * workload.n_alpha * steps
    g = kernels["gemm_loss"]
    tflops = g.total_work / (g.total_ms * 1e-3) / 1e12
    return {
        "value": evals / dt, "ms_per_step": dt / steps * 1e3,
        "config": {"workload": workload.name,
                   "linears": [f"{s.name}:{s.c_out}x{s.c_in}" for s in workload.linears],
                   "n_tok": workload.n_tok, "bits": workload.bits, "group": workload.group,
                   "n_alpha": workload.n_alpha, "evals_per_step": len(layers) * workload.n_alpha,
                   "act_bits": act_bits},
        "fused_kernel_tflops": tflops, "pct_fp16_mfma_peak": 100.0 * tflops / PEAK_FP16_TFLOPS,
        "roofline": {"bound": "mfma", "kernel": "gemm_loss", "achieved": tflops, "peak": PEAK_FP16_TFLOPS,
                     "unit": "TFLOP/s", "frac": tflops / PEAK_FP16_TFLOPS,
                     "avg_launch_ms": g.total_ms / g.launches, "flops_per_launch": g.total_work / g.launches,
                     "traffic": recorded_traffic(workload.name) if act_bits == 0 else None},
        "kernels": {k.name: {"launches": k.launches, "ms": round(k.total_ms, 4),
                             "rate": (k.total_work / (k.total_ms * 1e-3) / 1e9) if k.total_ms > 0 else None,
                             "rate_unit": "GFLOP/s" if k.name.startswith("gemm") else "GB/s"}
                    for k in kernels.values()},
        "per_linear": per_linear,
        "best_alpha_index": [int(l[5][1].item()) for l in layers],
    }


def second_moment_leg(tlq, torch, workload, layers, p, al, steps, warmup):
    """The same searches in the second-moment form (tlq_token_gram + tlq_scale_search_gram): one
    step = for every linear its channel statistic, the weighted second-moment matrix of its
    tokens and the 20-candidate search through it.  (A real layer shares the matrix between q/k/v
    and between gate/up; here every linear has its own synthetic input, so each pays for its
    own.)  Reported next to the headline, never as `value`: it does not run the tokens through
    every candidate.  Its losses are compared with those of the token form on the same inputs."""
    import numpy as np
    dev = layers[0][1].device
    n_tok = workload.n_tok
    cmax = max(s.c_in for s in workload.linears)
    gram = torch.empty(tlq.token_gram_bytes(cmax), dtype=torch.uint8, device=dev)
    ws = torch.empty(max(max(tlq.token_gram_workspace_bytes(n_tok, s.c_in), tlq.x_stat_workspace_bytes(n_tok, s.c_in),
                             tlq.scale_search_gram_workspace_bytes(s.c_in, s.c_out, workload.n_alpha, p))
                         for s in workload.linears), dtype=torch.uint8, device=dev)
    outs = [(torch.empty(s.c_in, dtype=torch.float32, device=dev), torch.empty_like(o[0]), torch.empty_like(o[1]),
             torch.empty_like(o[2])) for s, _, _, _, _, o in layers]

    def step():
        for (spec, X, W, Y, w, _), (xs, best, idx, losses) in zip(layers, outs):
            tlq.x_stat(X, p, xs, workspace=ws)
            g = tlq.token_gram(X, w, p, gram[:tlq.token_gram_bytes(spec.c_in)], workspace=ws)
            tlq.scale_search_gram(g, W, al, p, xs, best, idx, losses, workspace=ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    tlq.profile_reset()
    tlq.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tlq.profile_enable(False)
    kernels = {k.name: k for k in tlq.profile_read()}
    rel, same = 0.0, True
    for (_, _, _, _, _, (_, idx_t, l_t)), (_, _, idx_g, l_g) in zip(layers, outs):
        a, b = l_t.cpu().numpy().astype(np.float64), l_g.cpu().numpy().astype(np.float64)
        rel = max(rel, float(np.max(np.abs(a - b) / a)))
        same = same and int(idx_t.item()) == int(idx_g.item())
    return {"value": len(layers) * workload.n_alpha * steps / dt, "unit": "evals/s", "ms_per_step": dt / steps * 1e3,
            "max_rel_vs_token_form": rel, "same_choices": same,
            "kernels": {k.name: {"launches": k.launches, "ms": round(k.total_ms, 4),
                                 "rate": (k.total_work / (k.total_ms * 1e-3) / 1e9) if k.total_ms > 0 else None,
                                 "rate_unit": "GFLOP/s" if k.name.startswith("gemm") else "GB/s"}
                        for k in kernels.values()}}


def oracle_leg(wl, tlq, torch, orc, workload, dev, p, n_samples, cands, x_abs_sum):
    """The oracle, as it stands, timed on a bounded sample of the workload's first linear:
    the first `n_samples` calibration samples and the candidates `cands` of the grid, with the
    channel statistic of ALL tokens.  The library then searches the same inputs (X, W, the
    oracle's Y_ref, token weights, the oracle's x_stat) and the two sets of losses are compared.
    evals/s counts full-size-equivalent candidate evaluations: candidates x (tokens in the
    sample / tokens of the workload) per second - an extrapolation unless the sample is whole."""
    import numpy as np
    li = 0
    spec = workload.linears[li]
    per = workload.n_vis + workload.n_txt
    n = n_samples * per
    X = wl.make_tokens(workload, li, samples=range(n_samples))
    W = wl.make_weight(workload, li)
    w = wl.make_token_weights(workload, li)[:n]
    al = wl.alpha_grid(workload.n_alpha)[list(cands)]
    x_stat = (x_abs_sum / np.float64(workload.n_tok)).astype(np.float32)   # definition of x_stat_mean, streamed
    if n == workload.n_tok:
        assert np.array_equal(x_stat, orc.x_stat_mean(X))
    Y = orc.ref_output(X, W).astype(np.float16)
    t0 = time.perf_counter()
    ref = orc.scale_search(X, W, Y, w, workload.bits, workload.group, al, x_stat=x_stat)
    dt = time.perf_counter() - t0
    frac = n / workload.n_tok
    whole = n == workload.n_tok
    base = {"value": len(cands) * frac / dt, "unit": "evals/s", "cores": host_cores(), "kind": "oracle",
            "extrapolated": not whole,
            "sample": f"{workload.name} {spec.name} {spec.c_out}x{spec.c_in}, "
                      f"{n} of {workload.n_tok} tokens ({'all' if whole else 'the first'} {n_samples} samples), "
                      f"{len(cands)} of {workload.n_alpha} candidates, {dt:.1f} s of numpy fp64"
                      + ("" if whole else f"; scaled by {frac:.5f} to full-size evaluations")}
    # the library on exactly these inputs
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    best = torch.empty(spec.c_in, dtype=torch.float32, device=dev)
    idx = torch.empty(1, dtype=torch.int32, device=dev)
    losses = torch.empty(len(cands), dtype=torch.float32, device=dev)
    tlq.scale_search(t(X), t(W), t(Y), t(w), t(al), p, best, idx, losses, x_stat_in=t(x_stat))
    torch.cuda.synchronize()
    got = losses.cpu().numpy().astype(np.float64)
    rel = np.abs(got - ref["losses"]) / ref["losses"]
    order = np.sort(ref["losses"])
    near_tie = len(order) > 1 and (order[1] - order[0]) <= 1e-3 * order[0]
    parity = {"parity_max_rel": float(rel.max()), "tolerance": 1e-3, "candidates": len(cands), "tokens": n,
              "same_choice": bool(int(idx.item()) == ref["best_idx"]) or bool(near_tie),
              "scales_equal": bool(np.array_equal(best.cpu().numpy(), ref["best_scales"]))
                              if int(idx.item()) == ref["best_idx"] else None}
    return base, parity


def stack_leg(torch, n_blocks=2):
    """Config 5 in short: the first `n_blocks` decoder blocks of the 13B-class stack (bf16 activations,
    W4 g128, PassAct2, 153,600 tokens, 7 linears x 20 alphas per block) calibrated sequentially
    by the stack driver, once per search form.  The 40 blocks of the full stack have identical
    shapes, so the 40-block figure is the per-block time x 40 (labelled as extrapolated; the
    full runs are in profiles/stack_cfg5_13b.md)."""
    from paper_2602_07899_amd import run_stack
    out = {"stack": "cfg5_13b_stack", "bits": 4, "blocks_run": n_blocks, "extrapolated_to_blocks": 40}
    for strategy in ("tokens", "gram"):
        r = run_stack.run("cfg5_13b_stack", 4, mode="passact2", n_layers=n_blocks, strategy=strategy,
                          log=lambda m: log(m.replace("[run_stack] ", "stack: ")))
        out[strategy] = {"wall_s": r["wall_s"], "s_per_block": r["wall_s"] / n_blocks,
                         "wall_s_40_blocks_extrapolated": r["wall_s"] / n_blocks * 40,
                         "search_kernels_s": r["search_kernels_s"], "propagate_kernels_s": r["propagate_kernels_s"],
                         "block_kernels_s": r["block_kernels_s"], "h_finite": r["h_finite"],
                         "best_idx_first_block": r["blocks"][0]["best_idx"]}
        torch.cuda.empty_cache()
    return out


def mfma_ceiling():
    """Context for the roofline fraction: what a register-only fp16 MFMA loop
    sustains on this device with constant and with pseudo-random operands."""
    import subprocess
    exe = os.path.join(ROOT, "paper_2602_07899_amd", "mfma_ceiling")
    if not os.path.exists(exe):
        return None
    try:
        r = subprocess.run([exe], capture_output=True, text=True, timeout=60)
        return json.loads(r.stdout.strip().splitlines()[-1]) if r.returncode == 0 else None
    except Exception:
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--act-bits", type=int, default=0,
                    help="also quantise activations per token inside every candidate (the paper's "
                         "W4A8 / W4A6 objective); 0 = the weight-only headline workload")
    ap.add_argument("--workload", default="cfg4_13b_w4", choices=("cfg4_13b_w4", "cfg2_7b_w4"),
                    help="headline workload; the default run also times cfg2_7b_w4 as a secondary block")
    ap.add_argument("--no-secondary", action="store_true", help="skip the secondary workload")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing and parity legs")
    ap.add_argument("--no-second-moment", action="store_true",
                    help="skip the second-moment-form leg (the same searches through the token Gram matrix)")
    ap.add_argument("--no-stack", action="store_true",
                    help="skip the short sequential-stack leg (two blocks of the 13B-class stack per search form)")
    ap.add_argument("--no-ceiling", action="store_true",
                    help="skip the register-only MFMA ceiling measurement (context only)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2602_07899_amd import tlq
    from paper_2602_07899_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    oracle_on = not args.no_cpu_baseline and args.act_bits == 0
    # bounded oracle samples: (calibration samples, candidates) - about 10-20 s of numpy fp64 each
    ORACLE_SAMPLE = {"cfg4_13b_w4": (8, tuple(range(0, 20, 2))), "cfg2_7b_w4": (16, tuple(range(20)))}

    def run(name):
        workload = wl.CONFIGS[name]
        p = tlq.params(bits=workload.bits, group=workload.group, act_bits=args.act_bits, x_dtype=tlq.F16,
                       yref_dtype=tlq.F16)
        al = torch.from_numpy(wl.alpha_grid(workload.n_alpha)).to(dev)
        layers, abs_sum = resident_inputs(wl, tlq, torch, workload, dev, p, want_abs_sum_of=0 if oracle_on else None)
        ws_bytes = max(tlq.scale_search_workspace_bytes(workload.n_tok, s.c_in, s.c_out, workload.n_alpha, p)
                       for s in workload.linears)
        workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        # one device-to-device copy of known size (reads and writes 83,886,080 bytes): the
        # calibration kernel for the FETCH_SIZE / WRITE_SIZE counters in profiling runs
        src = layers[0][1].view(-1)[:41943040]
        torch.empty_like(src).copy_(src)
        torch.cuda.synchronize()
        res = timed_workload(wl, tlq, torch, workload, layers, p, al, workspace, args.steps, args.warmup,
                             args.act_bits)
        log(f"{name}: {res['value']:.1f} evals/s, gemm_loss {res['fused_kernel_tflops']:.1f} TFLOP/s")
        if args.act_bits == 0 and not args.no_second_moment:
            res["second_moment_form"] = second_moment_leg(tlq, torch, workload, layers, p, al, args.steps, args.warmup)
            log(f"{name}: second-moment form {res['second_moment_form']['value']:.1f} evals/s, "
                f"max rel vs token form {res['second_moment_form']['max_rel_vs_token_form']:.2e}")
        if oracle_on:
            from oracle import tlq_oracle as orc
            ns, cands = ORACLE_SAMPLE[name]
            p0 = tlq.params(bits=workload.bits, group=workload.group, x_dtype=tlq.F16, yref_dtype=tlq.F16)
            res["cpu_baseline"], res["parity"] = oracle_leg(wl, tlq, torch, orc, workload, dev, p0, ns, cands, abs_sum)
            log(f"{name}: oracle {res['cpu_baseline']['value']:.4f} evals/s, parity_max_rel "
                f"{res['parity']['parity_max_rel']:.2e}")
        del layers, workspace
        torch.cuda.empty_cache()
        return res

    head = run(args.workload)
    result = {
        "metric": METRIC, "value": head["value"], "unit": "evals/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
    }
    for k in ("config", "fused_kernel_tflops", "pct_fp16_mfma_peak", "roofline", "cpu_baseline", "parity",
              "kernels", "per_linear", "best_alpha_index", "second_moment_form"):
        if k in head:
            result[k] = head[k]
    if not args.no_secondary:
        other = "cfg2_7b_w4" if args.workload == "cfg4_13b_w4" else "cfg4_13b_w4"
        sec = run(other)
        sec["unit"] = "evals/s"
        result["secondary"] = sec
    if args.act_bits == 0 and not args.no_stack:
        result["stack"] = stack_leg(torch)
    result["peak_hbm_bytes"] = int(torch.cuda.max_memory_allocated())
    result["source_fingerprint"] = source_fingerprint()
    # the paper publishes no speed figure for this path; its cost figures are about memory
    result["paper_context"] = ("paper (Sec. 3.2.2 and its memory table): calibrating a 7B VLM on 128 samples takes one "
                               "A100-80GB with the prior layer-wise method and 3 x RTX3090-24GB with its distributed "
                               "split (7.1-18.8 GB peak per GPU); no calibration time, throughput or kernel timing is given")
    if not args.no_ceiling:
        result["mfma_ceiling"] = mfma_ceiling()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
