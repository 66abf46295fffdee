"""Seeded synthetic calibration inputs (shapes and value distributions only).

These generators stand in for the paper's calibration data (128 image-caption
samples, Sec. 4.1) and model weights, neither of which is available offline.
They hold none of the method's arithmetic: they only draw random tensors with
the structure of vision-language calibration activations - many "visual"
tokens followed by a few "text" tokens per sample, a small fixed set of
outlier channels that are much larger on text tokens than on visual ones, and
token-importance weights that are heavy-tailed on visual tokens and larger on
text tokens.  Both the CPU oracle's tests and the GPU path's tests and
benchmark draw their inputs from here.

Every sample is drawn from its own counter-derived generator
(seed, stream id, sample index), so any subset of samples can be regenerated
without producing the whole tensor.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


def alpha_grid(n: int = 20) -> np.ndarray:
    """alpha_k = k / n, k = 0..n-1, as float32 (n points in [0, 1))."""
    return (np.arange(n, dtype=np.float64) / n).astype(np.float32)


@dataclass(frozen=True)
class LinearSpec:
    name: str
    c_out: int
    c_in: int


@dataclass(frozen=True)
class Workload:
    """One synthetic calibration workload (a set of linear layers that see
    n_samples * (n_vis + n_txt) tokens)."""
    name: str
    linears: tuple
    n_samples: int
    n_vis: int
    n_txt: int
    bits: int = 4
    group: int = 128
    n_alpha: int = 20
    seed: int = 0
    w_std: float = 0.02
    # outlier channels: explicit count, or a fraction of c_in
    n_outlier: int | None = None
    outlier_frac: float = 0.01
    txt_mult: float = 30.0
    vis_mult: float = 5.0
    # token-weight recipe: "uniform" (config 1) or "lognormal" (configs 2-5)
    weight_kind: str = "lognormal"
    act_dtype: str = "f16"

    @property
    def n_tok(self) -> int:
        return self.n_samples * (self.n_vis + self.n_txt)


LLAMA7B = (LinearSpec("q_proj", 4096, 4096), LinearSpec("k_proj", 4096, 4096),
           LinearSpec("v_proj", 4096, 4096), LinearSpec("o_proj", 4096, 4096),
           LinearSpec("gate_proj", 11008, 4096), LinearSpec("up_proj", 11008, 4096),
           LinearSpec("down_proj", 4096, 11008))
LLAMA13B = (LinearSpec("q_proj", 5120, 5120), LinearSpec("k_proj", 5120, 5120),
            LinearSpec("v_proj", 5120, 5120), LinearSpec("o_proj", 5120, 5120),
            LinearSpec("gate_proj", 13824, 5120), LinearSpec("up_proj", 13824, 5120),
            LinearSpec("down_proj", 5120, 13824))

CONFIGS = {
    # single small layer: the full-parity case the oracle finishes in under a second
    "cfg1_small": Workload("cfg1_small", (LinearSpec("linear", 512, 512),), n_samples=1,
                           n_vis=192, n_txt=64, bits=4, n_outlier=4, txt_mult=20.0,
                           vis_mult=1.0, weight_kind="uniform"),
    # 7B-class decoder layer, 16 samples x 640 tokens, W4 g128: the benchmark workload
    "cfg2_7b_w4": Workload("cfg2_7b_w4", LLAMA7B, n_samples=16, n_vis=576, n_txt=64, bits=4),
    # same shapes, W3, 64 samples
    "cfg3_7b_w3": Workload("cfg3_7b_w3", LLAMA7B, n_samples=64, n_vis=576, n_txt=64, bits=3),
    # scaled-down 7-linear chain (hidden 512, ffn 1408) for full-oracle parity of the
    # quantisation-exposed sequential calibration
    "cfg3_mini_w3": Workload("cfg3_mini_w3", (LinearSpec("q_proj", 512, 512), LinearSpec("k_proj", 512, 512),
                                              LinearSpec("v_proj", 512, 512), LinearSpec("o_proj", 512, 512),
                                              LinearSpec("gate_proj", 1408, 512), LinearSpec("up_proj", 1408, 512),
                                              LinearSpec("down_proj", 512, 1408)),
                             n_samples=5, n_vis=96, n_txt=32, bits=3, n_alpha=8, n_outlier=5),
    # 13B-class shapes, 128 samples x 1200 tokens
    "cfg4_13b_w4": Workload("cfg4_13b_w4", LLAMA13B, n_samples=128, n_vis=1152, n_txt=48, bits=4),
}


@dataclass(frozen=True)
class StackWorkload:
    """A stack of synthetic decoder blocks calibrated in sequence: hidden width
    n_heads*128, every block holding the 7 linears q, k, v, o, gate, up, down."""
    name: str
    n_layers: int
    n_heads: int
    ffn: int
    n_samples: int
    n_vis: int
    n_txt: int
    bits: tuple = (4, 3)
    group: int = 128
    n_alpha: int = 20
    seed: int = 0
    w_std: float = 0.02
    n_outlier: int | None = None
    outlier_frac: float = 0.01
    txt_mult: float = 30.0
    vis_mult: float = 5.0
    act_dtype: str = "bf16"

    @property
    def hidden(self) -> int:
        return self.n_heads * 128

    @property
    def seq_len(self) -> int:
        return self.n_vis + self.n_txt

    @property
    def n_tok(self) -> int:
        return self.n_samples * self.seq_len

    def shapes(self) -> tuple:
        d, f = self.hidden, self.ffn
        return ((d, d), (d, d), (d, d), (d, d), (f, d), (f, d), (d, f))

    def as_workload(self) -> Workload:
        """The token/importance recipe of the stack's embedding, as a one-linear workload."""
        return Workload(self.name, (LinearSpec("embed", self.hidden, self.hidden),), n_samples=self.n_samples,
                        n_vis=self.n_vis, n_txt=self.n_txt, seed=self.seed, n_outlier=self.n_outlier,
                        outlier_frac=self.outlier_frac, txt_mult=self.txt_mult, vis_mult=self.vis_mult)


STACKS = {
    # 13B-class: 40 blocks, hidden 5120 (40 heads), ffn 13824, 128 samples x 1200 tokens, bf16, W4 then W3
    "cfg5_13b_stack": StackWorkload("cfg5_13b_stack", n_layers=40, n_heads=40, ffn=13824, n_samples=128,
                                    n_vis=1152, n_txt=48),
    # scaled-down stack for full-oracle parity: 2 blocks, hidden 256 (2 heads), ffn 384, 3 x 72 tokens
    "cfg5_mini_stack": StackWorkload("cfg5_mini_stack", n_layers=2, n_heads=2, ffn=384, n_samples=3, n_vis=48,
                                     n_txt=24, n_alpha=6, n_outlier=3, w_std=0.06),
}


def make_stack_weights(sw: StackWorkload, layer: int) -> list:
    """The 7 weight matrices of one block, float32 values ~ N(0, w_std^2) (the caller
    rounds them to the activation type); seeded per (stack seed * 1000 + layer, linear)."""
    out = []
    for li, (co, ci) in enumerate(sw.shapes()):
        g = _rng(sw.seed * 1000 + layer, 2000 + li, 0)
        out.append(g.standard_normal((co, ci), dtype=np.float32) * np.float32(sw.w_std))
    return out


def _rng(seed: int, stream: int, index: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(stream), int(index)])


def outlier_channels(wl: Workload, lin_idx: int) -> np.ndarray:
    """Fixed sorted set of outlier channel indices for one linear's input."""
    c_in = wl.linears[lin_idx].c_in
    n = wl.n_outlier if wl.n_outlier is not None else int(round(wl.outlier_frac * c_in))
    return np.sort(_rng(wl.seed, 1000 + lin_idx, 0).choice(c_in, size=n, replace=False))


def make_weight(wl: Workload, lin_idx: int) -> np.ndarray:
    """W [c_out, c_in] fp16 ~ N(0, w_std^2)."""
    spec = wl.linears[lin_idx]
    g = _rng(wl.seed, 2000 + lin_idx, 0)
    w = g.standard_normal((spec.c_out, spec.c_in), dtype=np.float32) * np.float32(wl.w_std)
    return w.astype(np.float16)


def make_sample_tokens(wl: Workload, lin_idx: int, sample: int) -> np.ndarray:
    """Activations of one calibration sample: [n_vis + n_txt, c_in] float32,
    visual tokens first, then text tokens, outlier channels amplified."""
    spec = wl.linears[lin_idx]
    g = _rng(wl.seed, 3000 + lin_idx, sample)
    x = g.standard_normal((wl.n_vis + wl.n_txt, spec.c_in), dtype=np.float32)
    oc = outlier_channels(wl, lin_idx)
    if wl.vis_mult != 1.0:
        x[: wl.n_vis, oc] *= np.float32(wl.vis_mult)
    x[wl.n_vis:, oc] *= np.float32(wl.txt_mult)
    return x


def make_tokens(wl: Workload, lin_idx: int, samples=None) -> np.ndarray:
    """X [n_tok, c_in] fp16 for all (or the listed) samples."""
    idx = range(wl.n_samples) if samples is None else samples
    return np.concatenate([make_sample_tokens(wl, lin_idx, b).astype(np.float16) for b in idx], axis=0)


def make_token_weights(wl: Workload, lin_idx: int) -> np.ndarray:
    """w_t [n_tok] float32, non-negative, normalised to sum 1 (in float64,
    then rounded)."""
    per = wl.n_vis + wl.n_txt
    w = np.empty((wl.n_samples, per), dtype=np.float64)
    for b in range(wl.n_samples):
        g = _rng(wl.seed, 4000 + lin_idx, b)
        if wl.weight_kind == "uniform":
            w[b, : wl.n_vis] = g.uniform(0.1, 1.0, wl.n_vis)
            w[b, wl.n_vis:] = g.uniform(1.0, 5.0, wl.n_txt)
        else:
            w[b, : wl.n_vis] = g.lognormal(0.0, 1.0, wl.n_vis)
            w[b, wl.n_vis:] = 4.0 * g.lognormal(0.0, 1.0, wl.n_txt)
    w = w.reshape(-1)
    return (w / w.sum()).astype(np.float32)


def chain_multipliers(wl: Workload, lin_idx: int) -> tuple:
    """Per-channel multipliers (visual rows, text rows) that re-impose the outlier
    channels on the exposed input of linear `lin_idx` in the sequential chain."""
    c_in = wl.linears[lin_idx].c_in
    mv = np.ones(c_in, dtype=np.float32)
    mt = np.ones(c_in, dtype=np.float32)
    oc = outlier_channels(wl, lin_idx)
    mv[oc] = wl.vis_mult
    mt[oc] = wl.txt_mult
    return mv, mt


def token_rows(wl: Workload, rows) -> tuple:
    """Map global token rows to (sample, offset) pairs."""
    per = wl.n_vis + wl.n_txt
    rows = np.asarray(rows, dtype=np.int64)
    return rows // per, rows % per


def make_token_subset(wl: Workload, lin_idx: int, rows) -> np.ndarray:
    """X[rows, :] fp16 regenerated from the per-sample generators."""
    samp, off = token_rows(wl, rows)
    out = np.empty((len(samp), wl.linears[lin_idx].c_in), dtype=np.float16)
    for b in np.unique(samp):
        xs = make_sample_tokens(wl, lin_idx, int(b)).astype(np.float16)
        sel = samp == b
        out[sel] = xs[off[sel]]
    return out


def tiny_layer(seed: int, n_tok: int, c_in: int, c_out: int, n_outlier: int = 1,
               mult: float = 8.0):
    """Very small dense problem for brute-force checks: returns
    (X fp16 [n_tok,c_in], W fp16 [c_out,c_in], w float32 [n_tok])."""
    g = _rng(seed, 9000, 0)
    X = g.standard_normal((n_tok, c_in), dtype=np.float32)
    if n_outlier:
        X[:, g.choice(c_in, size=n_outlier, replace=False)] *= np.float32(mult)
    W = g.standard_normal((c_out, c_in), dtype=np.float32) * np.float32(0.05)
    w = g.uniform(0.1, 1.0, n_tok)
    return X.astype(np.float16), W.astype(np.float16), (w / w.sum()).astype(np.float32)
