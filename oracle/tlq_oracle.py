"""CPU oracle for the TLQ layer-wise scale search (test infrastructure only).

This module is the plain, slow, obviously-correct definition of what the GPU
library computes.  It is *test infrastructure*: only tests, the smoke check
and the benchmark's cpu_baseline leg may import it.  It shares no code with
the HIP path and imports nothing from the product package.

Everything follows the paper's Method section:

  * scale = x_stat ** r, one value per input channel  (Sec. 3.1.2, the
    "scale" equation; r is called alpha here and in the C ABI);
  * the per-layer objective  r* = argmin_r E || f_fp(x) - f_q(x; scale) ||^2
    (Sec. 3.2.1, first two equations);
  * f_fp(x) = W x + b ,  f_q(x; scale) = Q_w(W * scale) Q_a(x / scale) + b
    (Sec. 3.2.1, third/fourth equations) with Q_a = identity (weight-only
    setting of this build), so the bias cancels in the residual;
  * the per-channel smoothing identity Y = (X diag(scale)^-1)(diag(scale) W)
    (Sec. 2.2, smoothing equation);
  * round-to-nearest integer quantisation (Sec. 2.2, first two equations); the
    paper writes out the symmetric form and says the asymmetric one follows
    the same way - the asymmetric min/max form used here is spelled out in
    ``fake_quant`` below;
  * PassAct2 propagation  x^(l) = f_q^(l-1)(x^(l-1); scale^(l-1))
    (Sec. 3.2.1, PassAct2 equation).

Precision: the contraction and the loss are evaluated in float64.  The
quantiser's grid parameters (step, zero point) and the integer codes are
evaluated in float32 with one rounding per operation, because the task fixes
"the same fp32 scale formula" on both sides so that integer codes can be
compared bit for bit.

Readings of points the paper leaves open (each is also listed in the design
notes of the repository):
  - x_stat is the plain mean of |x| over all tokens (the "x_mean" base row of
    the ablation table); any other statistic can be passed in explicitly.
  - x_stat is floored at 2**-14 before the power so that dead channels do not
    give a zero scale; alpha = 0 still gives exactly 1.
  - the expectation in the objective is  sum_t w_t * mean_o (residual^2) with
    caller-supplied token weights; w_t = 1/N gives the plain elementwise MSE.
  - W is [C_out, C_in]; scale multiplies columns of W and divides columns of X.
  - ties between candidates resolve to the smallest alpha; a candidate whose
    loss is not finite is reported as +inf and never selected.
  - activation quantisation (act_bits > 0): x/scale is formed in float32 as
    x * float32(1/scale), the per-token step uses max|.| floored at 1e-5.

Parity pins (see tests/test_oracle_pins.py): brute force on tiny layers
(oracle/brute.py), hand-worked quantiser example (tests/golden), alpha=0 and
alpha=1 closed forms, uniform-weight MSE, smoothing identity with an identity
quantiser, grid idempotence, Delta^2/12 error energy (Sec. 2.2), power-of-two
scale invariance, max-code closed form for the symmetric variant, the
quadratic-form identity of the token second-moment matrix.
Every function of this module has at least one such pin; the sequential-chain
module (oracle/chain.py) is pinned by tests/test_oracle_chain_pins.py and the
decoder-stack module (oracle/stack.py) by tests/test_oracle_stack_pins.py.  Not pinned, and not
pinnable here: that these definitions reproduce the paper's downstream accuracy
tables - that needs the trained models and evaluation suites (parity unpinned
for accuracy).
"""
from __future__ import annotations

import numpy as np

XSTAT_FLOOR = np.float32(2.0 ** -14)
RANGE_FLOOR = np.float32(1e-5)

_F32 = np.float32


def to_f64(a):
    """Exact widening of an fp16 / bf16-as-fp32 / fp32 array to float64."""
    return np.asarray(a).astype(np.float64)


# --------------------------------------------------------------------------
# S0  x_stat
# --------------------------------------------------------------------------
def x_stat_mean(X):
    """x_stat_c = (1/N) sum_t |X[t, c]|   (Sec. 3.1.2 x_stat, mean variant of
    the ablation table).  Sum in float64 (exact for fp16 inputs at the sizes
    used here), one division, one rounding to float32."""
    X = to_f64(X)
    n = X.shape[0]
    return (np.abs(X).sum(axis=0) / np.float64(n)).astype(np.float32)


def x_stat_max(X, token_mask=None):
    """x_stat_c = max_{i in I} |X[i, c]|   (Sec. 3.1.2, x_stat equation).
    ``token_mask`` selects the important-token set I; None means all tokens
    (the "x_max" row of the ablation table)."""
    X = np.abs(to_f64(X))
    if token_mask is not None:
        X = X[np.asarray(token_mask, dtype=bool)]
    return X.max(axis=0).astype(np.float32)


def token_importance(G, n_samples, l2=False):
    """sum_n = sum_b || g_{b,n} ||  (Sec. 3.1.2, gradient-statistic equation).
    G: [n_samples * N, C] per-sample gradients w.r.t. the layer input, sample
    major.  The text describes the norm as the absolute values averaged over
    the channel dimension (l2=False, the reading taken); l2=True uses the
    Euclidean norm instead.  float64; returns [N]."""
    G = to_f64(G)
    n_pos = G.shape[0] // n_samples
    G = G.reshape(n_samples, n_pos, -1)
    per = np.sqrt((G * G).sum(axis=2)) if l2 else np.abs(G).mean(axis=2)
    return per.sum(axis=0)


def top_fraction_mask(sum_n, k):
    """I = Top_k({sum_n})  (Sec. 3.1.2, selection equation; the paper keeps the
    top 50 %).  Ties go to the lower position.  Returns a bool mask [N]."""
    sum_n = np.asarray(sum_n)
    order = np.lexsort((np.arange(sum_n.size), -sum_n))   # by value descending, then index
    mask = np.zeros(sum_n.size, dtype=bool)
    mask[order[:k]] = True
    return mask


def x_stat_topk_max(X, pos_mask):
    """x_stat_c = max_{i in I} |X_{i,c}|  (Sec. 3.1.2, x_stat equation) where I is a set of
    token positions and X stacks samples of len(pos_mask) tokens each."""
    X = np.abs(to_f64(X))
    period = len(pos_mask)
    rows = np.asarray(pos_mask, bool)[np.arange(X.shape[0]) % period]
    return X[rows].max(axis=0).astype(np.float32)


# --------------------------------------------------------------------------
# S1  scale table
# --------------------------------------------------------------------------
def scale_table(x_stat, alpha_grid):
    """s[k, c] = max(x_stat_c, floor) ** alpha_k   (Sec. 3.1.2 scale equation,
    Sec. 3.2.1 per-layer form).  float64 pow, rounded once to float32."""
    xs = np.maximum(np.asarray(x_stat, dtype=np.float32), XSTAT_FLOOR).astype(np.float64)
    al = np.asarray(alpha_grid, dtype=np.float32).astype(np.float64)
    return np.power(xs[None, :], al[:, None]).astype(np.float32)


# --------------------------------------------------------------------------
# S2  group-wise asymmetric (and per-row symmetric) fake quantisation
# --------------------------------------------------------------------------
def fake_quant(W, s, bits, group, symmetric=False):
    """Quantise-dequantise W * diag(s) on a per-(row, group) grid.

    W      [C_out, C_in] fp16/bf16/fp32 array (values used exactly)
    s      [C_in] float32 per-input-channel scale, or None for ones
    group  number of consecutive input channels sharing a grid; 0 = whole row

    Asymmetric form (the min/max analogue of Sec. 2.2's quantiser), all in
    float32, one rounding per operation:
        ws    = W * s
        mx,mn = max / min of ws over the group
        rng   = max(mx - mn, 1e-5)
        delta = rng / (2**bits - 1)
        zp    = clip(rint(-mn / delta), 0, 2**bits - 1)
        q     = clip(rint(ws / delta) + zp, 0, 2**bits - 1)
        deq   = (q - zp) * delta
    Symmetric form (Sec. 2.2 first two equations, per row/group):
        delta = max(max|ws|, 1e-5) / (2**(bits-1) - 1)
        q     = clip(rint(ws / delta), -2**(bits-1), 2**(bits-1) - 1)
        deq   = q * delta ; codes are stored offset by 2**(bits-1), zp = 2**(bits-1)
    rint is round-half-to-even.

    Returns codes uint8 [C_out, C_in], zp uint8 [C_out, G], delta float32
    [C_out, G], deq float32 [C_out, C_in].
    """
    W32 = np.asarray(W).astype(np.float32)
    c_out, c_in = W32.shape
    g = c_in if group == 0 else int(group)
    if c_in % g != 0:
        raise ValueError("c_in must be a multiple of group")
    G = c_in // g
    if s is None:
        ws = W32.copy()
    else:
        ws = W32 * np.asarray(s, dtype=np.float32)[None, :]
    ws = ws.reshape(c_out, G, g)
    if not symmetric:
        qmax = _F32(2 ** bits - 1)
        mx = ws.max(axis=2)
        mn = ws.min(axis=2)
        rng = np.maximum(mx - mn, RANGE_FLOOR)
        delta = (rng / qmax).astype(np.float32)
        zp = np.clip(np.rint((-mn) / delta), _F32(0), qmax).astype(np.float32)
        q = np.clip(np.rint(ws / delta[:, :, None]) + zp[:, :, None], _F32(0), qmax)
        q = q.astype(np.float32)
        deq = ((q - zp[:, :, None]) * delta[:, :, None]).astype(np.float32)
    else:
        half = 2 ** (bits - 1)
        amax = np.maximum(np.abs(ws).max(axis=2), RANGE_FLOOR)
        delta = (amax / _F32(half - 1)).astype(np.float32)
        qs = np.clip(np.rint(ws / delta[:, :, None]), _F32(-half), _F32(half - 1)).astype(np.float32)
        deq = (qs * delta[:, :, None]).astype(np.float32)
        zp = np.full((c_out, G), half, dtype=np.float32)
        q = qs + _F32(half)
    codes = q.astype(np.uint8).reshape(c_out, c_in)
    return codes, zp.astype(np.uint8), delta, deq.reshape(c_out, c_in)


def requantise_on_grid(values, delta, zp, bits, group):
    """Codes of ``values`` on an already fixed (delta, zp) grid - used by the
    idempotence pin: quantising dequantised values again must not move them."""
    v = np.asarray(values, dtype=np.float32)
    c_out, c_in = v.shape
    g = c_in if group == 0 else int(group)
    v = v.reshape(c_out, c_in // g, g)
    qmax = _F32(2 ** bits - 1)
    q = np.clip(np.rint(v / delta[:, :, None]) + zp.astype(np.float32)[:, :, None], _F32(0), qmax)
    return q.astype(np.uint8).reshape(c_out, c_in)


# --------------------------------------------------------------------------
# Q_a  per-token symmetric activation fake quantisation
# --------------------------------------------------------------------------
def recip_scale(s):
    """float32( 1 / float64(s) ): the reciprocal both sides multiply by."""
    return (1.0 / np.asarray(s, np.float32).astype(np.float64)).astype(np.float32)


def act_quant(X, inv_s, act_bits):
    """Q_a(x / scale) of Sec. 3.2.1 with the symmetric per-token quantiser of
    Sec. 2.2 (first two equations, X = activations, one step per token row):
        xt      = float32(X) * inv_s                    (float32, one rounding)
        sigma_t = max(max_c |xt[t,c]|, 1e-5) / (2**(n-1) - 1)
        code    = clip(rint(xt / sigma_t), -2**(n-1), 2**(n-1) - 1)
        xhat    = code * sigma_t
    inv_s is the float32 reciprocal of the channel scale (None = ones).  All grid
    arithmetic is float32, one rounding per operation, round-half-to-even.
    Returns codes int16 [N, C], sigma float32 [N]."""
    xt = np.asarray(X).astype(np.float32)
    if inv_s is not None:
        xt = xt * np.asarray(inv_s, np.float32)[None, :]
    half = 2 ** (act_bits - 1)
    amax = np.maximum(np.abs(xt).max(axis=1), RANGE_FLOOR)
    sigma = (amax / _F32(half - 1)).astype(np.float32)
    codes = np.clip(np.rint(xt / sigma[:, None]), _F32(-half), _F32(half - 1))
    return codes.astype(np.int16), sigma


def quantised_output_aq(X, deq, s, act_bits):
    """f_q with activation quantisation, bias-free, float64:
    Yq[t,o] = sigma_t * sum_c code[t,c] * deq[o,c]   (Sec. 3.2.1 f_q)."""
    codes, sigma = act_quant(X, None if s is None else recip_scale(s), act_bits)
    return (codes.astype(np.float64) @ to_f64(deq).T) * sigma.astype(np.float64)[:, None]


# --------------------------------------------------------------------------
# S3 / S4  quantised layer output and the weighted objective
# --------------------------------------------------------------------------
def ref_output(X, W):
    """f_fp without bias: Y = X W^T in float64 (Sec. 3.2.1 f_fp)."""
    return to_f64(X) @ to_f64(W).T


def quantised_output(X, deq, s=None, inv_s=None):
    """f_q without bias and with Q_a = identity:
    Yq = (X diag(s)^-1) deq^T  in float64 (Sec. 3.2.1 f_q, Sec. 2.2 smoothing).
    Exactly one of ``s`` (divide) / ``inv_s`` (multiply) may be given."""
    Xs = to_f64(X)
    if s is not None:
        Xs = Xs / to_f64(s)[None, :]
    elif inv_s is not None:
        Xs = Xs * to_f64(inv_s)[None, :]
    return Xs @ to_f64(deq).T


def per_token_err(Y_ref, Yq):
    """e_t = (1/C_out) sum_o (Y_ref[t,o] - Yq[t,o])^2, float64."""
    d = to_f64(Y_ref) - Yq
    return (d * d).sum(axis=1) / np.float64(d.shape[1])


def weighted_layer_err(X, deq, Y_ref, token_w, s=None, inv_s=None):
    """L = sum_t w_t e_t  (Sec. 3.2.1 objective; the expectation is the
    w-weighted sum over tokens).  Returns (L, e) in float64."""
    e = per_token_err(Y_ref, quantised_output(X, deq, s=s, inv_s=inv_s))
    return float((to_f64(token_w) * e).sum()), e


def token_second_moment(X, token_w, rows=None, cols=None):
    """G[i, j] = sum_t w_t x_t[i] x_t[j], float64 (all of it, or the listed rows x cols).

    With Q_a = identity the quantised layer is linear in x, so the objective of Sec. 3.2.1 with
    f_fp(x) = W x is  sum_t w_t (1/C_out) ||(W - What) x_t||^2 = (1/C_out) sum_o d_o^T G d_o  with
    d_o the rows of W - What: this matrix is all the objective needs from the tokens."""
    Xd, w = to_f64(X), to_f64(token_w)
    A = Xd if rows is None else Xd[:, rows]
    B = Xd if cols is None else Xd[:, cols]
    return (A * w[:, None]).T @ B


# --------------------------------------------------------------------------
# S0..S5  the search
# --------------------------------------------------------------------------
def select_best(losses):
    """First minimum over finite losses; -1 if none is finite."""
    L = np.asarray(losses, dtype=np.float64)
    fin = np.isfinite(L)
    if not fin.any():
        return -1
    Lm = np.where(fin, L, np.inf)
    return int(np.argmin(Lm))


def scale_search(X, W, Y_ref, token_w, bits, group, alpha_grid,
                 x_stat=None, s_table=None, symmetric=False, act_bits=0):
    """Exhaustive search over the alpha grid (Sec. 3.2.1).

    Returns dict with s_table [A, C_in] f32, losses [A] f64 (+inf where not
    finite), best_idx, best_scales [C_in] f32, x_stat [C_in] f32.
    ``s_table`` may be supplied to bypass the pow step (used when comparing
    integer codes against a device that evaluated pow itself)."""
    if x_stat is None:
        x_stat = x_stat_mean(X)
    if s_table is None:
        s_table = scale_table(x_stat, alpha_grid)
    A = s_table.shape[0]
    losses = np.empty(A, dtype=np.float64)
    for k in range(A):
        _, _, _, deq = fake_quant(W, s_table[k], bits, group, symmetric=symmetric)
        if act_bits:
            e = per_token_err(Y_ref, quantised_output_aq(X, deq, s_table[k], act_bits))
            L = float((to_f64(token_w) * e).sum())
        else:
            L, _ = weighted_layer_err(X, deq, Y_ref, token_w, s=s_table[k])
        losses[k] = L if np.isfinite(L) else np.inf
    best = select_best(losses)
    best_scales = s_table[best].copy() if best >= 0 else np.full(s_table.shape[1], np.nan, np.float32)
    return {"x_stat": np.asarray(x_stat, np.float32), "s_table": s_table, "losses": losses,
            "best_idx": best, "best_scales": best_scales}


def apply_best(X, W, s, bits, group, symmetric=False, act_bits=0):
    """PassAct2 input of the next layer: f_q(x; scale*) in float64
    (Sec. 3.2.1 PassAct2 equation); the caller casts to its activation type."""
    _, _, _, deq = fake_quant(W, s, bits, group, symmetric=symmetric)
    if act_bits:
        return quantised_output_aq(X, deq, s, act_bits)
    return quantised_output(X, deq, s=s)


# --------------------------------------------------------------------------
# storage rounding helper for bf16 test inputs
# --------------------------------------------------------------------------
def round_to_bf16(a):
    """Round float32 to bfloat16 (round-half-to-even), returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    r = ((u + bias) >> 16) << 16
    out = r.astype(np.uint32).view(np.float32).reshape(a.shape)
    return np.where(np.isnan(a), a, out)
