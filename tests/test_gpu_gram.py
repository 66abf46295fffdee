"""GPU parity of the second-moment form of the weight-only search (tlq_token_gram,
tlq_scale_search_gram) against the CPU oracle: the oracle is the plain definition - the search
of Sec. 3.2.1 with the exact full-precision target f_fp(x) = W x - and, for the intermediate
matrix, the token second moment written out.  Losses within 1e-3 relative, chosen alpha identical
unless the oracle's two best are within that tolerance."""
import numpy as np
import pytest

from oracle import tlq_oracle as orc
from paper_2602_07899_amd import tlq
from paper_2602_07899_amd import workloads as wl

pytestmark = pytest.mark.gpu
LOSS_RTOL = 1e-3


def dev(a, gpu, bf16=False):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if bf16:
        t = t.to(torch.bfloat16)
    return t.to(gpu)


def layer(seed, n_tok, c_in, c_out, bf16=False, txt_every=5, weights="lognormal"):
    """Synthetic layer with the structure of the benchmark inputs: N(0,1) tokens, 1 % outlier
    channels (x5, x30 on every txt_every-th token), N(0, 0.02^2) weights, heavy-tailed token weights."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n_tok, c_in)).astype(np.float32)
    oc = rng.choice(c_in, max(1, c_in // 100), replace=False)
    txt = (np.arange(n_tok) % txt_every) == 0
    X[np.ix_(~txt, oc)] *= 5.0
    X[np.ix_(txt, oc)] *= 30.0
    W = (rng.standard_normal((c_out, c_in)) * 0.02).astype(np.float32)
    if weights == "uniform":
        w = np.full(n_tok, 1.0 / n_tok)
    else:
        w = np.exp(rng.standard_normal(n_tok))
        w[txt] *= 4.0
        w /= w.sum()
    if bf16:
        X, W = orc.round_to_bf16(X), orc.round_to_bf16(W)
    else:
        X, W = X.astype(np.float16), W.astype(np.float16)
    return X, W, w.astype(np.float32)


def gram_search(X_np, W_np, w_np, p, gpu, bf16, alpha):
    import torch
    X, W, w = dev(X_np, gpu, bf16), dev(W_np, gpu, bf16), dev(w_np, gpu)
    n, ci = X.shape
    al = dev(alpha, gpu)
    xs = torch.empty(ci, dtype=torch.float32, device=gpu)
    tlq.x_stat(X, p, xs)
    gram = torch.empty(tlq.token_gram_bytes(ci), dtype=torch.uint8, device=gpu)
    tlq.token_gram(X, w, p, gram)
    best = torch.empty(ci, dtype=torch.float32, device=gpu)
    idx = torch.empty(1, dtype=torch.int32, device=gpu)
    losses = torch.empty(len(alpha), dtype=torch.float32, device=gpu)
    st = torch.empty((len(alpha), ci), dtype=torch.float32, device=gpu)
    tlq.scale_search_gram(gram, W, al, p, xs, best, idx, losses, s_table_out=st)
    torch.cuda.synchronize()
    return gram, xs.cpu().numpy(), losses.cpu().numpy(), int(idx.item()), best.cpu().numpy(), st.cpu().numpy()


def decode_gram(gram, c_in):
    f, cs, C = tlq.gram_views(gram, c_in)
    cs = cs.double().cpu().numpy()
    return float(f.item()) * cs[:, None] * cs[None, :] * C.double().cpu().numpy()


def check_losses(gl, ol, gbest, where):
    gl, ol = np.asarray(gl, np.float64), np.asarray(ol, np.float64)
    rel = np.abs(gl - ol) / ol
    assert np.all(rel < LOSS_RTOL), f"{where}: loss mismatch, max rel {rel.max():.3e}"
    ob = orc.select_best(ol)
    if gbest != ob:
        srt = np.sort(ol)
        assert (srt[1] - srt[0]) / srt[0] < LOSS_RTOL, f"{where}: argmin differs: {gbest} vs {ob}"
    return float(rel.max())


# sizes span several 256-tiles with ragged tails in every dimension; c_in = 200 takes the general
# contraction kernel (c_in % 64 != 0), n_tok = 37 a single partial k-tile of the token product
CASES = [
    # n_tok, c_in, c_out, bits, group, symmetric, bf16, weights
    (700, 384, 520, 4, 128, 0, False, "lognormal"),
    (1500, 640, 300, 3, 128, 0, False, "lognormal"),
    (300, 256, 256, 4, 128, 0, False, "uniform"),
    (900, 512, 770, 4, 128, 0, True, "lognormal"),
    (640, 1024, 260, 3, 128, 0, True, "lognormal"),
    (500, 200, 130, 4, 40, 0, False, "lognormal"),
    (450, 320, 200, 4, 0, 1, False, "lognormal"),
    (600, 256, 192, 8, 128, 0, False, "lognormal"),
    (800, 384, 256, 6, 0, 1, True, "lognormal"),
    (37, 128, 64, 2, 64, 0, False, "lognormal"),
    (1, 64, 8, 4, 64, 0, False, "uniform"),
]


@pytest.mark.parametrize("n_tok,c_in,c_out,bits,group,sym,bf16,weights", CASES)
def test_gram_search_matches_oracle(gpu, n_tok, c_in, c_out, bits, group, sym, bf16, weights):
    X, W, w = layer(n_tok + c_in, n_tok, c_in, c_out, bf16, weights=weights)
    dt = tlq.BF16 if bf16 else tlq.F16
    p = tlq.params(bits=bits, group=group, symmetric=sym, x_dtype=dt, yref_dtype=dt)
    alpha = wl.alpha_grid(20)
    gram, xs, losses, bi, best, st = gram_search(X, W, w, p, gpu, bf16, alpha)
    assert np.array_equal(xs, orc.x_stat_mean(X))
    # the matrix itself, element by element: fp16 operands and fp16 storage, balanced per channel
    G = decode_gram(gram, c_in)
    Go = orc.token_second_moment(X, w)
    dg = np.sqrt(np.diag(Go))
    assert np.all(np.abs(G - Go) <= 2.0 ** -9 * dg[:, None] * dg[None, :] + 1e-30)
    assert np.all(np.abs(G - G.T) <= 2.0 ** -11 * dg[:, None] * dg[None, :])
    # the search against the definition with the exact full-precision target
    ref = orc.scale_search(X, W, orc.ref_output(X, W), w, bits, group, alpha, x_stat=xs, s_table=st,
                           symmetric=bool(sym))
    worst = check_losses(losses, ref["losses"], bi, f"{n_tok}x{c_in}x{c_out}")
    np.testing.assert_array_equal(best, st[bi])
    ost = orc.scale_table(xs, alpha)
    assert np.max(np.abs(st.view(np.int32) - ost.view(np.int32))) <= 1
    print(f"max rel {worst:.2e}, best {bi}")


def test_gram_search_agrees_with_token_search(gpu):
    """Both forms on one layer whose channel magnitudes span five decades (the balancing keeps the
    fp16 matrix accurate where a single global scale would lose the small channels), W4 and W3."""
    import torch
    rng = np.random.default_rng(5)
    n, ci, co = 4096, 768, 512
    X, W, w = layer(77, n, ci, co)
    X = (X.astype(np.float32) * np.exp(rng.uniform(np.log(1e-3), np.log(30.0), ci))[None, :]).astype(np.float16)
    alpha = wl.alpha_grid(20)
    for bits in (4, 3):
        p = tlq.params(bits=bits, group=128)
        gram, xs, lg, bg, _, st = gram_search(X, W, w, p, gpu, False, alpha)
        ref = orc.scale_search(X, W, orc.ref_output(X, W), w, bits, 128, alpha, x_stat=xs, s_table=st)
        check_losses(lg, ref["losses"], bg, f"W{bits} gram")
        Xd, Wd, wd = dev(X, gpu), dev(W, gpu), dev(w, gpu)
        Y = torch.empty((n, co), dtype=torch.float32, device=gpu)
        pf = tlq.params(bits=bits, group=128, yref_dtype=tlq.F32)
        tlq.ref_output(Xd, Wd, Y, pf)
        best = torch.empty(ci, dtype=torch.float32, device=gpu)
        idx = torch.empty(1, dtype=torch.int32, device=gpu)
        ld = torch.empty(20, dtype=torch.float32, device=gpu)
        tlq.scale_search(Xd, Wd, Y, wd, dev(alpha, gpu), pf, best, idx, ld)
        rel = np.abs(ld.cpu().numpy().astype(np.float64) - lg) / lg
        assert rel.max() < LOSS_RTOL, rel.max()


def test_gram_wide_layer_with_ragged_tile_row(gpu):
    """C_in = 8512 = 33 tile rows + 64 channels: the token product runs with 8 x 4 patches and four
    splits, the quadratic form's last tile row holds only part of a diagonal block.  Sampled entries
    of the matrix and the search over 48 output rows against the oracle."""
    rng = np.random.default_rng(33)
    n, ci, co = 20000, 8512, 48
    X, W, w = layer(31, n, ci, co)
    alpha = wl.alpha_grid(20)
    p = tlq.params(bits=4, group=64)
    gram, xs, lg, bg, _, st = gram_search(X, W, w, p, gpu, False, alpha)
    ri = np.sort(np.concatenate([rng.choice(ci, 20, replace=False), [0, 255, 256, 8447, 8448, 8511]]))
    rj = np.sort(np.concatenate([rng.choice(ci, 20, replace=False), [1, 8191, 8192, 8450, 8511]]))
    f, cs, C = tlq.gram_views(gram, ci)
    import torch
    csn = cs.double().cpu().numpy()
    Cs = C[torch.from_numpy(ri).to(gpu)][:, torch.from_numpy(rj).to(gpu)].double().cpu().numpy()
    G = float(f.item()) * csn[ri][:, None] * csn[rj][None, :] * Cs
    Go = orc.token_second_moment(X, w, rows=ri, cols=rj)
    dg = np.sqrt(float(f.item()) * csn ** 2 * torch.diagonal(C).double().cpu().numpy())
    assert np.all(np.abs(G - Go) <= 2.0 ** -9 * dg[ri][:, None] * dg[rj][None, :])
    ref = orc.scale_search(X, W, orc.ref_output(X, W), w, 4, 64, alpha, x_stat=xs, s_table=st)
    worst = check_losses(lg, ref["losses"], bg, "wide layer")
    print(f"max rel {worst:.2e}, best {bg}")


def test_gram_strided_operands(gpu):
    """X and W as column slices of wider matrices (row strides larger than C_in): same bits as the
    dense call."""
    import torch
    X, W, w = layer(12, 700, 384, 200)
    p = tlq.params(bits=4, group=128)
    alpha = wl.alpha_grid(20)
    gram0, xs0, l0, b0, _, _ = gram_search(X, W, w, p, gpu, False, alpha)
    Xw = torch.full((700, 512), 7.0, dtype=torch.float16, device=gpu)
    Ww = torch.full((200, 448), -3.0, dtype=torch.float16, device=gpu)
    Xw[:, 64:448] = dev(X, gpu)
    Ww[:, 32:416] = dev(W, gpu)
    Xs, Wsl = Xw[:, 64:448], Ww[:, 32:416]
    assert Xs.stride(0) == 512 and Wsl.stride(0) == 448
    xs = torch.empty(384, dtype=torch.float32, device=gpu)
    tlq.x_stat(Xs, p, xs)
    gram = torch.empty(tlq.token_gram_bytes(384), dtype=torch.uint8, device=gpu)
    tlq.token_gram(Xs, dev(w, gpu), p, gram)
    out = (torch.empty(384, dtype=torch.float32, device=gpu), torch.empty(1, dtype=torch.int32, device=gpu),
           torch.empty(20, dtype=torch.float32, device=gpu))
    tlq.scale_search_gram(gram, Wsl, dev(alpha, gpu), p, xs, *out)
    torch.cuda.synchronize()
    for a, b in zip(tlq.gram_views(gram, 384), tlq.gram_views(gram0, 384)):      # (padding bytes are not written)
        assert torch.equal(a, b)
    assert np.array_equal(out[2].cpu().numpy(), l0) and int(out[1].item()) == b0


def test_gram_search_correlated_channels(gpu):
    """Activations dominated by one direction shared by all channels (x_t = 10 z_t a + noise), the
    structure real decoder activations have: every entry of the balanced matrix is then of order
    one and the quadratic form sums C_in^2 comparable terms."""
    rng = np.random.default_rng(21)
    n, ci, co = 3000, 512, 384
    _, W, w = layer(9, n, ci, co)
    a = rng.standard_normal(ci) * np.exp(rng.uniform(-2, 2, ci))
    X = (10.0 * rng.standard_normal((n, 1)) * a[None, :] + rng.standard_normal((n, ci))).astype(np.float16)
    alpha = wl.alpha_grid(20)
    for bits in (4, 3):
        p = tlq.params(bits=bits, group=128)
        gram, xs, lg, bg, _, st = gram_search(X, W, w, p, gpu, False, alpha)
        ref = orc.scale_search(X, W, orc.ref_output(X, W), w, bits, 128, alpha, x_stat=xs, s_table=st)
        worst = check_losses(lg, ref["losses"], bg, f"correlated W{bits}")
        print(f"W{bits}: max rel {worst:.2e}")


def test_gram_degenerate_inputs(gpu):
    """All-zero token weights give zero losses and the first candidate; a dead channel (all-zero
    column of X) is harmless; one dominant token weight is handled by the max-normalisation."""
    import torch
    X, W, w = layer(3, 400, 256, 96)
    X[:, 17] = 0
    p = tlq.params(bits=4, group=128)
    alpha = wl.alpha_grid(20)
    _, xs, l0, b0, _, _ = gram_search(X, W, np.zeros_like(w), p, gpu, False, alpha)
    assert np.all(l0 == 0.0) and b0 == 0
    w1 = w.copy()
    w1[7] = 1e6
    gram, xs, l1, b1, _, st = gram_search(X, W, w1, p, gpu, False, alpha)
    ref = orc.scale_search(X, W, orc.ref_output(X, W), w1, 4, 128, alpha, x_stat=xs, s_table=st)
    check_losses(l1, ref["losses"], b1, "dominant weight")
    G = decode_gram(gram, 256)
    assert np.all(G[17] == 0) and np.all(G[:, 17] == 0)


def test_gram_error_paths(gpu):
    import torch
    X, W, w = layer(4, 64, 128, 32)
    Xd, Wd, wd = dev(X, gpu), dev(W, gpu), dev(w, gpu)
    p = tlq.params(bits=4, group=128)
    gram = torch.empty(tlq.token_gram_bytes(128), dtype=torch.uint8, device=gpu)
    with pytest.raises(tlq.TlqError) as e:
        tlq.token_gram(Xd, wd, p, gram[:1024])
    assert e.value.status == tlq.ERR_WORKSPACE
    with pytest.raises(tlq.TlqError) as e:
        tlq.token_gram(Xd, wd, p, gram, workspace=torch.empty(256, dtype=torch.uint8, device=gpu))
    assert e.value.status == tlq.ERR_WORKSPACE
    tlq.token_gram(Xd, wd, p, gram)
    xs = torch.ones(128, dtype=torch.float32, device=gpu)
    out = (torch.empty(128, dtype=torch.float32, device=gpu), torch.empty(1, dtype=torch.int32, device=gpu),
           torch.empty(20, dtype=torch.float32, device=gpu))
    al = dev(wl.alpha_grid(20), gpu)
    with pytest.raises(tlq.TlqError) as e:
        tlq.scale_search_gram(gram, Wd, al, tlq.params(bits=4, group=128, act_bits=8), xs, *out)
    assert e.value.status == tlq.ERR_UNSUPPORTED
    with pytest.raises(tlq.TlqError) as e:
        tlq.scale_search_gram(gram, Wd, al, tlq.params(bits=4, group=96), xs, *out)
    assert e.value.status == tlq.ERR_SHAPE
    tlq.scale_search_gram(gram, Wd, al, p, xs, *out)
    torch.cuda.synchronize()
    assert np.all(np.isfinite(out[2].cpu().numpy()))


def test_gram_full_size_13b(gpu):
    """cfg4 q_proj at its full 153,600 tokens.  (1) Sampled entries of the second-moment matrix
    against the oracle's sums over all tokens.  (2) The search over 16 sampled output rows of W with
    the full-size matrix against the oracle's search on those rows over ALL tokens (the objective is
    additive over tokens, so the oracle goes sample by sample).  (3) The search over the whole
    layer against the token-form search of the library (itself tied to the oracle on sampled
    tokens in test_gpu_parity)."""
    import torch
    c = wl.CONFIGS["cfg4_13b_w4"]
    li = 0
    spec = c.linears[li]
    per = c.n_vis + c.n_txt
    X = torch.empty((c.n_tok, spec.c_in), dtype=torch.float16, device=gpu)
    rng = np.random.default_rng(0)
    ri, rj = np.sort(rng.choice(spec.c_in, 24, replace=False)), np.sort(rng.choice(spec.c_in, 24, replace=False))
    ri[:3] = wl.outlier_channels(c, li)[:3]
    w_np = wl.make_token_weights(c, li)
    Gs = np.zeros((24, 24))
    abs_sum = np.zeros(spec.c_in)
    for b in range(c.n_samples):
        xb = wl.make_sample_tokens(c, li, b).astype(np.float16)
        X[b * per:(b + 1) * per].copy_(torch.from_numpy(xb))
        Gs += orc.token_second_moment(xb, w_np[b * per:(b + 1) * per], rows=ri, cols=rj)
        abs_sum += np.abs(xb.astype(np.float64)).sum(axis=0)
    W_np = wl.make_weight(c, li)
    W, w = dev(W_np, gpu), dev(w_np, gpu)
    p = tlq.params(bits=c.bits, group=c.group)
    alpha = wl.alpha_grid(20)
    al = dev(alpha, gpu)
    xs = torch.empty(spec.c_in, dtype=torch.float32, device=gpu)
    tlq.x_stat(X, p, xs)
    xs_np = xs.cpu().numpy()
    assert np.array_equal(xs_np, (abs_sum / c.n_tok).astype(np.float32))
    gram = torch.empty(tlq.token_gram_bytes(spec.c_in), dtype=torch.uint8, device=gpu)
    tlq.token_gram(X, w, p, gram)
    f, cs, C = tlq.gram_views(gram, spec.c_in)
    csn = cs.double().cpu().numpy()
    Cs = C[torch.from_numpy(ri).to(gpu)][:, torch.from_numpy(rj).to(gpu)].double().cpu().numpy()
    G = float(f.item()) * csn[ri][:, None] * csn[rj][None, :] * Cs
    dg = np.sqrt(float(f.item()) * csn ** 2 * torch.diagonal(C).double().cpu().numpy())
    assert np.all(np.abs(G - Gs) <= 2.0 ** -9 * dg[ri][:, None] * dg[rj][None, :])
    # (2) sampled output rows, all tokens
    rows = np.sort(rng.choice(spec.c_out, 16, replace=False))
    Wr_np = np.ascontiguousarray(W_np[rows])
    best = torch.empty(spec.c_in, dtype=torch.float32, device=gpu)
    idx = torch.empty(1, dtype=torch.int32, device=gpu)
    lr = torch.empty(20, dtype=torch.float32, device=gpu)
    st = torch.empty((20, spec.c_in), dtype=torch.float32, device=gpu)
    tlq.scale_search_gram(gram, dev(Wr_np, gpu), al, p, xs, best, idx, lr, s_table_out=st)
    st_np = st.cpu().numpy()
    Lo = np.zeros(20)
    for b in range(c.n_samples):
        xb = wl.make_sample_tokens(c, li, b).astype(np.float16)
        Lo += orc.scale_search(xb, Wr_np, orc.ref_output(xb, Wr_np), w_np[b * per:(b + 1) * per], c.bits, c.group,
                               alpha, x_stat=xs_np, s_table=st_np)["losses"]
    worst = check_losses(lr.cpu().numpy(), Lo, int(idx.item()), "sampled rows, all tokens")
    # (3) the whole layer, both forms
    lg = torch.empty(20, dtype=torch.float32, device=gpu)
    tlq.scale_search_gram(gram, W, al, p, xs, best, idx, lg)
    Y = torch.empty((c.n_tok, spec.c_out), dtype=torch.float16, device=gpu)
    tlq.ref_output(X, W, Y, p)
    b2 = torch.empty_like(best)
    i2 = torch.empty_like(idx)
    ld = torch.empty_like(lg)
    tlq.scale_search(X, W, Y, w, al, p, b2, i2, ld, x_stat_in=xs)
    torch.cuda.synchronize()
    lgn, ldn = lg.cpu().numpy().astype(np.float64), ld.cpu().numpy().astype(np.float64)
    rel = np.abs(lgn - ldn) / ldn
    assert rel.max() < LOSS_RTOL, rel.max()
    assert int(idx.item()) == int(i2.item())
    print(f"full-size: sampled rows vs oracle max rel {worst:.2e}; gram vs token form max rel {rel.max():.2e}, "
          f"best {int(idx.item())}")
