"""The library allocates nothing, never synchronises and clears its scratch with
kernels, so a whole scale search can be captured into a HIP graph.  The graph is
replayed several times with eager work and synchronisations in between, on
changing inputs, and every replay is compared with the eager result."""
import numpy as np
import pytest

from paper_2602_07899_amd import tlq
from paper_2602_07899_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("act_bits,bf16", [(0, False), (8, False), (0, True)])
def test_scale_search_graph_replays_match_eager(gpu, act_bits, bf16):
    import torch
    c = wl.CONFIGS["cfg1_small"]
    dt = torch.bfloat16 if bf16 else torch.float16
    code = tlq.BF16 if bf16 else tlq.F16
    p = tlq.params(bits=c.bits, group=c.group, act_bits=act_bits, x_dtype=code, yref_dtype=code)
    n, ci, co = 300, 512, 384                       # ragged token count
    g = torch.Generator(device="cpu")
    g.manual_seed(5)
    W = (torch.randn((co, ci), generator=g) * 0.02).to(dt).to(gpu)
    X = torch.empty((n, ci), dtype=dt, device=gpu)
    Y = torch.empty((n, co), dtype=dt, device=gpu)
    w = torch.rand(n, generator=g).to(gpu)
    w /= w.sum()
    al = torch.from_numpy(wl.alpha_grid(8)).to(gpu)
    ws = torch.empty(tlq.scale_search_workspace_bytes(n, ci, co, 8, p), dtype=torch.uint8, device=gpu)
    out = [torch.empty(ci, dtype=torch.float32, device=gpu), torch.empty(1, dtype=torch.int32, device=gpu),
           torch.empty(8, dtype=torch.float32, device=gpu), torch.empty((8, ci), dtype=torch.float32, device=gpu)]

    def fresh_inputs(seed):
        gg = torch.Generator(device="cpu")
        gg.manual_seed(seed)
        x = torch.randn((n, ci), generator=gg)
        x[:, 7] *= 25.0 + seed
        X.copy_(x.to(dt))
        tlq.ref_output(X, W, Y, p)

    def search():
        tlq.scale_search(X, W, Y, w, al, p, out[0], out[1], out[2], s_table_out=out[3], workspace=ws)

    fresh_inputs(0)
    side = torch.cuda.Stream()                      # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        search()                                    # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        search()
    for seed in (1, 2, 3, 4):
        fresh_inputs(seed)
        search()
        torch.cuda.synchronize()
        eager = [t.clone() for t in out]
        ws.fill_(0xAB)                              # the search must not depend on what the workspace held
        for t in out:
            t.fill_(-7 if t.dtype == torch.int32 else float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for e, r in zip(eager, out):
            assert torch.equal(e, r), seed
        assert bool(torch.isfinite(out[2]).all())


@pytest.mark.parametrize("bf16", [False, True])
def test_gram_search_graph_replays_match_eager(gpu, bf16):
    """The second-moment form (statistic, token second-moment matrix, search through it) captured
    as one graph; workspace and result buffer are poisoned between the eager run and each replay."""
    import torch
    dt = torch.bfloat16 if bf16 else torch.float16
    code = tlq.BF16 if bf16 else tlq.F16
    p = tlq.params(bits=4, group=128, x_dtype=code, yref_dtype=code)
    n, ci, co = 9000, 512, 384          # two splits of the token product, ragged in every dimension
    g = torch.Generator(device="cpu")
    g.manual_seed(6)
    W = (torch.randn((co, ci), generator=g) * 0.02).to(dt).to(gpu)
    X = torch.empty((n, ci), dtype=dt, device=gpu)
    w = torch.rand(n, generator=g).to(gpu)
    w /= w.sum()
    al = torch.from_numpy(wl.alpha_grid(8)).to(gpu)
    ws = torch.empty(max(tlq.token_gram_workspace_bytes(n, ci), tlq.x_stat_workspace_bytes(n, ci),
                         tlq.scale_search_gram_workspace_bytes(ci, co, 8, p)), dtype=torch.uint8, device=gpu)
    gram = torch.empty(tlq.token_gram_bytes(ci), dtype=torch.uint8, device=gpu)
    xs = torch.empty(ci, dtype=torch.float32, device=gpu)
    out = [torch.empty(ci, dtype=torch.float32, device=gpu), torch.empty(1, dtype=torch.int32, device=gpu),
           torch.empty(8, dtype=torch.float32, device=gpu), torch.empty((8, ci), dtype=torch.float32, device=gpu)]

    def fresh_inputs(seed):
        gg = torch.Generator(device="cpu")
        gg.manual_seed(seed)
        x = torch.randn((n, ci), generator=gg)
        x[:, 7] *= 25.0 + seed
        X.copy_(x.to(dt))

    def search():
        tlq.x_stat(X, p, xs, workspace=ws)
        tlq.token_gram(X, w, p, gram, workspace=ws)
        tlq.scale_search_gram(gram, W, al, p, xs, out[0], out[1], out[2], s_table_out=out[3], workspace=ws)

    fresh_inputs(0)
    side = torch.cuda.Stream()                      # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        search()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        search()
    for seed in (1, 2, 3):
        fresh_inputs(seed)
        search()
        torch.cuda.synchronize()
        eager = [t.clone() for t in out]
        ws.fill_(0xAB)
        gram.fill_(0xCD)
        for t in out:
            t.fill_(-7 if t.dtype == torch.int32 else float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for e, r in zip(eager, out):
            assert torch.equal(e, r), seed
        assert bool(torch.isfinite(out[2]).all())
