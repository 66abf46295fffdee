"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and every argument error is reported before
anything could be launched."""
import ctypes as C
import os
import re

import pytest

from paper_2602_07899_amd import tlq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "tlq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tlq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert len(names) >= 15
    l = tlq.lib()
    for n in names:
        assert hasattr(l, n), f"{n} declared in tlq.h but not exported"
    assert set(names) == set(tlq.EXPORTS), "binding and header disagree"
    assert tlq.version() == 100
    assert tlq.status_string(tlq.OK) == "ok"
    assert "workspace" in tlq.status_string(tlq.ERR_WORKSPACE)


def test_params_struct_layout():
    assert C.sizeof(tlq.Params) == 32
    p = tlq.params()
    assert p.struct_size == 32 and p.bits == 4 and p.group == 128


FAKE = C.c_void_p(0x1000)        # aligned, never dereferenced: validation fails first
ODD = C.c_void_p(0x1004)


def _search(p, X=FAKE, n=256, ci=512, ldx=512, W=FAKE, co=512, ldw=512, Y=FAKE, ldy=512, w=FAKE,
            al=FAKE, na=20, best=FAKE, idx=FAKE, losses=FAKE, ws=FAKE, wsb=1 << 40):
    return tlq.lib().tlq_scale_search(X, n, ci, ldx, W, co, ldw, Y, ldy, w, al, na, C.byref(p), None,
                                      best, idx, losses, None, ws, wsb, None)


def test_scale_search_rejects_bad_arguments():
    p = tlq.params()
    assert _search(p, X=None) == tlq.ERR_NULL
    assert _search(p, losses=None) == tlq.ERR_NULL
    assert _search(p, n=0) == tlq.ERR_SHAPE
    assert _search(p, ldx=256) == tlq.ERR_SHAPE               # stride smaller than row
    assert _search(p, ci=520, ldx=520, ldw=520) == tlq.ERR_SHAPE   # not a multiple of group
    assert _search(p, ci=508, ldx=512, ldw=512) == tlq.ERR_SHAPE   # not a multiple of 8
    assert _search(p, na=0) == tlq.ERR_SHAPE
    assert _search(p, na=tlq.MAX_ALPHA + 1) == tlq.ERR_SHAPE
    assert _search(p, X=ODD) == tlq.ERR_ALIGN
    assert _search(p, ldy=516) == tlq.ERR_ALIGN
    assert _search(p, ws=None) == tlq.ERR_WORKSPACE
    assert _search(p, wsb=1024) == tlq.ERR_WORKSPACE
    for field, bad in [("bits", 1), ("bits", 9), ("group", 100), ("symmetric", 2), ("act_bits", 1), ("act_bits", 9),
                       ("xstat_kind", 2), ("x_dtype", tlq.F32), ("yref_dtype", 3), ("struct_size", 28)]:
        q = tlq.params()
        setattr(q, field, bad)
        assert _search(q) == tlq.ERR_UNSUPPORTED, field


def test_other_entry_points_reject_bad_arguments():
    l = tlq.lib()
    p = tlq.params()
    bp = C.byref(p)
    assert l.tlq_x_stat(None, 4, 8, 8, bp, FAKE, FAKE, 1 << 30, None) == tlq.ERR_NULL
    assert l.tlq_x_stat(FAKE, 4, 12, 16, bp, FAKE, FAKE, 1 << 30, None) == tlq.ERR_SHAPE
    assert l.tlq_x_stat(FAKE, 4, 8, 8, bp, FAKE, None, 0, None) == tlq.ERR_WORKSPACE
    assert l.tlq_scale_table(FAKE, 8, None, 4, FAKE, None) == tlq.ERR_NULL
    assert l.tlq_scale_table(FAKE, 8, FAKE, 0, FAKE, None) == tlq.ERR_SHAPE
    assert l.tlq_fake_quant(None, 4, 128, 128, None, bp, None, None, None, None, 0, None) == tlq.ERR_NULL
    assert l.tlq_fake_quant(FAKE, 4, 192, 192, None, bp, None, None, None, None, 0, None) == tlq.ERR_SHAPE
    assert l.tlq_fake_quant(ODD, 4, 128, 128, None, bp, None, None, None, None, 0, None) == tlq.ERR_ALIGN
    assert l.tlq_fake_quant(FAKE, 4, 128, 128, None, bp, None, None, None, FAKE, 64, None) == tlq.ERR_SHAPE
    assert l.tlq_weighted_layer_err(FAKE, 4, 128, 128, FAKE, 4, 128, None, FAKE, 8, None, bp, FAKE,
                                    None, FAKE, 1 << 30, None) == tlq.ERR_NULL
    assert l.tlq_weighted_layer_err(FAKE, 4, 128, 128, FAKE, 4, 128, None, FAKE, 8, FAKE, bp, FAKE,
                                    None, FAKE, 16, None) == tlq.ERR_WORKSPACE
    assert l.tlq_ref_output(FAKE, 4, 128, 128, FAKE, 4, 128, None, 8, bp, None) == tlq.ERR_NULL
    assert l.tlq_ref_output(FAKE, 4, 128, 128, FAKE, 4, 128, FAKE, 2, bp, None) == tlq.ERR_SHAPE
    assert l.tlq_apply_best(FAKE, 4, 128, 128, FAKE, 4, 128, None, bp, FAKE, 8, FAKE, 1 << 30,
                            None) == tlq.ERR_NULL
    assert l.tlq_apply_best(FAKE, 4, 128, 128, FAKE, 4, 128, FAKE, bp, FAKE, 8, FAKE, 8,
                            None) == tlq.ERR_WORKSPACE
    assert l.tlq_profile_get(99, None, 0, None, None, None) == tlq.ERR_SHAPE
    assert l.tlq_token_importance(None, 2, 4, 8, 8, 0, bp, FAKE, FAKE, 1 << 20, None) == tlq.ERR_NULL
    assert l.tlq_token_importance(FAKE, 2, 4, 8, 4, 0, bp, FAKE, FAKE, 1 << 20, None) == tlq.ERR_SHAPE
    assert l.tlq_token_importance(FAKE, 2, 4, 8, 8, 0, bp, FAKE, None, 0, None) == tlq.ERR_WORKSPACE
    assert l.tlq_topk_mask(FAKE, 4, 5, FAKE, None) == tlq.ERR_SHAPE
    assert l.tlq_topk_mask(FAKE, 1 << 20, 5, FAKE, None) == tlq.ERR_UNSUPPORTED
    assert l.tlq_x_stat_masked(FAKE, 4, 8, 8, None, 2, bp, FAKE, FAKE, 1 << 20, None) == tlq.ERR_NULL
    assert l.tlq_x_stat_masked(FAKE, 4, 8, 8, FAKE, 0, bp, FAKE, FAKE, 1 << 20, None) == tlq.ERR_SHAPE
    assert l.tlq_rmsnorm_mul(None, 4, 8, 8, None, 0, None, None, 0, 0, bp, FAKE, 8, None) == tlq.ERR_NULL
    assert l.tlq_rmsnorm_mul(FAKE, 4, 8, 8, None, 0, None, None, 0, 0, bp, FAKE, 4, None) == tlq.ERR_SHAPE
    assert l.tlq_rmsnorm_mul(FAKE, 4, 8, 8, None, 0, None, None, 4, 2, bp, FAKE, 8, None) == tlq.ERR_SHAPE
    att = lambda **k: l.tlq_causal_attention(k.get("Q", FAKE), k.get("ld", 256), FAKE, 256, FAKE, 256, k.get("n", 64),
                                             k.get("heads", 2), k.get("dh", 128), k.get("seq", 32), bp,
                                             k.get("out", FAKE), k.get("ldo", 256), None)
    assert att(Q=None) == tlq.ERR_NULL and att(out=None) == tlq.ERR_NULL
    assert att(dh=64) == tlq.ERR_UNSUPPORTED
    assert att(seq=48) == tlq.ERR_SHAPE            # 64 tokens are not whole samples of 48
    assert att(seq=0) == tlq.ERR_SHAPE and att(heads=0) == tlq.ERR_SHAPE and att(n=0) == tlq.ERR_SHAPE
    assert att(ld=128) == tlq.ERR_SHAPE and att(ldo=200) == tlq.ERR_SHAPE      # narrower than heads*128
    assert att(Q=ODD) == tlq.ERR_ALIGN and att(ld=260) == tlq.ERR_ALIGN
    for fn in (l.tlq_silu_mul, l.tlq_residual_add):
        assert fn(None, 8, FAKE, 8, 4, 8, bp, FAKE, 8, None) == tlq.ERR_NULL
        assert fn(FAKE, 8, FAKE, 8, 4, 8, bp, None, 8, None) == tlq.ERR_NULL
        assert fn(FAKE, 16, FAKE, 16, 4, 12, bp, FAKE, 16, None) == tlq.ERR_SHAPE   # width not a multiple of 8
        assert fn(FAKE, 8, FAKE, 4, 4, 8, bp, FAKE, 8, None) == tlq.ERR_SHAPE
        assert fn(FAKE, 8, FAKE, 8, 0, 8, bp, FAKE, 8, None) == tlq.ERR_SHAPE
        assert fn(ODD, 8, FAKE, 8, 4, 8, bp, FAKE, 8, None) == tlq.ERR_ALIGN


def test_workspace_queries():
    p = tlq.params()
    q = tlq.scale_search_workspace_bytes
    assert q(0, 512, 512, 20, p) == 0 and q(256, 512, 512, 0, p) == 0
    small, big = q(256, 512, 512, 20, p), q(10240, 4096, 4096, 20, p)
    assert small % 256 == 0 and small >= 20 * 512 * 512 * 2
    assert big >= 20 * 4096 * 4096 * 2 and big < 20 * 4096 * 4096 * 2 + (64 << 20)
    assert q(256, 512, 512, 10, p) < small
    bad = tlq.params(bits=1)
    assert q(256, 512, 512, 20, bad) == 0
    assert tlq.x_stat_workspace_bytes(256, 512) >= 2 * 512 * 8
    assert tlq.apply_best_workspace_bytes(256, 512, 512, p) >= 512 * 512 * 2
    pb = tlq.params(x_dtype=tlq.BF16)
    assert (tlq.apply_best_workspace_bytes(256, 512, 512, pb)
            >= tlq.apply_best_workspace_bytes(256, 512, 512, p) + 256 * 512 * 2)
    assert q(256, 512, 512, 20, pb) >= small + 256 * 512 * 2
    assert tlq.weighted_layer_err_workspace_bytes(256, 512, 512, p) >= 512 * 512 * 2


@pytest.mark.parametrize("shape", [
    (256, 512, 512, 20),            # small case: one tile column
    (10240, 4096, 4096, 20),        # 7B attention linear: one token chunk
    (10240, 4096, 11008, 20),       # 43 tile rows: last patch row has 3 (3 x 10 patches)
    (10240, 11008, 4096, 20),       # deep linear: several token chunks of 2 patches, last of 1
    (40960, 4096, 11008, 20),       # 160 tile columns in chunks of 4 patches
    (153600, 5120, 13824, 20),      # 54 tile rows: last patch row has 2 (2 x 16 patches)
    (153600, 13824, 5120, 20),
    (700, 512, 300, 3), (5000, 1024, 1300, 2), (9000, 64, 2304, 1), (100000, 8192, 768, 2),
    (257, 8, 257, 64), (1, 8, 1, 1), (70000, 2048, 256, 7),
])
def test_block_to_tile_map_covers_every_tile_once(shape):
    """The contraction kernels derive (candidate, tile) from the block id alone; the host replay of
    that map must hit every tile of every candidate exactly once, including the regrouped
    incomplete patch row and a short last token chunk."""
    n_tok, c_in, c_out, n_cand = shape
    bad, blocks = tlq.selftest_tile_map(n_tok, c_in, c_out, n_cand)
    tiles = n_cand * -(-n_tok // 256) * -(-c_out // 256)
    assert bad == 0
    assert blocks >= tiles and blocks % 256 == 0
    if tiles >= 20000:
        assert blocks <= 1.02 * tiles          # the regrouped patch row leaves < 2 % dead slots
    assert tlq.selftest_tile_map(0, 8, 8, 1)[0] == -1
