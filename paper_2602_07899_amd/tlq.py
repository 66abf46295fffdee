"""Thin ctypes binding of libtlq.so (same names as include/tlq.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  Tensors are torch CUDA(ROCm) tensors used as device memory; work is
enqueued on torch's current stream.  The library is loaded on first use and a
missing build is an error - there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtlq.so")

OK, ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_ALIGN, ERR_LAUNCH = range(7)
F16, BF16, F32 = 0, 1, 2
MAX_ALPHA = 64


class Params(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("bits", C.c_int32), ("group", C.c_int32),
                ("symmetric", C.c_int32), ("act_bits", C.c_int32), ("xstat_kind", C.c_int32),
                ("x_dtype", C.c_int32), ("yref_dtype", C.c_int32)]


def params(bits=4, group=128, symmetric=0, act_bits=0, xstat_kind=0, x_dtype=F16, yref_dtype=F16):
    return Params(C.sizeof(Params), bits, group, symmetric, act_bits, xstat_kind, x_dtype, yref_dtype)


class TlqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None

_P = C.c_void_p
_I64 = C.c_int64
_I32 = C.c_int32
_SZ = C.c_size_t
_PP = C.POINTER(Params)

_SIGNATURES = {
    "tlq_status_string": (C.c_char_p, [C.c_int]),
    "tlq_version": (C.c_int, []),
    "tlq_x_stat_workspace_bytes": (_SZ, [_I64, _I64]),
    "tlq_x_stat": (C.c_int, [_P, _I64, _I64, _I64, _PP, _P, _P, _SZ, _P]),
    "tlq_x_stat_static": (C.c_int, [_P, _I64, _I64, _I64, _PP, _P, _P]),
    "tlq_token_importance_workspace_bytes": (_SZ, [_I64, _I64]),
    "tlq_token_importance": (C.c_int, [_P, _I64, _I64, _I64, _I64, _I32, _PP, _P, _P, _SZ, _P]),
    "tlq_topk_mask": (C.c_int, [_P, _I64, _I64, _P, _P]),
    "tlq_x_stat_masked": (C.c_int, [_P, _I64, _I64, _I64, _P, _I64, _PP, _P, _P, _SZ, _P]),
    "tlq_scale_table": (C.c_int, [_P, _I64, _P, _I32, _P, _P]),
    "tlq_fake_quant": (C.c_int, [_P, _I64, _I64, _I64, _P, _PP, _P, _P, _P, _P, _I64, _P]),
    "tlq_act_fake_quant": (C.c_int, [_P, _I64, _I64, _I64, _P, _PP, _P, _P, _P]),
    "tlq_weighted_layer_err_workspace_bytes": (_SZ, [_I64, _I64, _I64, _PP]),
    "tlq_weighted_layer_err": (C.c_int, [_P, _I64, _I64, _I64, _P, _I64, _I64, _P, _P, _I64, _P,
                                         _PP, _P, _P, _P, _SZ, _P]),
    "tlq_scale_search_workspace_bytes": (_SZ, [_I64, _I64, _I64, _I32, _PP]),
    "tlq_scale_search": (C.c_int, [_P, _I64, _I64, _I64, _P, _I64, _I64, _P, _I64, _P, _P, _I32,
                                   _PP, _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "tlq_prepared_tokens_bytes": (_SZ, [_I64, _I64, _PP]),
    "tlq_prepare_tokens": (C.c_int, [_P, _I64, _I64, _I64, _PP, _P, _SZ, _P]),
    "tlq_scale_search_prepared": (C.c_int, [_P, _I64, _I64, _I64, _P, _I64, _I64, _P, _I64, _P, _P, _I32,
                                            _PP, _P, _P, _P, _P, _P, _P, _SZ, _P, _P]),
    "tlq_apply_best_prepared": (C.c_int, [_P, _I64, _I64, _I64, _P, _I64, _I64, _P, _PP, _P, _I64, _P, _SZ, _P, _P]),
    "tlq_token_gram_bytes": (_SZ, [_I64]),
    "tlq_token_gram_workspace_bytes": (_SZ, [_I64, _I64]),
    "tlq_token_gram": (C.c_int, [_P, _I64, _I64, _I64, _P, _PP, _P, _SZ, _P, _SZ, _P]),
    "tlq_scale_search_gram_workspace_bytes": (_SZ, [_I64, _I64, _I32, _PP]),
    "tlq_scale_search_gram": (C.c_int, [_P, _I64, _P, _I64, _I64, _P, _I32, _PP, _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "tlq_ref_output": (C.c_int, [_P, _I64, _I64, _I64, _P, _I64, _I64, _P, _I64, _PP, _P]),
    "tlq_apply_best_workspace_bytes": (_SZ, [_I64, _I64, _I64, _PP]),
    "tlq_apply_best": (C.c_int, [_P, _I64, _I64, _I64, _P, _I64, _I64, _P, _PP, _P, _I64, _P, _SZ, _P]),
    "tlq_rmsnorm_mul": (C.c_int, [_P, _I64, _I64, _I64, _P, _I64, _P, _P, _I32, _I32, _PP, _P, _I64, _P]),
    "tlq_causal_attention": (C.c_int, [_P, _I64, _P, _I64, _P, _I64, _I64, _I32, _I32, _I32, _PP, _P, _I64, _P]),
    "tlq_silu_mul": (C.c_int, [_P, _I64, _P, _I64, _I64, _I64, _PP, _P, _I64, _P]),
    "tlq_residual_add": (C.c_int, [_P, _I64, _P, _I64, _I64, _I64, _PP, _P, _I64, _P]),
    "tlq_selftest_tile_map": (C.c_int64, [_I64, _I64, _I64, _I32, C.POINTER(C.c_int64)]),
    "tlq_profile_enable": (C.c_int, [C.c_int]),
    "tlq_profile_enabled": (C.c_int, []),
    "tlq_profile_reset": (C.c_int, []),
    "tlq_profile_collect": (C.c_int, []),
    "tlq_profile_count": (C.c_int, []),
    "tlq_profile_get": (C.c_int, [C.c_int, C.c_char_p, _SZ, C.POINTER(C.c_int64),
                                  C.POINTER(C.c_double), C.POINTER(C.c_double)]),
}
EXPORTS = tuple(_SIGNATURES)


def lib():
    """Load libtlq.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2602_07899_amd.build` (no fallback path exists)")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def selftest_tile_map(n_tok, c_in, c_out, n_cand):
    """(defects, workgroups) of the contraction kernels' block -> tile map for one shape (host only)."""
    blocks = C.c_int64(0)
    bad = lib().tlq_selftest_tile_map(n_tok, c_in, c_out, n_cand, C.byref(blocks))
    return int(bad), int(blocks.value)


def status_string(status: int) -> str:
    return lib().tlq_status_string(int(status)).decode()


def version() -> int:
    return lib().tlq_version()


def _check(status, where):
    if status != OK:
        raise TlqError(status, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(nbytes, like):
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=like.device)


def _ld(t):
    assert t.dim() == 2 and t.stride(1) == 1, "matrices must be row-major with unit column stride"
    return t.stride(0)


# ------------------------------------------------------------------ entry points
def x_stat_workspace_bytes(n_tok, c_in):
    return lib().tlq_x_stat_workspace_bytes(n_tok, c_in)


def x_stat(X, p, out, workspace=None):
    n, c = X.shape
    ws = workspace if workspace is not None else _ws(x_stat_workspace_bytes(n, c), X)
    _check(lib().tlq_x_stat(_ptr(X), n, c, _ld(X), C.byref(p), _ptr(out), _ptr(ws), ws.numel(),
                            _stream()), "tlq_x_stat")
    return out


def x_stat_static(X, p, out):
    """tlq_x_stat without a workspace: partial sums go to the library's fixed device array."""
    n, c = X.shape
    _check(lib().tlq_x_stat_static(_ptr(X), n, c, _ld(X), C.byref(p), _ptr(out), _stream()),
           "tlq_x_stat_static")
    return out


def token_importance(G, n_samples, p, sum_n, l2=False, workspace=None):
    rows, c = G.shape
    n_pos = rows // n_samples
    ws = workspace if workspace is not None else _ws(lib().tlq_token_importance_workspace_bytes(n_samples, n_pos), G)
    _check(lib().tlq_token_importance(_ptr(G), n_samples, n_pos, c, _ld(G), 1 if l2 else 0, C.byref(p),
                                      _ptr(sum_n), _ptr(ws), ws.numel(), _stream()), "tlq_token_importance")
    return sum_n


def topk_mask(sum_n, k, mask):
    _check(lib().tlq_topk_mask(_ptr(sum_n), sum_n.numel(), k, _ptr(mask), _stream()), "tlq_topk_mask")
    return mask


def x_stat_masked(X, pos_mask, p, out, workspace=None):
    n, c = X.shape
    ws = workspace if workspace is not None else _ws(x_stat_workspace_bytes(n, c), X)
    _check(lib().tlq_x_stat_masked(_ptr(X), n, c, _ld(X), _ptr(pos_mask), pos_mask.numel(), C.byref(p),
                                   _ptr(out), _ptr(ws), ws.numel(), _stream()), "tlq_x_stat_masked")
    return out


def scale_table(x_stat_t, alpha_grid, out):
    _check(lib().tlq_scale_table(_ptr(x_stat_t), x_stat_t.numel(), _ptr(alpha_grid),
                                 alpha_grid.numel(), _ptr(out), _stream()), "tlq_scale_table")
    return out


def fake_quant(W, s, p, codes=None, zp=None, delta=None, Wdq=None):
    co, ci = W.shape
    _check(lib().tlq_fake_quant(_ptr(W), co, ci, _ld(W), _ptr(s), C.byref(p), _ptr(codes), _ptr(zp),
                                _ptr(delta), _ptr(Wdq), 0 if Wdq is None else _ld(Wdq), _stream()),
           "tlq_fake_quant")


def act_fake_quant(X, inv_s, p, codes, sigma):
    n, c = X.shape
    _check(lib().tlq_act_fake_quant(_ptr(X), n, c, _ld(X), _ptr(inv_s), C.byref(p), _ptr(codes),
                                    _ptr(sigma), _stream()), "tlq_act_fake_quant")


def weighted_layer_err_workspace_bytes(n_tok, c_in, c_out, p):
    return lib().tlq_weighted_layer_err_workspace_bytes(n_tok, c_in, c_out, C.byref(p))


def weighted_layer_err(X, Wdq, inv_s, Y_ref, token_w, p, loss, per_token_err=None, workspace=None):
    n, ci = X.shape
    co = Wdq.shape[0]
    ws = workspace if workspace is not None else _ws(
        weighted_layer_err_workspace_bytes(n, ci, co, p), X)
    _check(lib().tlq_weighted_layer_err(_ptr(X), n, ci, _ld(X), _ptr(Wdq), co, _ld(Wdq), _ptr(inv_s),
                                        _ptr(Y_ref), _ld(Y_ref), _ptr(token_w), C.byref(p),
                                        _ptr(loss), _ptr(per_token_err), _ptr(ws), ws.numel(),
                                        _stream()), "tlq_weighted_layer_err")
    return loss


def scale_search_workspace_bytes(n_tok, c_in, c_out, n_alpha, p):
    return lib().tlq_scale_search_workspace_bytes(n_tok, c_in, c_out, n_alpha, C.byref(p))


def prepared_tokens_bytes(n_tok, c_in, p):
    return lib().tlq_prepared_tokens_bytes(n_tok, c_in, C.byref(p))


def prepare_tokens(X, p, prepared):
    """Fill `prepared` (uint8 tensor of prepared_tokens_bytes bytes) from X; see tlq.h."""
    n, ci = X.shape
    _check(lib().tlq_prepare_tokens(_ptr(X), n, ci, _ld(X), C.byref(p), _ptr(prepared),
                                    0 if prepared is None else prepared.numel(), _stream()), "tlq_prepare_tokens")
    return prepared


def scale_search(X, W, Y_ref, token_w, alpha_grid, p, best_scales, best_idx, losses,
                 x_stat_in=None, s_table_out=None, workspace=None, prepared=None):
    n, ci = X.shape
    co = W.shape[0]
    na = alpha_grid.numel()
    ws = workspace if workspace is not None else _ws(scale_search_workspace_bytes(n, ci, co, na, p), X)
    if prepared is None:
        _check(lib().tlq_scale_search(_ptr(X), n, ci, _ld(X), _ptr(W), co, _ld(W), _ptr(Y_ref),
                                      _ld(Y_ref), _ptr(token_w), _ptr(alpha_grid), na, C.byref(p),
                                      _ptr(x_stat_in), _ptr(best_scales), _ptr(best_idx), _ptr(losses),
                                      _ptr(s_table_out), _ptr(ws), ws.numel(), _stream()),
               "tlq_scale_search")
    else:
        _check(lib().tlq_scale_search_prepared(_ptr(X), n, ci, _ld(X), _ptr(W), co, _ld(W), _ptr(Y_ref),
                                               _ld(Y_ref), _ptr(token_w), _ptr(alpha_grid), na, C.byref(p),
                                               _ptr(x_stat_in), _ptr(best_scales), _ptr(best_idx), _ptr(losses),
                                               _ptr(s_table_out), _ptr(ws), ws.numel(), _stream(), _ptr(prepared)),
               "tlq_scale_search_prepared")


def token_gram_bytes(c_in):
    return int(lib().tlq_token_gram_bytes(c_in))


def token_gram_workspace_bytes(n_tok, c_in):
    return int(lib().tlq_token_gram_workspace_bytes(n_tok, c_in))


def token_gram(X, token_w, p, gram, workspace=None):
    """Fill `gram` (uint8 tensor of token_gram_bytes(c_in) bytes) with the weighted second-moment
    matrix of the tokens; see tlq.h."""
    n, ci = X.shape
    ws = workspace if workspace is not None else _ws(token_gram_workspace_bytes(n, ci), X)
    _check(lib().tlq_token_gram(_ptr(X), n, ci, _ld(X), _ptr(token_w), C.byref(p), _ptr(gram),
                                0 if gram is None else gram.numel(), _ptr(ws), ws.numel(), _stream()),
           "tlq_token_gram")
    return gram


def gram_views(gram, c_in):
    """(factor [1] f64, col_scale [c_in] f32, C [c_in, c_in] f16) views of a filled gram buffer:
    G[i, j] = factor * col_scale[i] * col_scale[j] * C[i, j]."""
    import torch
    a256 = lambda n: (n + 255) // 256 * 256
    o1, o2 = 256, 256 + a256(4 * c_in)
    return (gram[:8].view(torch.float64), gram[o1:o1 + 4 * c_in].view(torch.float32),
            gram[o2:o2 + 2 * c_in * c_in].view(torch.float16).view(c_in, c_in))


def scale_search_gram_workspace_bytes(c_in, c_out, n_alpha, p):
    return int(lib().tlq_scale_search_gram_workspace_bytes(c_in, c_out, n_alpha, C.byref(p)))


def scale_search_gram(gram, W, alpha_grid, p, x_stat, best_scales, best_idx, losses,
                      s_table_out=None, workspace=None):
    co, ci = W.shape
    na = alpha_grid.numel()
    ws = workspace if workspace is not None else _ws(scale_search_gram_workspace_bytes(ci, co, na, p), W)
    _check(lib().tlq_scale_search_gram(_ptr(gram), ci, _ptr(W), co, _ld(W), _ptr(alpha_grid), na, C.byref(p),
                                       _ptr(x_stat), _ptr(best_scales), _ptr(best_idx), _ptr(losses),
                                       _ptr(s_table_out), _ptr(ws), ws.numel(), _stream()),
           "tlq_scale_search_gram")


def ref_output(X, W, Y, p):
    n, ci = X.shape
    co = W.shape[0]
    _check(lib().tlq_ref_output(_ptr(X), n, ci, _ld(X), _ptr(W), co, _ld(W), _ptr(Y), _ld(Y),
                                C.byref(p), _stream()), "tlq_ref_output")
    return Y


def apply_best_workspace_bytes(n_tok, c_in, c_out, p):
    return lib().tlq_apply_best_workspace_bytes(n_tok, c_in, c_out, C.byref(p))


def apply_best(X, W, s, p, X_next, workspace=None, prepared=None):
    n, ci = X.shape
    co = W.shape[0]
    ws = workspace if workspace is not None else _ws(apply_best_workspace_bytes(n, ci, co, p), X)
    if prepared is None:
        _check(lib().tlq_apply_best(_ptr(X), n, ci, _ld(X), _ptr(W), co, _ld(W), _ptr(s), C.byref(p),
                                    _ptr(X_next), _ld(X_next), _ptr(ws), ws.numel(), _stream()),
               "tlq_apply_best")
    else:
        _check(lib().tlq_apply_best_prepared(_ptr(X), n, ci, _ld(X), _ptr(W), co, _ld(W), _ptr(s), C.byref(p),
                                             _ptr(X_next), _ld(X_next), _ptr(ws), ws.numel(), _stream(),
                                             _ptr(prepared)), "tlq_apply_best_prepared")
    return X_next


def rmsnorm_mul(Z, p, X_out, Zb=None, m_a=None, m_b=None, period=0, split=0):
    n, c = Z.shape
    _check(lib().tlq_rmsnorm_mul(_ptr(Z), n, c, _ld(Z), _ptr(Zb), 0 if Zb is None else _ld(Zb), _ptr(m_a),
                                 _ptr(m_b), period, split, C.byref(p), _ptr(X_out), _ld(X_out), _stream()),
           "tlq_rmsnorm_mul")
    return X_out


def causal_attention(Q, K, V, n_heads, seq_len, p, Out):
    """Q, K, V, Out: [n_tok, >= n_heads*128] (column slices of a wider matrix are fine)."""
    _check(lib().tlq_causal_attention(_ptr(Q), _ld(Q), _ptr(K), _ld(K), _ptr(V), _ld(V), Q.shape[0], n_heads,
                                      128, seq_len, C.byref(p), _ptr(Out), _ld(Out), _stream()),
           "tlq_causal_attention")
    return Out


def silu_mul(G, U, p, Out):
    n, c = G.shape
    _check(lib().tlq_silu_mul(_ptr(G), _ld(G), _ptr(U), _ld(U), n, c, C.byref(p), _ptr(Out), _ld(Out), _stream()),
           "tlq_silu_mul")
    return Out


def residual_add(H, Z, p, Out):
    n, c = H.shape
    _check(lib().tlq_residual_add(_ptr(H), _ld(H), _ptr(Z), _ld(Z), n, c, C.byref(p), _ptr(Out), _ld(Out),
                                  _stream()), "tlq_residual_add")
    return Out


# ------------------------------------------------------------------ profiling
@dataclass
class KernelTime:
    name: str
    launches: int
    total_ms: float
    total_work: float


def profile_enable(on: bool):
    _check(lib().tlq_profile_enable(1 if on else 0), "tlq_profile_enable")


def profile_reset():
    _check(lib().tlq_profile_reset(), "tlq_profile_reset")


def profile_read():
    """Wait for recorded events and return the per-kernel totals."""
    l = lib()
    _check(l.tlq_profile_collect(), "tlq_profile_collect")
    out = []
    for i in range(l.tlq_profile_count()):
        name = C.create_string_buffer(64)
        n, ms, work = C.c_int64(), C.c_double(), C.c_double()
        _check(l.tlq_profile_get(i, name, 64, C.byref(n), C.byref(ms), C.byref(work)), "tlq_profile_get")
        out.append(KernelTime(name.value.decode(), n.value, ms.value, work.value))
    return out
