// C ABI entry points: argument validation, workspace carving, launch plans.
// Validation touches no HIP API, so every error path returns before anything
// is enqueued.
#include "common.h"

using namespace tlq;

namespace {

struct Carver {
  unsigned char* base; size_t off;
  explicit Carver(void* p) : base((unsigned char*)p), off(0) {}
  template <typename T> T* take(size_t count) {
    T* r = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += align_up(count * sizeof(T), 256);
    return r;
  }
};

tlq_status check_params(const tlq_params* p) {
  if (!p) return TLQ_ERR_NULL;
  if (p->struct_size != sizeof(tlq_params)) return TLQ_ERR_UNSUPPORTED;
  if (p->bits < 2 || p->bits > 8) return TLQ_ERR_UNSUPPORTED;
  if (p->group < 0 || (p->group % 8) != 0) return TLQ_ERR_UNSUPPORTED;
  if (p->symmetric != 0 && p->symmetric != 1) return TLQ_ERR_UNSUPPORTED;
  if (p->act_bits != 0 && (p->act_bits < 2 || p->act_bits > 8)) return TLQ_ERR_UNSUPPORTED;
  if (p->xstat_kind != 0 && p->xstat_kind != 1) return TLQ_ERR_UNSUPPORTED;
  if (p->x_dtype != TLQ_F16 && p->x_dtype != TLQ_BF16) return TLQ_ERR_UNSUPPORTED;
  if (p->yref_dtype != TLQ_F16 && p->yref_dtype != TLQ_BF16 && p->yref_dtype != TLQ_F32)
    return TLQ_ERR_UNSUPPORTED;
  return TLQ_OK;
}

bool dims_ok(int64_t rows, int64_t cols, int64_t ld) {
  return rows > 0 && cols > 0 && ld >= cols && rows < (1LL << 31) && cols < (1LL << 31);
}
bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }
bool mat16_aligned(const void* p, int64_t ld) { return aligned(p, 16) && (ld % 8) == 0; }
bool mat_aligned(const void* p, int64_t ld, int dtype) {
  return dtype == TLQ_F32 ? (aligned(p, 16) && (ld % 4) == 0) : mat16_aligned(p, ld);
}
tlq_status check_cin(int64_t c_in, const tlq_params* p) {
  if ((c_in % 8) != 0) return TLQ_ERR_SHAPE;
  if (p->group != 0 && (c_in % p->group) != 0) return TLQ_ERR_SHAPE;
  return TLQ_OK;
}
tlq_status check_ws(const void* ws, size_t have, size_t need) {
  if (need == 0) return TLQ_OK;
  if (!ws || have < need) return TLQ_ERR_WORKSPACE;
  if (!aligned(ws, 256)) return TLQ_ERR_ALIGN;
  return TLQ_OK;
}
tlq_status hip_status(hipError_t e) { return e == hipSuccess ? TLQ_OK : TLQ_ERR_LAUNCH; }

#define TLQ_TRY(expr) do { tlq_status st_ = (expr); if (st_ != TLQ_OK) return st_; } while (0)
#define TLQ_HIP(expr) do { if ((expr) != hipSuccess) return TLQ_ERR_LAUNCH; } while (0)

// ---- workspace plans -----------------------------------------------------------
// With bf16 inputs the computed operand is kept in fp16 and the tokens are re-expressed
// exactly in fp16 (see launch_xprep): `xh` holds them, `xmax` the bits of max|X|.
// With activation quantisation (act_bits > 0) every candidate has its own token matrix
// (fp16 integer codes, `xc`, produced `act_batch` candidates at a time) and per-token
// steps `sig`; the tokens themselves are never an MFMA operand, so `xh` is not needed.
constexpr size_t kActBatchBytes = (size_t)8 << 30;
int act_batch(int64_t n_tok, int64_t c_in, int n_alpha) {
  const size_t per = (size_t)n_tok * c_in * 2;
  size_t nb = kActBatchBytes / (per ? per : 1);
  if (nb < 1) nb = 1;
  return nb > (size_t)n_alpha ? n_alpha : (int)nb;
}
// The folded weights are rounded to 16 bits relative to their own size, while the loss measures
// the much smaller quantisation error.  At real layer sizes and 2..5 bits that rounding is far
// below the 1e-3 bar (it averages over millions of residual terms); it shows from 6 bits on and
// on problems smaller than one 256 x 256 tile, where a few terms carry the loss.  The search then
// contracts the tokens with F_k = What_k - W, which is rounded relative to the small difference,
// and compares with D0 = Y_ref - X W^T kept in float: Y_ref - X What_k^T = D0 - X F_k^T.
bool use_diff_form(const tlq_params* p, int64_t n_tok, int64_t c_out) {
  return p->act_bits == 0 && (p->bits >= 6 || n_tok * c_out < 256 * 256);
}
struct SearchPlan {
  double* xs_partial; float* x_stat; float* s_table; float* inv_table; float* partial;
  uint16_t* what; uint32_t* xmax; uint16_t* xh; float* sig; float* rsig; uint16_t* xc; int nb; size_t bytes;
  int64_t tiles_o, tiles_t;
  float* d0; int64_t ldd;   // difference form: Y_ref - X W^T as float
};
SearchPlan plan_search(void* ws, int64_t n_tok, int64_t c_in, int64_t c_out, int n_alpha, bool bf16,
                       bool act, bool diff) {
  SearchPlan s;
  Carver c(ws);
  gemm_tile_counts(n_tok, c_out, &s.tiles_o, &s.tiles_t);
  s.xs_partial = c.take<double>((size_t)xstat_chunks(n_tok) * c_in);
  s.x_stat = c.take<float>((size_t)c_in);
  s.s_table = c.take<float>((size_t)n_alpha * c_in);
  s.inv_table = c.take<float>((size_t)n_alpha * c_in);
  s.partial = c.take<float>((size_t)n_alpha * s.tiles_o * s.tiles_t);
  s.what = c.take<uint16_t>((size_t)n_alpha * c_out * c_in);
  s.xmax = c.take<uint32_t>(1);
  s.xh = (bf16 && !act) ? c.take<uint16_t>((size_t)n_tok * c_in) : nullptr;
  s.nb = act ? act_batch(n_tok, c_in, n_alpha) : 0;
  s.sig = act ? c.take<float>((size_t)n_alpha * n_tok) : nullptr;
  s.rsig = act ? c.take<float>((size_t)s.nb * n_tok) : nullptr;
  s.xc = act ? c.take<uint16_t>((size_t)s.nb * n_tok * c_in) : nullptr;
  s.ldd = (int64_t)align_up((size_t)c_out, 4);
  s.d0 = diff ? c.take<float>((size_t)n_tok * s.ldd) : nullptr;
  s.bytes = c.off;
  return s;
}

struct ErrPlan {
  float* partial; float* tok_partial; uint16_t* folded; uint32_t* xmax; uint16_t* xh; float* sig;
  size_t bytes; int64_t tiles_o, tiles_t;   // xh doubles as the code matrix in act mode
};
ErrPlan plan_err(void* ws, int64_t n_tok, int64_t c_in, int64_t c_out, bool bf16, bool act) {
  ErrPlan e;
  Carver c(ws);
  gemm_tile_counts(n_tok, c_out, &e.tiles_o, &e.tiles_t);
  e.partial = c.take<float>((size_t)e.tiles_o * e.tiles_t);
  e.tok_partial = c.take<float>((size_t)e.tiles_o * n_tok);
  e.folded = c.take<uint16_t>((size_t)c_out * c_in);
  e.xmax = c.take<uint32_t>(1);
  e.xh = (bf16 || act) ? c.take<uint16_t>((size_t)n_tok * c_in) : nullptr;
  e.sig = act ? c.take<float>((size_t)n_tok) : nullptr;
  e.bytes = c.off;
  return e;
}

// Tokens re-expressed for the matrix cores (see launch_xprep), shared by several calls on one X:
// [bits of max|X| : 256 bytes][X * 2^-shift as fp16, dense n_tok x c_in].
struct Prepared { const uint32_t* xmax; const uint16_t* xh; };
bool needs_prepared(const tlq_params* p) { return p->x_dtype == TLQ_BF16 && p->act_bits == 0; }
Prepared view_prepared(const void* buf) {
  return Prepared{(const uint32_t*)buf, (const uint16_t*)((const unsigned char*)buf + 256)};
}

// Second-moment form: the caller-held result of tlq_token_gram
// [double factor : 256 bytes][float col_scale[c_in]][fp16 C[c_in, c_in]]
struct GramView { double* factor; float* col_scale; uint16_t* C; size_t bytes; };
GramView view_gram(void* buf, int64_t c_in) {
  Carver c(buf);
  GramView v;
  v.factor = c.take<double>(1);
  v.col_scale = c.take<float>((size_t)c_in);
  v.C = c.take<uint16_t>((size_t)c_in * c_in);
  v.bytes = c.off;
  return v;
}
// The token product has only (c_in / 256)^2 / 2 output tiles and a very long contraction: it is
// split along the tokens into n_split partial products (summed afterwards in a fixed order) so
// that the launch has a few thousand workgroups.
struct GramPlan { float* wmax; int* e; uint16_t* xst; float* H; int64_t kp, kc; int n_split; size_t bytes; };
GramPlan plan_gram(void* ws, int64_t n_tok, int64_t c_in) {
  GramPlan g;
  Carver c(ws);
  int64_t to, tt;
  gemm_tile_counts(c_in, c_in, &to, &tt);
  const int64_t live = to * (to + 1) / 2;
  // measured: more, shorter splits run faster up to 16 (5120 channels: 6.0 ms with 4, 3.9 ms with 16;
  // beyond 16 it collapses); 13824 channels: 4 splits 28.2 ms, 5: 29.7, 12 - 16: 27.5 + a longer sum
  int64_t ns = (5000 + live - 1) / live;
  const int64_t max_ns = n_tok / 4096;                 // at least 4096 tokens (64 k-tiles) per split
  ns = ns > 16 ? 16 : ns;
  ns = ns > max_ns ? max_ns : ns;
  g.n_split = (int)(ns < 1 ? 1 : ns);
  g.kc = (int64_t)align_up((size_t)((n_tok + g.n_split - 1) / g.n_split), 64);
  g.kp = g.kc * g.n_split;
  g.wmax = c.take<float>(1);
  g.e = c.take<int>((size_t)c_in);
  g.xst = c.take<uint16_t>((size_t)c_in * g.kp);
  g.H = c.take<float>((size_t)g.n_split * c_in * c_in);
  g.bytes = c.off;
  return g;
}
struct GramSearchPlan { float* s_table; float* inv_table; float* partial; uint16_t* dq; size_t bytes;
                        int64_t tiles_o, tiles_t; };
GramSearchPlan plan_gram_search(void* ws, int64_t c_in, int64_t c_out, int n_alpha) {
  GramSearchPlan s;
  Carver c(ws);
  gemm_tile_counts(c_out, c_in, &s.tiles_o, &s.tiles_t);   // weight rows take the token role
  s.s_table = c.take<float>((size_t)n_alpha * c_in);
  s.inv_table = c.take<float>((size_t)n_alpha * c_in);
  s.partial = c.take<float>((size_t)n_alpha * s.tiles_o * s.tiles_t);
  s.dq = c.take<uint16_t>((size_t)n_alpha * c_out * c_in);
  s.bytes = c.off;
  return s;
}
}  // namespace

extern "C" {

const char* tlq_status_string(int s) {
  switch (s) {
    case TLQ_OK: return "ok";
    case TLQ_ERR_NULL: return "required pointer is NULL";
    case TLQ_ERR_SHAPE: return "invalid or inconsistent shape";
    case TLQ_ERR_UNSUPPORTED: return "unsupported parameter value";
    case TLQ_ERR_WORKSPACE: return "workspace missing or too small";
    case TLQ_ERR_ALIGN: return "pointer or stride not aligned";
    case TLQ_ERR_LAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

int tlq_version(void) { return TLQ_VERSION; }

// host-side self check of the contraction kernels' block -> tile map (no GPU work)
int64_t tlq_selftest_tile_map(int64_t n_tok, int64_t c_in, int64_t c_out, int32_t n_cand, int64_t* blocks) {
  return tile_map_defects(n_tok, c_in, c_out, n_cand, blocks);
}

// ------------------------------------------------------------------------ S0
size_t tlq_x_stat_workspace_bytes(int64_t n_tok, int64_t c_in) {
  if (n_tok <= 0 || c_in <= 0) return 0;
  return align_up((size_t)xstat_chunks(n_tok) * (size_t)c_in * sizeof(double), 256);
}

tlq_status tlq_x_stat(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                      const tlq_params* p, float* x_stat, void* workspace,
                      size_t workspace_bytes, void* stream) {
  if (!X || !x_stat) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (!dims_ok(n_tok, c_in, ldx) || (c_in % 8) != 0) return TLQ_ERR_SHAPE;
  if (!mat16_aligned(X, ldx)) return TLQ_ERR_ALIGN;
  TLQ_TRY(check_ws(workspace, workspace_bytes, tlq_x_stat_workspace_bytes(n_tok, c_in)));
  return hip_status(launch_xstat(X, n_tok, c_in, ldx, p->x_dtype == TLQ_BF16, p->xstat_kind,
                                 (double*)workspace, x_stat, (hipStream_t)stream));
}

// ------------------------------------------- gradient-guided selection (Sec. 3.1.2)
size_t tlq_token_importance_workspace_bytes(int64_t n_samples, int64_t n_pos) {
  if (n_samples <= 0 || n_pos <= 0) return 0;
  return align_up((size_t)n_samples * (size_t)n_pos * sizeof(double), 256);
}

tlq_status tlq_token_importance(const void* G, int64_t n_samples, int64_t n_pos, int64_t c,
                                int64_t ldg, int32_t l2, const tlq_params* p, double* sum_n,
                                void* workspace, size_t workspace_bytes, void* stream) {
  if (!G || !sum_n) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (n_samples <= 0 || n_pos <= 0 || c <= 0 || ldg < c || n_samples * n_pos >= (1LL << 31))
    return TLQ_ERR_SHAPE;
  if (l2 != 0 && l2 != 1) return TLQ_ERR_UNSUPPORTED;
  if (!aligned(G, 2) || !aligned(sum_n, 8)) return TLQ_ERR_ALIGN;
  TLQ_TRY(check_ws(workspace, workspace_bytes, tlq_token_importance_workspace_bytes(n_samples, n_pos)));
  return hip_status(launch_token_importance(G, n_samples, n_pos, c, ldg, p->x_dtype == TLQ_BF16, l2 != 0,
                                            (double*)workspace, sum_n, (hipStream_t)stream));
}

tlq_status tlq_topk_mask(const double* sum_n, int64_t n_pos, int64_t k, uint8_t* mask, void* stream) {
  if (!sum_n || !mask) return TLQ_ERR_NULL;
  if (n_pos <= 0 || k < 0 || k > n_pos) return TLQ_ERR_SHAPE;
  if (n_pos > 65536) return TLQ_ERR_UNSUPPORTED;
  return hip_status(launch_topk_mask(sum_n, n_pos, k, mask, (hipStream_t)stream));
}

tlq_status tlq_x_stat_masked(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                             const uint8_t* pos_mask, int64_t period, const tlq_params* p,
                             float* x_stat, void* workspace, size_t workspace_bytes, void* stream) {
  if (!X || !x_stat || !pos_mask) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (!dims_ok(n_tok, c_in, ldx) || (c_in % 8) != 0 || period <= 0 || period > n_tok) return TLQ_ERR_SHAPE;
  if (!mat16_aligned(X, ldx)) return TLQ_ERR_ALIGN;
  TLQ_TRY(check_ws(workspace, workspace_bytes, tlq_x_stat_workspace_bytes(n_tok, c_in)));
  return hip_status(launch_xstat(X, n_tok, c_in, ldx, p->x_dtype == TLQ_BF16, 1, (double*)workspace,
                                 x_stat, (hipStream_t)stream, pos_mask, period));
}

// ------------------------------------------------------------------------ S1
tlq_status tlq_scale_table(const float* x_stat, int64_t c_in, const float* alpha_grid,
                           int32_t n_alpha, float* s_table, void* stream) {
  if (!x_stat || !alpha_grid || !s_table) return TLQ_ERR_NULL;
  if (c_in <= 0 || n_alpha <= 0 || n_alpha > TLQ_MAX_ALPHA) return TLQ_ERR_SHAPE;
  return hip_status(launch_scale_table(x_stat, c_in, alpha_grid, n_alpha, s_table, nullptr, nullptr,
                                       (hipStream_t)stream));
}

// ------------------------------------------------------------------------ S2
tlq_status tlq_fake_quant(const void* W, int64_t c_out, int64_t c_in, int64_t ldw,
                          const float* s, const tlq_params* p, uint8_t* codes, uint8_t* zp,
                          float* delta, void* Wdq, int64_t ld_dq, void* stream) {
  if (!W) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (!dims_ok(c_out, c_in, ldw)) return TLQ_ERR_SHAPE;
  TLQ_TRY(check_cin(c_in, p));
  if (Wdq && ld_dq < c_in) return TLQ_ERR_SHAPE;
  if (!mat16_aligned(W, ldw)) return TLQ_ERR_ALIGN;
  if (Wdq && !mat16_aligned(Wdq, ld_dq)) return TLQ_ERR_ALIGN;
  if ((codes && !aligned(codes, 8)) || (s && !aligned(s, 16)) || (delta && !aligned(delta, 4)))
    return TLQ_ERR_ALIGN;
  QuantArgs q{};
  q.W = W; q.c_out = c_out; q.c_in = c_in; q.ldw = ldw; q.bf16 = p->x_dtype == TLQ_BF16;
  q.bits = p->bits; q.group = p->group; q.symmetric = p->symmetric;
  q.s_table = s; q.inv_table = nullptr; q.n_cand = 1;
  q.what = nullptr; q.what_cand_stride = 0;
  q.codes = codes; q.zp = zp; q.delta = delta; q.wdq = Wdq; q.ld_dq = ld_dq;
  return hip_status(launch_fake_quant(q, (hipStream_t)stream));
}

// ------------------------------------------------------------------------ Q_a
tlq_status tlq_act_fake_quant(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                              const float* inv_s, const tlq_params* p, void* codes, float* sigma,
                              void* stream) {
  if (!X || !codes || !sigma) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (p->act_bits == 0) return TLQ_ERR_UNSUPPORTED;
  if (!dims_ok(n_tok, c_in, ldx) || (c_in % 8) != 0) return TLQ_ERR_SHAPE;
  if (!mat16_aligned(X, ldx) || !aligned(codes, 16) || (inv_s && !aligned(inv_s, 4))) return TLQ_ERR_ALIGN;
  return hip_status(launch_act_quant(X, n_tok, c_in, ldx, p->x_dtype == TLQ_BF16, inv_s, 0, 1,
                                     p->act_bits, codes, sigma, nullptr, (hipStream_t)stream));
}

// -------------------------------------------------------------------- S3 + S4
size_t tlq_weighted_layer_err_workspace_bytes(int64_t n_tok, int64_t c_in, int64_t c_out,
                                              const tlq_params* p) {
  if (n_tok <= 0 || c_in <= 0 || c_out <= 0 || check_params(p) != TLQ_OK) return 0;
  return plan_err(nullptr, n_tok, c_in, c_out, p->x_dtype == TLQ_BF16, p->act_bits != 0).bytes;
}

tlq_status tlq_weighted_layer_err(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                                  const void* Wdq, int64_t c_out, int64_t ldw,
                                  const float* inv_s, const void* Y_ref, int64_t ldy,
                                  const float* token_w, const tlq_params* p, float* loss,
                                  float* per_token_err, void* workspace, size_t workspace_bytes,
                                  void* stream) {
  if (!X || !Wdq || !Y_ref || !token_w || !loss) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (!dims_ok(n_tok, c_in, ldx) || !dims_ok(c_out, c_in, ldw) || !dims_ok(n_tok, c_out, ldy))
    return TLQ_ERR_SHAPE;
  if ((c_in % 8) != 0) return TLQ_ERR_SHAPE;
  if (!mat16_aligned(X, ldx) || !mat16_aligned(Wdq, ldw) || !mat_aligned(Y_ref, ldy, p->yref_dtype))
    return TLQ_ERR_ALIGN;
  TLQ_TRY(check_ws(workspace, workspace_bytes,
                   tlq_weighted_layer_err_workspace_bytes(n_tok, c_in, c_out, p)));
  hipStream_t st = (hipStream_t)stream;
  const bool bf16 = p->x_dtype == TLQ_BF16;
  const bool act = p->act_bits != 0;
  ErrPlan e = plan_err(workspace, n_tok, c_in, c_out, bf16, act);
  GemmArgs g{};
  g.X = X; g.n_tok = n_tok; g.c_in = c_in; g.ldx = ldx;
  g.Wh = Wdq; g.c_out = c_out; g.ldw = ldw; g.w_cand_stride = 0; g.n_cand = 1; g.bf16 = bf16;
  if (act) {
    // Q_a(x * inv_s) as exact fp16 integer codes + per-token steps; the weights stay unfolded
    TLQ_HIP(launch_act_quant(X, n_tok, c_in, ldx, bf16, inv_s, 0, 1, p->act_bits, e.xh, e.sig, nullptr, st));
    g.X = e.xh; g.ldx = c_in; g.tok_scale = e.sig; g.bf16 = false;
    if (bf16) {
      TLQ_HIP(launch_fold_scale(Wdq, c_out, c_in, ldw, true, nullptr, nullptr, true, e.folded, st));
      g.Wh = e.folded; g.ldw = c_in;
    }
  } else if (inv_s) {
    // the folded operand is a computed value: with bf16 inputs keep it (and X) in fp16
    if (bf16) {
      TLQ_HIP(launch_xprep(X, n_tok, c_in, ldx, e.xmax, e.xh, st));
      g.X = e.xh; g.ldx = c_in; g.bf16 = false;
    }
    TLQ_HIP(launch_fold_scale(Wdq, c_out, c_in, ldw, bf16, inv_s, bf16 ? e.xmax : nullptr, bf16,
                              e.folded, st));
    g.Wh = e.folded; g.ldw = c_in;
  }
  g.Yref = Y_ref; g.ldy = ldy; g.yref_dtype = p->yref_dtype; g.token_w = token_w;
  g.partial = e.partial; g.tok_partial = per_token_err ? e.tok_partial : nullptr;
  TLQ_HIP(launch_gemm_loss(g, st));
  TLQ_HIP(launch_finalize(e.partial, 1, e.tiles_o * e.tiles_t, c_out, nullptr, c_in, loss, nullptr,
                          nullptr, st));
  if (per_token_err)
    TLQ_HIP(launch_token_err_reduce(e.tok_partial, e.tiles_o, n_tok, c_out, per_token_err, st));
  return TLQ_OK;
}

// ------------------------------------------------------------------- S0 .. S5
size_t tlq_scale_search_workspace_bytes(int64_t n_tok, int64_t c_in, int64_t c_out,
                                        int32_t n_alpha, const tlq_params* p) {
  if (n_tok <= 0 || c_in <= 0 || c_out <= 0 || n_alpha <= 0 || n_alpha > TLQ_MAX_ALPHA ||
      check_params(p) != TLQ_OK)
    return 0;
  return plan_search(nullptr, n_tok, c_in, c_out, n_alpha, p->x_dtype == TLQ_BF16, p->act_bits != 0,
                     use_diff_form(p, n_tok, c_out)).bytes;
}

static tlq_status scale_search_impl(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                            const void* W, int64_t c_out, int64_t ldw, const void* Y_ref,
                            int64_t ldy, const float* token_w, const float* alpha_grid,
                            int32_t n_alpha, const tlq_params* p, const float* x_stat_in,
                            float* best_scales, int32_t* best_idx, float* losses,
                            float* s_table_out, void* workspace, size_t workspace_bytes,
                            void* stream, const void* prepared) {
  if (!X || !W || !Y_ref || !token_w || !alpha_grid || !best_scales || !best_idx || !losses)
    return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (n_alpha <= 0 || n_alpha > TLQ_MAX_ALPHA) return TLQ_ERR_SHAPE;
  if (!dims_ok(n_tok, c_in, ldx) || !dims_ok(c_out, c_in, ldw) || !dims_ok(n_tok, c_out, ldy))
    return TLQ_ERR_SHAPE;
  TLQ_TRY(check_cin(c_in, p));
  if (!mat16_aligned(X, ldx) || !mat16_aligned(W, ldw) || !mat_aligned(Y_ref, ldy, p->yref_dtype))
    return TLQ_ERR_ALIGN;
  TLQ_TRY(check_ws(workspace, workspace_bytes,
                   tlq_scale_search_workspace_bytes(n_tok, c_in, c_out, n_alpha, p)));
  hipStream_t st = (hipStream_t)stream;
  const bool bf16 = p->x_dtype == TLQ_BF16;
  const bool act = p->act_bits != 0;
  const bool diff = use_diff_form(p, n_tok, c_out);
  SearchPlan s = plan_search(workspace, n_tok, c_in, c_out, n_alpha, bf16, act, diff);
  if (prepared && !aligned(prepared, 256)) return TLQ_ERR_ALIGN;
  const bool use_prep = prepared && needs_prepared(p);
  if (use_prep) {   // the caller's copy replaces the workspace one
    const Prepared v = view_prepared(prepared);
    s.xmax = const_cast<uint32_t*>(v.xmax); s.xh = const_cast<uint16_t*>(v.xh);
  }

  const float* x_stat = x_stat_in;
  if (!x_stat) {  // S0
    TLQ_HIP(launch_xstat(X, n_tok, c_in, ldx, bf16, p->xstat_kind, s.xs_partial, s.x_stat, st));
    x_stat = s.x_stat;
  }
  if (bf16 && !act && !use_prep) TLQ_HIP(launch_xprep(X, n_tok, c_in, ldx, s.xmax, s.xh, st));
  // S1
  TLQ_HIP(launch_scale_table(x_stat, c_in, alpha_grid, n_alpha, s.s_table, s.inv_table,
                             (bf16 && !act) ? s.xmax : nullptr, st));
  if (s_table_out)
    TLQ_HIP(hipMemcpyAsync(s_table_out, s.s_table, (size_t)n_alpha * c_in * sizeof(float),
                           hipMemcpyDeviceToDevice, st));
  // S2: all candidates' folded operands in one pass over W
  QuantArgs q{};
  q.W = W; q.c_out = c_out; q.c_in = c_in; q.ldw = ldw; q.bf16 = bf16;
  q.bits = p->bits; q.group = p->group; q.symmetric = p->symmetric;
  // (with activation quantisation 1/s belongs to Q_a's argument, so the weights stay unfolded)
  q.s_table = s.s_table; q.inv_table = act ? nullptr : s.inv_table; q.n_cand = n_alpha;
  q.what = s.what; q.what_cand_stride = c_out * c_in; q.what_f16 = true;
  q.diff = diff; q.xmax_bits = (diff && bf16) ? s.xmax : nullptr;
  TLQ_HIP(launch_fake_quant(q, st));
  if (diff) {  // D0 = Y_ref - X W^T (exact products of the 16-bit inputs, float accumulation)
    GemmArgs r{};
    r.X = X; r.n_tok = n_tok; r.c_in = c_in; r.ldx = ldx;
    r.Wh = W; r.c_out = c_out; r.ldw = ldw; r.w_cand_stride = 0; r.n_cand = 1; r.bf16 = bf16;
    r.Yout = s.d0; r.ldo = s.ldd; r.yout_dtype = TLQ_F32;
    TLQ_HIP(launch_gemm_store(r, st));
    TLQ_HIP(launch_sub_from_y(Y_ref, ldy, p->yref_dtype, s.d0, s.ldd, n_tok, c_out, st));
  }
  // S3 + S4: one launch over the stacked candidates (fp16 operands in either case)
  GemmArgs g{};
  g.X = bf16 ? (const void*)s.xh : X; g.n_tok = n_tok; g.c_in = c_in; g.ldx = bf16 ? c_in : ldx;
  g.Wh = s.what; g.c_out = c_out; g.ldw = c_in; g.w_cand_stride = c_out * c_in;
  g.n_cand = n_alpha; g.bf16 = false;
  g.Yref = Y_ref; g.ldy = ldy; g.yref_dtype = p->yref_dtype; g.token_w = token_w;
  if (diff) { g.Yref = s.d0; g.ldy = s.ldd; g.yref_dtype = TLQ_F32; }
  g.partial = s.partial; g.tok_partial = nullptr;
  if (!act) {
    // patch shape by measurement: 8 x 4 tiles gain ~1 % on square and widening layers and lose
    // 0.5 - 3 % on the narrowing, deep ones (down_proj)
    g.wide_patch = c_in <= 2 * c_out;
    TLQ_HIP(launch_gemm_loss(g, st));
  } else {
    // Q_a(x / s_k) differs per candidate: quantise the tokens for a batch of candidates,
    // contract each candidate with its own code matrix, scale by the per-token step
    const int64_t tiles = s.tiles_o * s.tiles_t;
    for (int k0 = 0; k0 < n_alpha; k0 += s.nb) {
      const int nb = (n_alpha - k0) < s.nb ? (n_alpha - k0) : s.nb;
      TLQ_HIP(launch_act_quant(X, n_tok, c_in, ldx, bf16, s.inv_table, k0, nb, p->act_bits, s.xc,
                               s.sig + (size_t)k0 * n_tok, s.rsig, st));
      GemmArgs b = g;
      b.X = s.xc; b.ldx = c_in; b.x_cand_stride = n_tok * c_in;
      b.cand_outer = true;   // nothing is shared between candidates here: walk them one after the other
      b.tok_scale = s.sig + (size_t)k0 * n_tok;
      b.Wh = s.what + (size_t)k0 * c_out * c_in; b.n_cand = nb;
      b.partial = s.partial + (size_t)k0 * tiles;
      TLQ_HIP(launch_gemm_loss(b, st));
    }
  }
  // S4 combine + S5
  TLQ_HIP(launch_finalize(s.partial, n_alpha, s.tiles_o * s.tiles_t, c_out, s.s_table, c_in, losses,
                          best_idx, best_scales, st));
  return TLQ_OK;
}

tlq_status tlq_scale_search(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                            const void* W, int64_t c_out, int64_t ldw, const void* Y_ref,
                            int64_t ldy, const float* token_w, const float* alpha_grid,
                            int32_t n_alpha, const tlq_params* p, const float* x_stat_in,
                            float* best_scales, int32_t* best_idx, float* losses,
                            float* s_table_out, void* workspace, size_t workspace_bytes,
                            void* stream) {
  return scale_search_impl(X, n_tok, c_in, ldx, W, c_out, ldw, Y_ref, ldy, token_w, alpha_grid, n_alpha, p,
                           x_stat_in, best_scales, best_idx, losses, s_table_out, workspace, workspace_bytes,
                           stream, nullptr);
}

tlq_status tlq_scale_search_prepared(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                                     const void* W, int64_t c_out, int64_t ldw, const void* Y_ref,
                                     int64_t ldy, const float* token_w, const float* alpha_grid,
                                     int32_t n_alpha, const tlq_params* p, const float* x_stat_in,
                                     float* best_scales, int32_t* best_idx, float* losses,
                                     float* s_table_out, void* workspace, size_t workspace_bytes,
                                     void* stream, const void* prepared) {
  return scale_search_impl(X, n_tok, c_in, ldx, W, c_out, ldw, Y_ref, ldy, token_w, alpha_grid, n_alpha, p,
                           x_stat_in, best_scales, best_idx, losses, s_table_out, workspace, workspace_bytes,
                           stream, prepared);
}

// ------------------------------------------------ tokens prepared once for several calls
size_t tlq_prepared_tokens_bytes(int64_t n_tok, int64_t c_in, const tlq_params* p) {
  if (n_tok <= 0 || c_in <= 0 || check_params(p) != TLQ_OK || !needs_prepared(p)) return 0;
  return 256 + align_up((size_t)n_tok * (size_t)c_in * 2, 256);
}

tlq_status tlq_prepare_tokens(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx, const tlq_params* p,
                              void* prepared, size_t prepared_bytes, void* stream) {
  if (!X) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (!dims_ok(n_tok, c_in, ldx) || (c_in % 8) != 0) return TLQ_ERR_SHAPE;
  if (!mat16_aligned(X, ldx)) return TLQ_ERR_ALIGN;
  const size_t need = tlq_prepared_tokens_bytes(n_tok, c_in, p);
  if (need == 0) return TLQ_OK;                       // nothing to prepare for these parameters
  if (!prepared || prepared_bytes < need) return TLQ_ERR_WORKSPACE;
  if (!aligned(prepared, 256)) return TLQ_ERR_ALIGN;
  const Prepared v = view_prepared(prepared);
  return hip_status(launch_xprep(X, n_tok, c_in, ldx, const_cast<uint32_t*>(v.xmax), const_cast<uint16_t*>(v.xh),
                                 (hipStream_t)stream));
}

// ---------------------------------------- second-moment form of the weight-only search
size_t tlq_token_gram_bytes(int64_t c_in) {
  if (c_in <= 0) return 0;
  return view_gram(nullptr, c_in).bytes;
}

size_t tlq_token_gram_workspace_bytes(int64_t n_tok, int64_t c_in) {
  if (n_tok <= 0 || c_in <= 0) return 0;
  return plan_gram(nullptr, n_tok, c_in).bytes;
}

tlq_status tlq_token_gram(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx, const float* token_w,
                          const tlq_params* p, void* gram, size_t gram_bytes, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (!X || !token_w) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (!dims_ok(n_tok, c_in, ldx) || (c_in % 8) != 0) return TLQ_ERR_SHAPE;
  if (!mat16_aligned(X, ldx) || !aligned(token_w, 4)) return TLQ_ERR_ALIGN;
  if (!gram || gram_bytes < tlq_token_gram_bytes(c_in)) return TLQ_ERR_WORKSPACE;
  if (!aligned(gram, 256)) return TLQ_ERR_ALIGN;
  TLQ_TRY(check_ws(workspace, workspace_bytes, tlq_token_gram_workspace_bytes(n_tok, c_in)));
  hipStream_t st = (hipStream_t)stream;
  const GramView v = view_gram(gram, c_in);
  const GramPlan g = plan_gram(workspace, n_tok, c_in);
  TLQ_HIP(launch_gram_operand(X, n_tok, c_in, ldx, p->x_dtype == TLQ_BF16, token_w, g.wmax, g.xst, g.kp, st));
  // H_s[j, i] = sum over the tokens of split s of xs[i, t] xs[j, t]: both operands are the transposed
  // tokens, the splits take the role of candidates (column ranges of the same matrix)
  GemmArgs r{};
  r.X = g.xst; r.n_tok = c_in; r.c_in = g.kc; r.ldx = g.kp; r.x_cand_stride = g.kc;
  r.Wh = g.xst; r.c_out = c_in; r.ldw = g.kp; r.w_cand_stride = g.kc; r.n_cand = g.n_split; r.bf16 = false;
  r.Yout = g.H; r.ldo = c_in; r.yout_dtype = TLQ_F32; r.o_cand_stride = c_in * c_in; r.tri = true;
  r.cand_outer = true; r.wide_patch = c_in >= 32 * 256;   // measured: 8 x 4 patches pay from ~32 tile rows on
  TLQ_HIP(launch_gemm_store(r, st));
  return hip_status(launch_gram_finish(g.H, c_in, g.n_split, c_in * c_in, g.wmax, g.e, v.factor, v.col_scale,
                                       v.C, st));
}

size_t tlq_scale_search_gram_workspace_bytes(int64_t c_in, int64_t c_out, int32_t n_alpha,
                                             const tlq_params* p) {
  if (c_in <= 0 || c_out <= 0 || n_alpha <= 0 || n_alpha > TLQ_MAX_ALPHA || check_params(p) != TLQ_OK)
    return 0;
  return plan_gram_search(nullptr, c_in, c_out, n_alpha).bytes;
}

tlq_status tlq_scale_search_gram(const void* gram, int64_t c_in, const void* W, int64_t c_out, int64_t ldw,
                                 const float* alpha_grid, int32_t n_alpha, const tlq_params* p,
                                 const float* x_stat, float* best_scales, int32_t* best_idx, float* losses,
                                 float* s_table_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!gram || !W || !alpha_grid || !x_stat || !best_scales || !best_idx || !losses) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (p->act_bits != 0) return TLQ_ERR_UNSUPPORTED;   // Q_a makes f_q non-linear in the tokens
  if (n_alpha <= 0 || n_alpha > TLQ_MAX_ALPHA) return TLQ_ERR_SHAPE;
  if (!dims_ok(c_out, c_in, ldw)) return TLQ_ERR_SHAPE;
  TLQ_TRY(check_cin(c_in, p));
  if (!mat16_aligned(W, ldw) || !aligned(gram, 256)) return TLQ_ERR_ALIGN;
  TLQ_TRY(check_ws(workspace, workspace_bytes,
                   tlq_scale_search_gram_workspace_bytes(c_in, c_out, n_alpha, p)));
  hipStream_t st = (hipStream_t)stream;
  const GramView v = view_gram(const_cast<void*>(gram), c_in);
  const GramSearchPlan s = plan_gram_search(workspace, c_in, c_out, n_alpha);
  TLQ_HIP(launch_scale_table(x_stat, c_in, alpha_grid, n_alpha, s.s_table, s.inv_table, nullptr, st));
  if (s_table_out)
    TLQ_HIP(hipMemcpyAsync(s_table_out, s.s_table, (size_t)n_alpha * c_in * sizeof(float),
                           hipMemcpyDeviceToDevice, st));
  // D'_k = (deq_k / s_k - W) * col_scale for every candidate, fp16
  QuantArgs q{};
  q.W = W; q.c_out = c_out; q.c_in = c_in; q.ldw = ldw; q.bf16 = p->x_dtype == TLQ_BF16;
  q.bits = p->bits; q.group = p->group; q.symmetric = p->symmetric;
  q.s_table = s.s_table; q.inv_table = s.inv_table; q.n_cand = n_alpha;
  q.what = s.dq; q.what_cand_stride = c_out * c_in; q.what_f16 = true;
  q.diff = true; q.xmax_bits = nullptr; q.col_scale = v.col_scale;
  TLQ_HIP(launch_fake_quant(q, st));
  // partial = sum_{o,i} (D'_k C)[o,i] D'_k[o,i]: the weight rows play the tokens, C the weights
  GemmArgs g{};
  g.X = s.dq; g.n_tok = c_out; g.c_in = c_in; g.ldx = c_in; g.x_cand_stride = c_out * c_in;
  g.Wh = v.C; g.c_out = c_in; g.ldw = c_in; g.w_cand_stride = 0; g.n_cand = n_alpha; g.bf16 = false;
  g.Yref = s.dq; g.ldy = c_in; g.yref_dtype = TLQ_F16; g.y_cand_stride = c_out * c_in;
  g.partial = s.partial; g.cand_outer = true;   // D'_k and C stay cache-resident for one candidate at a time
  g.wide_patch = true;   // consecutive patches keep their 8 panels of C and fetch 4 new ones of D'_k
  g.sym_k = true;        // C is symmetric: contract from each tile's diagonal block on, the rest counted twice
  TLQ_HIP(launch_gemm_dot(g, st));
  TLQ_HIP(launch_finalize(s.partial, n_alpha, s.tiles_o * s.tiles_t, c_out, s.s_table, c_in, losses,
                          best_idx, best_scales, st, v.factor));
  return TLQ_OK;
}

// ---------------------------------------------------------------- f_fp output
tlq_status tlq_ref_output(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                          const void* W, int64_t c_out, int64_t ldw, void* Y, int64_t ldy,
                          const tlq_params* p, void* stream) {
  if (!X || !W || !Y) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (!dims_ok(n_tok, c_in, ldx) || !dims_ok(c_out, c_in, ldw) || !dims_ok(n_tok, c_out, ldy))
    return TLQ_ERR_SHAPE;
  if ((c_in % 8) != 0) return TLQ_ERR_SHAPE;
  if (!mat16_aligned(X, ldx) || !mat16_aligned(W, ldw) || !mat_aligned(Y, ldy, p->yref_dtype))
    return TLQ_ERR_ALIGN;
  GemmArgs g{};
  g.X = X; g.n_tok = n_tok; g.c_in = c_in; g.ldx = ldx;
  g.Wh = W; g.c_out = c_out; g.ldw = ldw; g.w_cand_stride = 0; g.n_cand = 1;
  g.bf16 = p->x_dtype == TLQ_BF16;
  g.Yout = Y; g.ldo = ldy; g.yout_dtype = p->yref_dtype;
  g.wide_patch = true;   // one candidate: 8 weight panels stay per patch row, 4 token panels change (+1 .. +4 % measured)
  return hip_status(launch_gemm_store(g, (hipStream_t)stream));
}

// ------------------------------------------------------------------------ S6
size_t tlq_apply_best_workspace_bytes(int64_t n_tok, int64_t c_in, int64_t c_out,
                                      const tlq_params* p) {
  if (n_tok <= 0 || c_in <= 0 || c_out <= 0 || check_params(p) != TLQ_OK) return 0;
  const bool xbuf = p->x_dtype == TLQ_BF16 || p->act_bits != 0;
  return align_up((size_t)c_in * sizeof(float), 256) + align_up((size_t)c_out * c_in * 2, 256) + 256 +
         (xbuf ? align_up((size_t)n_tok * c_in * 2, 256) : 0) +
         (p->act_bits != 0 ? align_up((size_t)n_tok * sizeof(float), 256) : 0);
}

static tlq_status apply_best_impl(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                          const void* W, int64_t c_out, int64_t ldw, const float* s,
                          const tlq_params* p, void* X_next, int64_t ld_next, void* workspace,
                          size_t workspace_bytes, void* stream, const void* prepared) {
  if (!X || !W || !s || !X_next) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (!dims_ok(n_tok, c_in, ldx) || !dims_ok(c_out, c_in, ldw) || !dims_ok(n_tok, c_out, ld_next))
    return TLQ_ERR_SHAPE;
  TLQ_TRY(check_cin(c_in, p));
  if (!mat16_aligned(X, ldx) || !mat16_aligned(W, ldw) || !mat16_aligned(X_next, ld_next) ||
      !aligned(s, 16))
    return TLQ_ERR_ALIGN;
  TLQ_TRY(check_ws(workspace, workspace_bytes, tlq_apply_best_workspace_bytes(n_tok, c_in, c_out, p)));
  hipStream_t st = (hipStream_t)stream;
  const bool bf16 = p->x_dtype == TLQ_BF16;
  Carver c(workspace);
  float* inv = c.take<float>((size_t)c_in);
  uint16_t* what = c.take<uint16_t>((size_t)c_out * c_in);
  uint32_t* xmax = c.take<uint32_t>(1);
  const bool act = p->act_bits != 0;
  uint16_t* xh = (bf16 || act) ? c.take<uint16_t>((size_t)n_tok * c_in) : nullptr;
  float* sig = act ? c.take<float>((size_t)n_tok) : nullptr;
  if (prepared && !aligned(prepared, 256)) return TLQ_ERR_ALIGN;
  if (prepared && needs_prepared(p)) {
    const Prepared v = view_prepared(prepared);
    xmax = const_cast<uint32_t*>(v.xmax); xh = const_cast<uint16_t*>(v.xh);
  } else if (bf16 && !act) {
    TLQ_HIP(launch_xprep(X, n_tok, c_in, ldx, xmax, xh, st));
  }
  TLQ_HIP(launch_recip(s, c_in, (bf16 && !act) ? xmax : nullptr, inv, st));
  if (act) TLQ_HIP(launch_act_quant(X, n_tok, c_in, ldx, bf16, inv, 0, 1, p->act_bits, xh, sig, nullptr, st));
  QuantArgs q{};
  q.W = W; q.c_out = c_out; q.c_in = c_in; q.ldw = ldw; q.bf16 = bf16;
  q.bits = p->bits; q.group = p->group; q.symmetric = p->symmetric;
  q.s_table = s; q.inv_table = act ? nullptr : inv; q.n_cand = 1; q.what = what; q.what_cand_stride = 0;
  q.what_f16 = true;
  TLQ_HIP(launch_fake_quant(q, st));
  GemmArgs g{};
  g.X = xh ? (const void*)xh : X; g.n_tok = n_tok; g.c_in = c_in; g.ldx = xh ? c_in : ldx;
  g.tok_scale = sig;
  g.Wh = what; g.c_out = c_out; g.ldw = c_in; g.w_cand_stride = 0; g.n_cand = 1; g.bf16 = false;
  g.Yout = X_next; g.ldo = ld_next; g.yout_dtype = p->x_dtype;
  g.wide_patch = true;   // one candidate: 8 weight panels stay per patch row, 4 token panels change (+1 .. +4 % measured)
  return hip_status(launch_gemm_store(g, st));
}

tlq_status tlq_apply_best(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                          const void* W, int64_t c_out, int64_t ldw, const float* s,
                          const tlq_params* p, void* X_next, int64_t ld_next, void* workspace,
                          size_t workspace_bytes, void* stream) {
  return apply_best_impl(X, n_tok, c_in, ldx, W, c_out, ldw, s, p, X_next, ld_next, workspace, workspace_bytes,
                         stream, nullptr);
}

tlq_status tlq_apply_best_prepared(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                                   const void* W, int64_t c_out, int64_t ldw, const float* s,
                                   const tlq_params* p, void* X_next, int64_t ld_next, void* workspace,
                                   size_t workspace_bytes, void* stream, const void* prepared) {
  return apply_best_impl(X, n_tok, c_in, ldx, W, c_out, ldw, s, p, X_next, ld_next, workspace, workspace_bytes,
                         stream, prepared);
}

// ------------------------------------------------------------ chain glue
tlq_status tlq_rmsnorm_mul(const void* Z, int64_t n_tok, int64_t c, int64_t ldz, const void* Zb,
                           int64_t ldzb, const float* m_a, const float* m_b, int32_t period,
                           int32_t split, const tlq_params* p, void* X_out, int64_t ld_out,
                           void* stream) {
  if (!Z || !X_out) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (!dims_ok(n_tok, c, ldz) || ld_out < c || (Zb && ldzb < c)) return TLQ_ERR_SHAPE;
  if (period < 0 || split < 0 || (period > 0 && split > period) || (period > 0 && (!m_a || !m_b)))
    return TLQ_ERR_SHAPE;
  if (!aligned(Z, 2) || !aligned(X_out, 2)) return TLQ_ERR_ALIGN;
  return hip_status(launch_rmsnorm_mul(Z, ldz, Zb, ldzb, n_tok, c, p->x_dtype == TLQ_BF16, m_a, m_b,
                                       period, split, X_out, ld_out, (hipStream_t)stream));
}

// ------------------------------------------------------------ decoder-block glue
tlq_status tlq_causal_attention(const void* Q, int64_t ldq, const void* K, int64_t ldk, const void* V,
                                int64_t ldv, int64_t n_tok, int32_t n_heads, int32_t head_dim,
                                int32_t seq_len, const tlq_params* p, void* Out, int64_t ldo,
                                void* stream) {
  if (!Q || !K || !V || !Out) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (head_dim != 128) return TLQ_ERR_UNSUPPORTED;
  if (n_tok <= 0 || n_heads <= 0 || n_heads > 65535 || seq_len <= 0 || seq_len > (1 << 24) ||
      (n_tok % seq_len) != 0 || n_tok / seq_len > 65535 || n_tok >= (1LL << 31))
    return TLQ_ERR_SHAPE;
  const int64_t width = (int64_t)n_heads * 128;
  if (ldq < width || ldk < width || ldv < width || ldo < width) return TLQ_ERR_SHAPE;
  if (!mat16_aligned(Q, ldq) || !mat16_aligned(K, ldk) || !mat16_aligned(V, ldv) || !mat16_aligned(Out, ldo))
    return TLQ_ERR_ALIGN;
  return hip_status(launch_causal_attention(Q, ldq, K, ldk, V, ldv, n_tok, n_heads, seq_len,
                                            p->x_dtype == TLQ_BF16, Out, ldo, (hipStream_t)stream));
}

static tlq_status pairwise(int mode, const void* A, int64_t lda, const void* B, int64_t ldb, int64_t n_tok,
                           int64_t c, const tlq_params* p, void* Out, int64_t ldo, void* stream) {
  if (!A || !B || !Out) return TLQ_ERR_NULL;
  TLQ_TRY(check_params(p));
  if (!dims_ok(n_tok, c, lda) || ldb < c || ldo < c || (c % 8) != 0) return TLQ_ERR_SHAPE;
  if (!mat16_aligned(A, lda) || !mat16_aligned(B, ldb) || !mat16_aligned(Out, ldo)) return TLQ_ERR_ALIGN;
  return hip_status(launch_pairwise(mode, A, lda, B, ldb, n_tok, c, p->x_dtype == TLQ_BF16, Out, ldo,
                                    (hipStream_t)stream));
}
tlq_status tlq_silu_mul(const void* G, int64_t ldg, const void* U, int64_t ldu, int64_t n_tok, int64_t c,
                        const tlq_params* p, void* Out, int64_t ldo, void* stream) {
  return pairwise(0, G, ldg, U, ldu, n_tok, c, p, Out, ldo, stream);
}
tlq_status tlq_residual_add(const void* H, int64_t ldh, const void* Z, int64_t ldz, int64_t n_tok,
                            int64_t c, const tlq_params* p, void* Out, int64_t ldo, void* stream) {
  return pairwise(1, H, ldh, Z, ldz, n_tok, c, p, Out, ldo, stream);
}

}  // extern "C"
