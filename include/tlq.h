/*
 * tlq.h - C ABI of libtlq: the data-parallel hot path of TLQ's layer-wise
 * scale search on one AMD MI355X (gfx950).
 *
 * What the library computes (paper: "Rethinking Practical and Efficient
 * Quantization Calibration for Vision-Language Models"):
 *   for one linear layer with weights W [c_out, c_in] and calibration tokens
 *   X [n_tok, c_in], and for every candidate exponent alpha_k of a grid,
 *     s_k      = x_stat ^ alpha_k                        (Sec. 3.1.2, scale eq.)
 *     Wq_k     = Q_w(W * diag(s_k))                       (Sec. 3.2.1, f_q)
 *     Yq_k     = (X * diag(s_k)^-1) * Wq_k^T              (Sec. 2.2, smoothing eq.)
 *     L_k      = sum_t w_t * (1/c_out) * sum_o (Y_ref[t,o] - Yq_k[t,o])^2
 *                                                         (Sec. 3.2.1, objective)
 *   and returns k* = argmin_k L_k together with s_{k*}.  Q_w is round-to-
 *   nearest integer quantisation (Sec. 2.2) on a min/max grid per group of
 *   consecutive input channels; activations stay in 16-bit floating point.
 *
 * Conventions that hold for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The
 *     library never allocates, frees or keeps device memory; scratch comes
 *     from the caller's `workspace` (size from the matching *_workspace_bytes
 *     query; 256-byte aligned).  A workspace that is too small gives
 *     TLQ_ERR_WORKSPACE and nothing is launched.
 *   - `stream` is the caller's hipStream_t passed as void* (NULL = the null
 *     stream).  All work is enqueued on it in order; no entry point
 *     synchronises with the host or copies to the host.  Outputs are device
 *     resident and valid once the stream reaches the end of the call.
 *   - The return value reports argument validation and launch errors only.
 *     Validation (every status except TLQ_ERR_LAUNCH) happens before any HIP call:
 *     nothing was launched and nothing was written.  TLQ_ERR_LAUNCH means the HIP
 *     runtime refused a launch part-way through the call: kernels enqueued before it
 *     may still run and the outputs and the workspace must be treated as undefined.
 *     Faults inside a kernel surface at the caller's next synchronisation.
 *   - Matrices are row-major with a row stride (`ld*`) in ELEMENTS.  16-bit
 *     matrices need 16-byte aligned base pointers and strides that are
 *     multiples of 8; otherwise TLQ_ERR_ALIGN.  c_in must be a multiple of 8
 *     and of `group` (TLQ_ERR_SHAPE otherwise).
 *   - Calls on different streams may run concurrently if their workspaces and
 *     outputs are disjoint.  The library keeps no state between calls except (a) the
 *     optional per-kernel timing (tlq_profile_*: one process-wide table behind a mutex)
 *     and (b) the fixed scratch array of tlq_x_stat_static.
 *   - Float vectors that are read 16 bytes at a time (`s` of tlq_fake_quant and
 *     tlq_apply_best) must be 16-byte aligned; `group` must be 0 or a multiple of 8
 *     (TLQ_ERR_UNSUPPORTED otherwise); uint8 code matrices must be 8-byte aligned.
 *   - act_bits > 0 (Sec. 3.2.1 f_q with Q_a; quantiser of Sec. 2.2 per token row):
 *     xt = x * float(1/s); sigma_t = max(max_c |xt|, 1e-5) / (2^(n-1)-1);
 *     code = clip(rint(xt/sigma_t), -2^(n-1), 2^(n-1)-1); f_q = sigma_t * code . deq^T.
 *     float arithmetic, round half to even.  Applies to tlq_scale_search,
 *     tlq_weighted_layer_err and tlq_apply_best.
 *   - x_dtype = BF16: inputs and 16-bit outputs are bf16.  Operands the library
 *     computes itself (the folded weights deq/s) are kept in fp16, and the tokens
 *     are re-expressed in fp16 in the workspace (exact for bf16 values after a
 *     power-of-two prescale), so bf16 inputs get the same loss accuracy as fp16.
 */
#ifndef TLQ_H
#define TLQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TLQ_VERSION 100 /* 0.1.0 */
#define TLQ_MAX_ALPHA 64 /* largest alpha grid one call accepts */

typedef enum {
  TLQ_OK = 0,
  TLQ_ERR_NULL = 1,        /* a required pointer is NULL */
  TLQ_ERR_SHAPE = 2,       /* a size is non-positive or inconsistent */
  TLQ_ERR_UNSUPPORTED = 3, /* a parameter value this build does not implement */
  TLQ_ERR_WORKSPACE = 4,   /* workspace missing or smaller than the query says */
  TLQ_ERR_ALIGN = 5,       /* pointer or stride alignment */
  TLQ_ERR_LAUNCH = 6       /* the HIP runtime rejected a launch */
} tlq_status;

typedef enum { TLQ_F16 = 0, TLQ_BF16 = 1, TLQ_F32 = 2 } tlq_dtype;

/* Plain-old-data parameter block, passed by const pointer. */
typedef struct tlq_params {
  uint32_t struct_size; /* = sizeof(tlq_params); anything else: TLQ_ERR_UNSUPPORTED */
  int32_t bits;         /* weight bits, 2..8 */
  int32_t group;        /* input channels per quantisation group; 0 = whole row */
  int32_t symmetric;    /* 0 = asymmetric min/max grid, 1 = symmetric max|.| grid */
  int32_t act_bits;     /* 0 = activations not quantised; 2..8 = per-token symmetric Q_a */
  int32_t xstat_kind;   /* 0 = mean |x| over tokens, 1 = max |x| over tokens */
  int32_t x_dtype;      /* tlq_dtype of X and of W and of the MFMA operands: F16 or BF16 */
  int32_t yref_dtype;   /* tlq_dtype of Y_ref (and of tlq_ref_output's result) */
} tlq_params;

const char* tlq_status_string(int status);
int tlq_version(void);

/* ---- S0: per-channel activation statistic (Sec. 3.1.2, x_stat; mean form of
 * the ablation table, or max).  x_stat[c] = (1/n_tok) sum_t |X[t,c]| rounded
 * once to float (sum and division in double), or max_t |X[t,c]|.
 * x_stat: out, float [c_in]. */
size_t tlq_x_stat_workspace_bytes(int64_t n_tok, int64_t c_in);
tlq_status tlq_x_stat(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                      const tlq_params* p, float* x_stat,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ---- tlq_x_stat for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same
 * result bit for bit as tlq_x_stat, but the partial sums live in a fixed 16 MiB device
 * array inside the library (one copy per GPU, held until the process ends) instead of a
 * caller workspace.  The call allocates and frees nothing, on the device or through any
 * library.  Limits: c_in <= TLQ_X_STAT_STATIC_MAX_C_IN (TLQ_ERR_WORKSPACE beyond it);
 * per-kernel timing must be off (TLQ_ERR_UNSUPPORTED while tlq_profile_enable(1) is in
 * force, because timing creates HIP events).  The stream must belong to the device that is
 * current at the call.  All calls on one GPU share that GPU's array: calls that overlap in
 * time on one GPU (different streams or threads) race on it and give wrong results;
 * serialise them.  Nothing in the array needs to survive between calls. */
#define TLQ_X_STAT_STATIC_MAX_C_IN 16384
tlq_status tlq_x_stat_static(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                             const tlq_params* p, float* x_stat, void* stream);

/* ---- gradient-guided token selection (Sec. 3.1.2).  G holds per-sample gradients with
 * respect to the layer input, sample major: [n_samples * n_pos, c] x_dtype.
 *   tlq_token_importance: sum_n[n] = sum_b ||g_{b,n}||, n < n_pos (gradient-statistic eq.);
 *     the norm is mean_c |g| (l2 = 0, the text's description) or the Euclidean norm (l2 = 1);
 *     double accumulation in a fixed order; sum_n: out double [n_pos].
 *   tlq_topk_mask: I = Top_k({sum_n}) (selection eq.; the paper keeps k = n_pos/2); ties go
 *     to the lower position; mask: out uint8 [n_pos], 1 = selected.  n_pos <= 65536.
 *   tlq_x_stat_masked: x_stat[c] = max over rows t with pos_mask[t mod period] != 0 of
 *     |X[t,c]| (x_stat eq.; X stacks samples of `period` positions); workspace as tlq_x_stat.
 * The result feeds tlq_scale_search through x_stat_in. */
size_t tlq_token_importance_workspace_bytes(int64_t n_samples, int64_t n_pos);
tlq_status tlq_token_importance(const void* G, int64_t n_samples, int64_t n_pos, int64_t c,
                                int64_t ldg, int32_t l2, const tlq_params* p, double* sum_n,
                                void* workspace, size_t workspace_bytes, void* stream);
tlq_status tlq_topk_mask(const double* sum_n, int64_t n_pos, int64_t k, uint8_t* mask, void* stream);
tlq_status tlq_x_stat_masked(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                             const uint8_t* pos_mask, int64_t period, const tlq_params* p,
                             float* x_stat, void* workspace, size_t workspace_bytes, void* stream);

/* ---- S1: candidate scales (Sec. 3.1.2 scale eq.; Sec. 3.2.1 per-layer form).
 * s_table[k,c] = float( pow( double(max(x_stat[c], 2^-14)), double(alpha[k]) ) ).
 * x_stat: in, float [c_in]; alpha_grid: in, float [n_alpha];
 * s_table: out, float [n_alpha, c_in]. */
tlq_status tlq_scale_table(const float* x_stat, int64_t c_in, const float* alpha_grid,
                           int32_t n_alpha, float* s_table, void* stream);

/* ---- S2: fake quantisation of W * diag(s) (Sec. 2.2 quantiser in min/max
 * form; Sec. 3.2.1 Q_w(W * scale)).  All grid arithmetic is float, one
 * rounding per operation, round-half-to-even:
 *   ws = W*s; rng = max(max_g ws - min_g ws, 1e-5); delta = rng/(2^bits-1);
 *   zp = clip(rint(-min/delta), 0, 2^bits-1);
 *   q  = clip(rint(ws/delta) + zp, 0, 2^bits-1);  deq = (q - zp)*delta.
 * (symmetric=1: delta = max(max_g|ws|,1e-5)/(2^(bits-1)-1), q = clip(rint(ws/
 * delta), -2^(bits-1), 2^(bits-1)-1), stored codes are q + 2^(bits-1), zp =
 * 2^(bits-1).)
 * W: in [c_out, c_in] x_dtype; s: in float [c_in] or NULL (= ones).
 * Outputs, each may be NULL (skipped): codes uint8 [c_out, c_in] (dense),
 * zp uint8 [c_out, G], delta float [c_out, G], G = c_in/group;
 * Wdq [c_out, c_in] x_dtype with row stride ld_dq = deq rounded to x_dtype. */
tlq_status tlq_fake_quant(const void* W, int64_t c_out, int64_t c_in, int64_t ldw,
                          const float* s, const tlq_params* p,
                          uint8_t* codes, uint8_t* zp, float* delta,
                          void* Wdq, int64_t ld_dq, void* stream);

/* ---- Q_a alone (Sec. 3.2.1 Q_a(x/scale); quantiser of Sec. 2.2 per token row; formula in
 * the conventions above).  Needs act_bits > 0.  inv_s: float [c_in] or NULL (ones).
 * codes: out [n_tok, c_in] dense, the integer codes stored as fp16 numbers (exact);
 * sigma: out float [n_tok]. */
tlq_status tlq_act_fake_quant(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                              const float* inv_s, const tlq_params* p, void* codes, float* sigma,
                              void* stream);

/* ---- S3+S4 for one given dequantised weight matrix (Sec. 3.2.1 objective
 * with f_q = (X*inv_s) Wdq^T):
 *   err[t] = (1/c_out) sum_o (Y_ref[t,o] - sum_c X[t,c]*inv_s[c]*Wdq[o,c])^2
 *   loss   = sum_t token_w[t] * err[t]
 * X [n_tok,c_in], Wdq [c_out,c_in]: x_dtype; inv_s: float [c_in] or NULL (ones);
 * Y_ref [n_tok,c_out] yref_dtype; token_w float [n_tok] (used as given).
 * loss: out float [1]; per_token_err: out float [n_tok] or NULL.
 * The operand that enters the matrix cores is round16(Wdq * inv_s); on problems with only a
 * handful of outputs that rounding can show in the loss beyond 1e-3 (tlq_scale_search, which
 * also sees W, avoids it there). */
size_t tlq_weighted_layer_err_workspace_bytes(int64_t n_tok, int64_t c_in, int64_t c_out,
                                              const tlq_params* p);
tlq_status tlq_weighted_layer_err(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                                  const void* Wdq, int64_t c_out, int64_t ldw,
                                  const float* inv_s,
                                  const void* Y_ref, int64_t ldy, const float* token_w,
                                  const tlq_params* p, float* loss, float* per_token_err,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* ---- S0..S5: the search (Sec. 3.2.1: r* = argmin_r E||f_fp(x) - f_q(x; x_stat^r)||^2).
 * x_stat_in: float [c_in] or NULL (then computed from X per xstat_kind).
 * alpha_grid: float [n_alpha], 1 <= n_alpha <= TLQ_MAX_ALPHA.
 * Outputs: best_scales float [c_in] (= s_table[best_idx]); best_idx int32 [1]
 * (first minimum; -1 if no candidate has a finite loss); losses float
 * [n_alpha] (+inf where not finite); s_table_out float [n_alpha, c_in] or NULL.
 * Arithmetic: 16-bit matrix-core operands, float accumulation.  Without
 * activation quantisation the operand is the folded weight
 * round16(deq_k / s_k); from 6 weight bits on, and for problems smaller than
 * 256 x 256 outputs, it is the difference round16(deq_k / s_k - W) and the
 * residual is formed against Y_ref - X W^T kept in float (one more
 * contraction and n_tok x c_out floats of workspace), because there the
 * rounding of the folded weight itself would show in the loss. */
size_t tlq_scale_search_workspace_bytes(int64_t n_tok, int64_t c_in, int64_t c_out,
                                        int32_t n_alpha, const tlq_params* p);
tlq_status tlq_scale_search(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                            const void* W, int64_t c_out, int64_t ldw,
                            const void* Y_ref, int64_t ldy, const float* token_w,
                            const float* alpha_grid, int32_t n_alpha, const tlq_params* p,
                            const float* x_stat_in,
                            float* best_scales, int32_t* best_idx, float* losses,
                            float* s_table_out,
                            void* workspace, size_t workspace_bytes, void* stream);

/* ---- tokens prepared once for several calls on the same X (Sec. 3.2.1: q/k/v and gate/up
 * are searched, and then propagated, on one exposed input).  With x_dtype = BF16 and act_bits = 0
 * every search and every propagation first re-expresses X in fp16 (see the conventions above);
 * tlq_prepare_tokens does that once into a caller buffer of tlq_prepared_tokens_bytes bytes
 * (256-byte aligned; 0 = these parameters need no preparation and `prepared` may be NULL), and
 * the *_prepared variants below take that buffer instead of repeating the conversion.  They
 * are otherwise identical to tlq_scale_search / tlq_apply_best (same arguments, same results
 * bit for bit); prepared = NULL makes them the plain calls.  The buffer must have been
 * filled from the same X, n_tok, c_in and parameters on the same stream order. */
size_t tlq_prepared_tokens_bytes(int64_t n_tok, int64_t c_in, const tlq_params* p);
tlq_status tlq_prepare_tokens(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                              const tlq_params* p, void* prepared, size_t prepared_bytes,
                              void* stream);
tlq_status tlq_scale_search_prepared(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                                     const void* W, int64_t c_out, int64_t ldw,
                                     const void* Y_ref, int64_t ldy, const float* token_w,
                                     const float* alpha_grid, int32_t n_alpha, const tlq_params* p,
                                     const float* x_stat_in,
                                     float* best_scales, int32_t* best_idx, float* losses,
                                     float* s_table_out,
                                     void* workspace, size_t workspace_bytes, void* stream,
                                     const void* prepared);
tlq_status tlq_apply_best_prepared(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                                   const void* W, int64_t c_out, int64_t ldw, const float* s,
                                   const tlq_params* p, void* X_next, int64_t ld_next,
                                   void* workspace, size_t workspace_bytes, void* stream,
                                   const void* prepared);

/* ---- the weight-only search in second-moment form (Sec. 3.2.1 objective with f_q linear in x,
 * i.e. act_bits == 0).  For f_fp(x) = x W^T and f_q(x) = x What_k^T the objective
 *   sum_t token_w[t] (1/c_out) ||f_fp(x_t) - f_q(x_t)||^2  =  (1/c_out) sum_o d_o^T G d_o,
 *   d_o = row o of W - What_k,   G = sum_t token_w[t] x_t x_t^T   [c_in, c_in],
 * so the tokens enter through G alone.  G does not depend on the candidate or on the linear:
 * linears that share an input (q/k/v, gate/up) share one G, and a candidate then costs
 * 2 c_out c_in^2 flops instead of 2 n_tok c_in c_out.  It pays when n_tok is well above c_in.
 * The target is the exact product x W^T (no rounded Y_ref enters), and no per-token error exists.
 *
 * tlq_token_gram writes a device-resident representation of G into `gram`
 * (tlq_token_gram_bytes(c_in) bytes, 256-byte aligned, caller-owned): a double `factor` at byte 0,
 * float col_scale[c_in] at byte 256, then (256-byte aligned) fp16 C[c_in, c_in], with
 *   G[i,j] = factor * col_scale[i] * col_scale[j] * C[i,j];
 * col_scale holds powers of two chosen so that |C| <= 2 whatever the spread of the channel
 * magnitudes.  Tokens must lie inside the fp16 range (|x| < 65504) - beyond it the losses come out
 * non-finite.  Workspace from the query.
 * tlq_scale_search_gram is tlq_scale_search with (X, Y_ref, token_w) replaced by `gram`; x_stat
 * [c_in] is required (tlq_x_stat of the same X).  act_bits != 0 -> TLQ_ERR_UNSUPPORTED.  Outputs,
 * non-finite rule and tie rule as for tlq_scale_search. */
size_t     tlq_token_gram_bytes(int64_t c_in);
size_t     tlq_token_gram_workspace_bytes(int64_t n_tok, int64_t c_in);
tlq_status tlq_token_gram(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                          const float* token_w /*[n_tok]*/, const tlq_params* p,
                          void* gram, size_t gram_bytes,
                          void* workspace, size_t workspace_bytes, void* stream);
size_t     tlq_scale_search_gram_workspace_bytes(int64_t c_in, int64_t c_out, int32_t n_alpha,
                                                 const tlq_params* p);
tlq_status tlq_scale_search_gram(const void* gram, int64_t c_in,
                                 const void* W, int64_t c_out, int64_t ldw,
                                 const float* alpha_grid, int32_t n_alpha, const tlq_params* p,
                                 const float* x_stat /*[c_in]*/,
                                 float* best_scales /*[c_in]*/, int32_t* best_idx /*[1]*/,
                                 float* losses /*[n_alpha]*/, float* s_table_out /*[n_alpha,c_in] or NULL*/,
                                 void* workspace, size_t workspace_bytes, void* stream);

/* ---- full-precision layer output (Sec. 3.2.1 f_fp without bias):
 * Y[t,o] = sum_c X[t,c] W[o,c], float accumulation, stored as yref_dtype. */
tlq_status tlq_ref_output(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                          const void* W, int64_t c_out, int64_t ldw,
                          void* Y, int64_t ldy, const tlq_params* p, void* stream);

/* ---- S6: quantisation-exposed propagation (Sec. 3.2.1 PassAct2):
 * X_next = f_q(X; s) = (X diag(s)^-1) Q_w(W diag(s))^T stored as x_dtype.
 * s: in float [c_in] (e.g. best_scales); X_next: out [n_tok, c_out]. */
size_t tlq_apply_best_workspace_bytes(int64_t n_tok, int64_t c_in, int64_t c_out,
                                      const tlq_params* p);
tlq_status tlq_apply_best(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                          const void* W, int64_t c_out, int64_t ldw, const float* s,
                          const tlq_params* p, void* X_next, int64_t ld_next,
                          void* workspace, size_t workspace_bytes, void* stream);

/* ---- glue of the synthetic sequential chain (the workload's construction, not the paper's method):
 * builds the exposed input of the next linear from the quantised output of the
 * previous one (Sec. 3.2.1 PassAct2 propagation).
 *   v = Z (or Z*Zb elementwise when Zb != NULL);
 *   X_out[t,c] = round16( v[t,c] / sqrt(mean_c v[t,:]^2 + 1e-6) * m(t)[c] ),
 *   m(t) = m_a if period == 0 or (t mod period) < split, else m_b; NULL = ones.
 * Z, Zb, X_out: [n_tok, c] x_dtype; m_a, m_b: float [c].  float arithmetic. */
tlq_status tlq_rmsnorm_mul(const void* Z, int64_t n_tok, int64_t c, int64_t ldz, const void* Zb,
                           int64_t ldzb, const float* m_a, const float* m_b, int32_t period,
                           int32_t split, const tlq_params* p, void* X_out, int64_t ld_out,
                           void* stream);

/* ---- decoder-block glue for sequential calibration of a stack (Sec. 3.2.1:
 * activations are propagated through the model between two searches; the block
 * itself is the workload's, not the paper's).  All matrices are 16-bit
 * (p->x_dtype) device pointers, 16-byte aligned, row strides in elements and
 * multiples of 8; nothing is allocated; work is enqueued on `stream`.
 *
 * tlq_causal_attention: Out[t, h*128 .. h*128+127] =
 *   sum_{j <= t, same sample} softmax_j(q_t . k_j / sqrt(128)) v_j  per head h.
 * Rows are grouped in consecutive blocks of seq_len (one calibration sample
 * each); n_tok must be a multiple of seq_len.  head_dim must be 128
 * (TLQ_ERR_UNSUPPORTED otherwise).  Q, K, V may be column slices of one matrix.
 * Scores and the softmax are float; probabilities are rounded to x_dtype before
 * the second product; Out is rounded to x_dtype. */
tlq_status tlq_causal_attention(const void* Q, int64_t ldq, const void* K, int64_t ldk, const void* V,
                                int64_t ldv, int64_t n_tok, int32_t n_heads, int32_t head_dim,
                                int32_t seq_len, const tlq_params* p, void* Out, int64_t ldo,
                                void* stream);
/* Out = G / (1 + exp(-G)) * U, elementwise in float, rounded to x_dtype; c % 8 == 0. */
tlq_status tlq_silu_mul(const void* G, int64_t ldg, const void* U, int64_t ldu, int64_t n_tok, int64_t c,
                        const tlq_params* p, void* Out, int64_t ldo, void* stream);
/* Out = H + Z, elementwise in float, rounded to x_dtype; Out may alias H or Z; c % 8 == 0. */
tlq_status tlq_residual_add(const void* H, int64_t ldh, const void* Z, int64_t ldz, int64_t n_tok,
                            int64_t c, const tlq_params* p, void* Out, int64_t ldo, void* stream);

/* ---- host-side self check (no GPU work, no device memory): walks the block -> tile map that
 * the contraction kernels (S3/S4, f_fp, S6) would use for this problem shape, in both of its
 * orders (candidates inside every patch row / candidate-outermost), and returns how many
 * (candidate, output tile) pairs are NOT produced exactly once - 0 for correct maps, -1 for an
 * invalid shape.  *blocks (may be NULL) receives the number of workgroups of the launch. */
int64_t tlq_selftest_tile_map(int64_t n_tok, int64_t c_in, int64_t c_out, int32_t n_cand,
                              int64_t* blocks);

/* ---- optional per-kernel timing (host-side bookkeeping only).
 * While enabled, every kernel the library launches is bracketed by HIP events
 * on the launch stream.  tlq_profile_collect waits for the recorded events
 * and folds them into per-kernel totals; tlq_profile_get reads entry i:
 * kernel name, number of launches, total milliseconds, and the total
 * algorithmic work (flops for the contraction kernels, bytes otherwise). */
tlq_status tlq_profile_enable(int on);
int tlq_profile_enabled(void);
tlq_status tlq_profile_reset(void);
tlq_status tlq_profile_collect(void);
int tlq_profile_count(void);
tlq_status tlq_profile_get(int i, char* name, size_t name_cap, int64_t* launches,
                           double* total_ms, double* total_work);

#ifdef __cplusplus
}
#endif
#endif /* TLQ_H */
