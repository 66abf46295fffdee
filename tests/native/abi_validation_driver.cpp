// Host-only driver for the sanitizer build of libtlq's argument-validation layer.
// Every call below must return before any GPU work could be enqueued (there is no GPU where
// this runs): it walks the error paths, the size queries and the host-side self test with
// AddressSanitizer and UndefinedBehaviorSanitizer watching the library's host code.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "tlq.h"

static int g_checks = 0, g_fail = 0;
#define EXPECT(expr, want)                                                                    \
  do {                                                                                        \
    const long long got_ = (long long)(expr);                                                 \
    ++g_checks;                                                                               \
    if (got_ != (long long)(want)) {                                                          \
      ++g_fail;                                                                               \
      std::printf("FAIL line %d: %s = %lld, want %lld\n", __LINE__, #expr, got_, (long long)(want)); \
    }                                                                                         \
  } while (0)

int main() {
  tlq_params p;
  std::memset(&p, 0, sizeof p);
  p.struct_size = sizeof p; p.bits = 4; p.group = 128; p.x_dtype = TLQ_F16; p.yref_dtype = TLQ_F16;
  void* A = (void*)0x10000;        // aligned, never dereferenced: validation fails first
  void* ODD = (void*)0x10004;
  float* F = (float*)A;
  int32_t* I = (int32_t*)A;

  for (int s = -1; s <= 8; ++s) EXPECT(tlq_status_string(s) != nullptr, 1);
  EXPECT(tlq_version(), TLQ_VERSION);

  // ---- parameter block
  tlq_params q = p;
  q.struct_size = 8;      EXPECT(tlq_x_stat(A, 8, 8, 8, &q, F, A, 1 << 20, nullptr), TLQ_ERR_UNSUPPORTED);
  q = p; q.bits = 9;      EXPECT(tlq_fake_quant(A, 8, 128, 128, nullptr, &q, nullptr, nullptr, nullptr, nullptr, 0, nullptr), TLQ_ERR_UNSUPPORTED);
  q = p; q.bits = 1;      EXPECT(tlq_fake_quant(A, 8, 128, 128, nullptr, &q, nullptr, nullptr, nullptr, nullptr, 0, nullptr), TLQ_ERR_UNSUPPORTED);
  q = p; q.group = 12;    EXPECT(tlq_fake_quant(A, 8, 128, 128, nullptr, &q, nullptr, nullptr, nullptr, nullptr, 0, nullptr), TLQ_ERR_UNSUPPORTED);
  q = p; q.group = -8;    EXPECT(tlq_fake_quant(A, 8, 128, 128, nullptr, &q, nullptr, nullptr, nullptr, nullptr, 0, nullptr), TLQ_ERR_UNSUPPORTED);
  q = p; q.symmetric = 2; EXPECT(tlq_fake_quant(A, 8, 128, 128, nullptr, &q, nullptr, nullptr, nullptr, nullptr, 0, nullptr), TLQ_ERR_UNSUPPORTED);
  q = p; q.act_bits = 1;  EXPECT(tlq_fake_quant(A, 8, 128, 128, nullptr, &q, nullptr, nullptr, nullptr, nullptr, 0, nullptr), TLQ_ERR_UNSUPPORTED);
  q = p; q.xstat_kind = 2; EXPECT(tlq_x_stat(A, 8, 8, 8, &q, F, A, 1 << 20, nullptr), TLQ_ERR_UNSUPPORTED);
  q = p; q.x_dtype = TLQ_F32; EXPECT(tlq_x_stat(A, 8, 8, 8, &q, F, A, 1 << 20, nullptr), TLQ_ERR_UNSUPPORTED);
  q = p; q.yref_dtype = 7; EXPECT(tlq_x_stat(A, 8, 8, 8, &q, F, A, 1 << 20, nullptr), TLQ_ERR_UNSUPPORTED);
  EXPECT(tlq_x_stat(A, 8, 8, 8, nullptr, F, A, 1 << 20, nullptr), TLQ_ERR_NULL);

  // ---- S0 and its no-allocation variant
  EXPECT(tlq_x_stat(nullptr, 8, 8, 8, &p, F, A, 1 << 20, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_x_stat(A, 0, 8, 8, &p, F, A, 1 << 20, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_x_stat(A, 8, 12, 16, &p, F, A, 1 << 20, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_x_stat(A, 8, 16, 8, &p, F, A, 1 << 20, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_x_stat(ODD, 8, 8, 8, &p, F, A, 1 << 20, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_x_stat(A, 8, 8, 12, &p, F, A, 1 << 20, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_x_stat(A, 1000, 512, 512, &p, F, A, 16, nullptr), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_x_stat(A, 1000, 512, 512, &p, F, nullptr, 1 << 30, nullptr), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_x_stat_workspace_bytes(0, 8), 0);
  EXPECT(tlq_x_stat_workspace_bytes(1000, 512), 8 * 512 * 8);
  EXPECT(tlq_x_stat_workspace_bytes((int64_t)1 << 30, 16384), (int64_t)128 * 16384 * 8);
  EXPECT(tlq_x_stat_static(nullptr, 8, 8, 8, &p, F, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_x_stat_static(A, 8, 8, 8, nullptr, F, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_x_stat_static(A, 8, TLQ_X_STAT_STATIC_MAX_C_IN + 8, TLQ_X_STAT_STATIC_MAX_C_IN + 8, &p, F, nullptr), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_x_stat_static(A, 8, 12, 16, &p, F, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_x_stat_static(ODD, 8, 8, 8, &p, F, nullptr), TLQ_ERR_ALIGN);

  // ---- selection helpers
  EXPECT(tlq_token_importance(nullptr, 2, 4, 8, 8, 0, &p, (double*)A, A, 1 << 20, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_token_importance(A, 2, 4, 8, 4, 0, &p, (double*)A, A, 1 << 20, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_token_importance(A, 2, 4, 8, 8, 3, &p, (double*)A, A, 1 << 20, nullptr), TLQ_ERR_UNSUPPORTED);
  EXPECT(tlq_token_importance(A, 2, 4, 8, 8, 0, &p, (double*)A, A, 8, nullptr), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_token_importance(A, (int64_t)1 << 20, (int64_t)1 << 20, 8, 8, 0, &p, (double*)A, A, 1 << 20, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_topk_mask(nullptr, 4, 2, (uint8_t*)A, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_topk_mask((double*)A, 4, 5, (uint8_t*)A, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_topk_mask((double*)A, 70000, 5, (uint8_t*)A, nullptr), TLQ_ERR_UNSUPPORTED);
  EXPECT(tlq_x_stat_masked(A, 8, 8, 8, nullptr, 4, &p, F, A, 1 << 20, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_x_stat_masked(A, 8, 8, 8, (uint8_t*)A, 0, &p, F, A, 1 << 20, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_x_stat_masked(A, 8, 8, 8, (uint8_t*)A, 9, &p, F, A, 1 << 20, nullptr), TLQ_ERR_SHAPE);

  // ---- S1, S2, Q_a
  EXPECT(tlq_scale_table(nullptr, 8, F, 2, F, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_scale_table(F, 0, F, 2, F, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_scale_table(F, 8, F, TLQ_MAX_ALPHA + 1, F, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_fake_quant(nullptr, 8, 128, 128, nullptr, &p, nullptr, nullptr, nullptr, nullptr, 0, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_fake_quant(A, 8, 192, 192, nullptr, &p, nullptr, nullptr, nullptr, nullptr, 0, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_fake_quant(A, 8, 128, 64, nullptr, &p, nullptr, nullptr, nullptr, nullptr, 0, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_fake_quant(A, 8, 128, 128, nullptr, &p, nullptr, nullptr, nullptr, A, 64, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_fake_quant(A, 8, 128, 128, (float*)ODD, &p, nullptr, nullptr, nullptr, nullptr, 0, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_fake_quant(A, 8, 128, 128, nullptr, &p, (uint8_t*)ODD, nullptr, nullptr, nullptr, 0, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_fake_quant(A, (int64_t)1 << 31, 128, 128, nullptr, &p, nullptr, nullptr, nullptr, nullptr, 0, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_act_fake_quant(A, 8, 8, 8, nullptr, &p, A, F, nullptr), TLQ_ERR_UNSUPPORTED);   // act_bits = 0
  q = p; q.act_bits = 8;
  EXPECT(tlq_act_fake_quant(A, 8, 8, 8, nullptr, &q, nullptr, F, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_act_fake_quant(A, 8, 12, 16, nullptr, &q, A, F, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_act_fake_quant(A, 8, 8, 8, nullptr, &q, ODD, F, nullptr), TLQ_ERR_ALIGN);

  // ---- S3 + S4
  EXPECT(tlq_weighted_layer_err(A, 8, 128, 128, A, 8, 128, nullptr, nullptr, 8, F, &p, F, nullptr, A, 1 << 30, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_weighted_layer_err(A, 8, 128, 128, A, 8, 64, nullptr, A, 8, F, &p, F, nullptr, A, 1 << 30, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_weighted_layer_err(A, 8, 124, 128, A, 8, 128, nullptr, A, 8, F, &p, F, nullptr, A, 1 << 30, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_weighted_layer_err(A, 8, 128, 128, A, 8, 128, nullptr, A, 12, F, &p, F, nullptr, A, 1 << 30, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_weighted_layer_err(A, 8, 128, 128, A, 8, 128, nullptr, A, 8, F, &p, F, nullptr, A, 64, nullptr), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_weighted_layer_err(A, 8, 128, 128, A, 8, 128, nullptr, A, 8, F, &p, F, nullptr, ODD, 1 << 30, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_weighted_layer_err_workspace_bytes(0, 128, 8, &p), 0);
  EXPECT(tlq_weighted_layer_err_workspace_bytes(8, 128, 8, nullptr), 0);
  EXPECT(tlq_weighted_layer_err_workspace_bytes(153600, 5120, 13824, &p) > (size_t)13824 * 5120 * 2, 1);

  // ---- the search and its prepared variant
  const size_t ws = tlq_scale_search_workspace_bytes(256, 512, 512, 20, &p);
  EXPECT(ws > (size_t)20 * 512 * 512 * 2, 1);
  EXPECT(tlq_scale_search_workspace_bytes(256, 512, 512, 0, &p), 0);
  EXPECT(tlq_scale_search_workspace_bytes(256, 512, 512, TLQ_MAX_ALPHA + 1, &p), 0);
  EXPECT(tlq_scale_search_workspace_bytes(153600, 13824, 5120, 20, &p) > (size_t)20 * 13824 * 5120 * 2, 1);
#define SEARCH(X, n, ci, ldx, W, co, ldw, Y, ldy, w, al, na, par, best, idx, ls, wsp, wsb) \
  tlq_scale_search(X, n, ci, ldx, W, co, ldw, Y, ldy, w, al, na, par, nullptr, best, idx, ls, nullptr, wsp, wsb, nullptr)
  EXPECT(SEARCH(nullptr, 256, 512, 512, A, 512, 512, A, 512, F, F, 20, &p, F, I, F, A, (size_t)1 << 40), TLQ_ERR_NULL);
  EXPECT(SEARCH(A, 256, 512, 512, A, 512, 512, A, 512, F, F, 20, &p, F, I, nullptr, A, (size_t)1 << 40), TLQ_ERR_NULL);
  EXPECT(SEARCH(A, 0, 512, 512, A, 512, 512, A, 512, F, F, 20, &p, F, I, F, A, (size_t)1 << 40), TLQ_ERR_SHAPE);
  EXPECT(SEARCH(A, 256, 512, 256, A, 512, 512, A, 512, F, F, 20, &p, F, I, F, A, (size_t)1 << 40), TLQ_ERR_SHAPE);
  EXPECT(SEARCH(A, 256, 520, 520, A, 512, 520, A, 512, F, F, 20, &p, F, I, F, A, (size_t)1 << 40), TLQ_ERR_SHAPE);
  EXPECT(SEARCH(A, 256, 512, 512, A, 512, 512, A, 512, F, F, 0, &p, F, I, F, A, (size_t)1 << 40), TLQ_ERR_SHAPE);
  EXPECT(SEARCH(A, 256, 512, 512, A, 512, 512, A, 512, F, F, TLQ_MAX_ALPHA + 1, &p, F, I, F, A, (size_t)1 << 40), TLQ_ERR_SHAPE);
  EXPECT(SEARCH(ODD, 256, 512, 512, A, 512, 512, A, 512, F, F, 20, &p, F, I, F, A, (size_t)1 << 40), TLQ_ERR_ALIGN);
  EXPECT(SEARCH(A, 256, 512, 512, A, 512, 512, A, 516, F, F, 20, &p, F, I, F, A, (size_t)1 << 40), TLQ_ERR_ALIGN);
  EXPECT(SEARCH(A, 256, 512, 512, A, 512, 512, A, 512, F, F, 20, &p, F, I, F, A, ws - 1), TLQ_ERR_WORKSPACE);
  EXPECT(SEARCH(A, 256, 512, 512, A, 512, 512, A, 512, F, F, 20, &p, F, I, F, nullptr, ws), TLQ_ERR_WORKSPACE);
  EXPECT(SEARCH(A, 256, 512, 512, A, 512, 512, A, 512, F, F, 20, &p, F, I, F, ODD, ws), TLQ_ERR_ALIGN);
  EXPECT(tlq_scale_search_prepared(A, 256, 512, 512, A, 512, 512, A, 512, F, F, 20, &p, nullptr, F, I, F, nullptr, A, ws - 1, nullptr, A), TLQ_ERR_WORKSPACE);
  q = p; q.x_dtype = TLQ_BF16; q.yref_dtype = TLQ_BF16;
  EXPECT(tlq_prepared_tokens_bytes(256, 512, &p), 0);
  EXPECT(tlq_prepared_tokens_bytes(256, 512, &q), 256 + 256 * 512 * 2);
  EXPECT(tlq_prepared_tokens_bytes(0, 512, &q), 0);
  EXPECT(tlq_prepare_tokens(nullptr, 256, 512, 512, &q, A, 1 << 30, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_prepare_tokens(A, 256, 512, 512, &q, A, 1024, nullptr), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_prepare_tokens(A, 256, 512, 512, &q, nullptr, 1 << 30, nullptr), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_prepare_tokens(A, 256, 512, 512, &q, ODD, 1 << 30, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_prepare_tokens(A, 256, 512, 512, &p, nullptr, 0, nullptr), TLQ_OK);   // fp16: nothing to do, nothing launched
  const size_t wsq = tlq_scale_search_workspace_bytes(256, 512, 512, 20, &q);
  EXPECT(tlq_scale_search_prepared(A, 256, 512, 512, A, 512, 512, A, 512, F, F, 20, &q, nullptr, F, I, F, nullptr, A, wsq, nullptr, ODD), TLQ_ERR_ALIGN);

  // ---- second-moment form
  const size_t gb = tlq_token_gram_bytes(512);
  EXPECT(gb >= (size_t)512 * 512 * 2 + 512 * 4 + 256, 1);
  EXPECT(tlq_token_gram_bytes(0), 0);
  const size_t gws = tlq_token_gram_workspace_bytes(9000, 512);
  EXPECT(gws >= (size_t)9000 * 512 * 2 + (size_t)512 * 512 * 4, 1);
  EXPECT(tlq_token_gram_workspace_bytes(0, 512), 0);
  EXPECT(tlq_token_gram(nullptr, 9000, 512, 512, F, &p, A, gb, A, gws, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_token_gram(A, 9000, 512, 512, nullptr, &p, A, gb, A, gws, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_token_gram(A, 9000, 516, 520, F, &p, A, (size_t)1 << 30, A, (size_t)1 << 40, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_token_gram(A, 9000, 512, 256, F, &p, A, gb, A, gws, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_token_gram(ODD, 9000, 512, 512, F, &p, A, gb, A, gws, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_token_gram(A, 9000, 512, 512, F, &p, A, gb - 1, A, gws, nullptr), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_token_gram(A, 9000, 512, 512, F, &p, nullptr, gb, A, gws, nullptr), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_token_gram(A, 9000, 512, 512, F, &p, ODD, gb, A, gws, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_token_gram(A, 9000, 512, 512, F, &p, A, gb, A, gws - 1, nullptr), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_token_gram(A, 9000, 512, 512, F, &p, A, gb, ODD, gws, nullptr), TLQ_ERR_ALIGN);
  const size_t gss = tlq_scale_search_gram_workspace_bytes(512, 384, 20, &p);
  EXPECT(gss >= (size_t)20 * 384 * 512 * 2, 1);
  EXPECT(tlq_scale_search_gram_workspace_bytes(512, 384, 0, &p), 0);
  EXPECT(tlq_scale_search_gram_workspace_bytes(512, 384, 20, nullptr), 0);
  EXPECT(tlq_scale_search_gram(nullptr, 512, A, 384, 512, F, 20, &p, F, F, I, F, nullptr, A, gss, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_scale_search_gram(A, 512, A, 384, 512, F, 20, &p, nullptr, F, I, F, nullptr, A, gss, nullptr), TLQ_ERR_NULL);
  q = p; q.act_bits = 8;
  EXPECT(tlq_scale_search_gram(A, 512, A, 384, 512, F, 20, &q, F, F, I, F, nullptr, A, gss, nullptr), TLQ_ERR_UNSUPPORTED);
  EXPECT(tlq_scale_search_gram(A, 512, A, 384, 512, F, 0, &p, F, F, I, F, nullptr, A, gss, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_scale_search_gram(A, 520, A, 384, 520, F, 20, &p, F, F, I, F, nullptr, A, (size_t)1 << 40, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_scale_search_gram(A, 512, A, 384, 256, F, 20, &p, F, F, I, F, nullptr, A, gss, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_scale_search_gram(ODD, 512, A, 384, 512, F, 20, &p, F, F, I, F, nullptr, A, gss, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_scale_search_gram(A, 512, ODD, 384, 512, F, 20, &p, F, F, I, F, nullptr, A, gss, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_scale_search_gram(A, 512, A, 384, 512, F, 20, &p, F, F, I, F, nullptr, A, gss - 1, nullptr), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_scale_search_gram(A, 512, A, 384, 512, F, 20, &p, F, F, I, F, nullptr, ODD, gss, nullptr), TLQ_ERR_ALIGN);

  // ---- f_fp, S6, glue  // ---- f_fp, S6, glue
  EXPECT(tlq_ref_output(A, 8, 128, 128, nullptr, 8, 128, A, 8, &p, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_ref_output(A, 8, 128, 128, A, 8, 128, A, 4, &p, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_ref_output(A, 8, 128, 128, A, 8, 128, ODD, 8, &p, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_apply_best(A, 8, 128, 128, A, 8, 128, nullptr, &p, A, 8, A, 1 << 30, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_apply_best(A, 8, 192, 192, A, 8, 192, F, &p, A, 8, A, 1 << 30, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_apply_best(A, 8, 128, 128, A, 8, 128, (float*)ODD, &p, A, 8, A, 1 << 30, nullptr), TLQ_ERR_ALIGN);
  EXPECT(tlq_apply_best(A, 8, 128, 128, A, 8, 128, F, &p, A, 8, A, 16, nullptr), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_apply_best_prepared(A, 8, 128, 128, A, 8, 128, F, &p, A, 8, A, 16, nullptr, A), TLQ_ERR_WORKSPACE);
  EXPECT(tlq_apply_best_workspace_bytes(8, 128, 8, nullptr), 0);
  EXPECT(tlq_rmsnorm_mul(nullptr, 8, 8, 8, nullptr, 0, nullptr, nullptr, 0, 0, &p, A, 8, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_rmsnorm_mul(A, 8, 8, 8, nullptr, 0, nullptr, nullptr, 4, 5, &p, A, 8, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_rmsnorm_mul(A, 8, 8, 8, nullptr, 0, nullptr, nullptr, 4, 2, &p, A, 8, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_causal_attention(A, 128, A, 128, A, 128, 8, 1, 64, 4, &p, A, 128, nullptr), TLQ_ERR_UNSUPPORTED);
  EXPECT(tlq_causal_attention(A, 128, A, 128, A, 128, 9, 1, 128, 4, &p, A, 128, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_causal_attention(A, 64, A, 128, A, 128, 8, 1, 128, 4, &p, A, 128, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_causal_attention(nullptr, 128, A, 128, A, 128, 8, 1, 128, 4, &p, A, 128, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_silu_mul(A, 8, nullptr, 8, 8, 8, &p, A, 8, nullptr), TLQ_ERR_NULL);
  EXPECT(tlq_silu_mul(A, 8, A, 8, 8, 12, &p, A, 16, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_residual_add(A, 8, A, 8, 8, 8, &p, ODD, 8, nullptr), TLQ_ERR_ALIGN);

  // ---- host-side self test of the block -> tile map, and the timing bookkeeping
  int64_t blocks = 0;
  EXPECT(tlq_selftest_tile_map(10240, 4096, 11008, 20, &blocks), 0);
  EXPECT(blocks % 256, 0);
  EXPECT(tlq_selftest_tile_map(153600, 5120, 13824, 20, nullptr), 0);
  EXPECT(tlq_selftest_tile_map(777, 64, 1300, 3, &blocks), 0);
  EXPECT(tlq_selftest_tile_map(-1, 64, 64, 1, nullptr), -1);
  EXPECT(tlq_profile_enabled(), 0);
  EXPECT(tlq_profile_count(), 0);
  char name[8];
  int64_t launches; double ms, work;
  EXPECT(tlq_profile_get(0, name, sizeof name, &launches, &ms, &work), TLQ_ERR_SHAPE);
  EXPECT(tlq_profile_get(-1, nullptr, 0, nullptr, nullptr, nullptr), TLQ_ERR_SHAPE);
  EXPECT(tlq_profile_reset(), TLQ_OK);

  std::printf("%d checks, %d failed\n", g_checks, g_fail);
  return g_fail == 0 ? 0 : 1;
}
