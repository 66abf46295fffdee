// Internal declarations shared by the libtlq translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "tlq.h"

namespace tlq {

constexpr float kXstatFloor = 6.103515625e-05f;  // 2^-14
constexpr float kRangeFloor = 1e-5f;

// 16-bit element types as raw bit patterns with exact widening to float.
struct F16 {
  using raw = _Float16;
  static __device__ __forceinline__ float to_float(uint16_t b) {
    return (float)__builtin_bit_cast(_Float16, b);
  }
  static __device__ __forceinline__ uint16_t from_float(float f) {
    return __builtin_bit_cast(uint16_t, (_Float16)f);  // round-to-nearest-even
  }
};
struct BF16 {
  using raw = __bf16;
  static __device__ __forceinline__ float to_float(uint16_t b) {
    return __builtin_bit_cast(float, (uint32_t)b << 16);
  }
  static __device__ __forceinline__ uint16_t from_float(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);  // round-to-nearest-even
    return (uint16_t)(u >> 16);
  }
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- profiling hooks (profile.cpp) ----------------------------------------
struct ProfScope {
  ProfScope(const char* name, hipStream_t stream, double work);
  ~ProfScope();
  int slot;
  hipStream_t stream;
  unsigned generation;
};

// ---- kernel launchers (each enqueues on `stream`, returns hipGetLastError) --
// S0: column mean/max of |X|; partial: double [n_chunks, c_in]
int xstat_chunks(int64_t n_tok);
// pos_mask (optional): only rows r with pos_mask[r % period] != 0 take part
hipError_t launch_xstat(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx, bool bf16,
                        int kind, double* partial, float* x_stat, hipStream_t stream,
                        const uint8_t* pos_mask = nullptr, int64_t period = 1);
// gradient-guided token selection (select.hip)
hipError_t launch_token_importance(const void* G, int64_t n_samples, int64_t n_pos, int64_t c, int64_t ldg,
                                   bool bf16, bool l2, double* row_norm, double* sum_n, hipStream_t stream);
hipError_t launch_topk_mask(const double* sum_n, int64_t n_pos, int64_t k, uint8_t* mask, hipStream_t stream);
// S1
// inv_table (optional) = 2^shift / s, where shift comes from `xmax_bits` (see launch_xprep) or is 0
hipError_t launch_scale_table(const float* x_stat, int64_t c_in, const float* alpha, int n_alpha,
                              float* s_table, float* inv_table, const uint32_t* xmax_bits,
                              hipStream_t stream);
// inv[c] = 2^shift / s[c]
hipError_t launch_recip(const float* s, int64_t c_in, const uint32_t* xmax_bits, float* inv,
                        hipStream_t stream);

// bf16 activations re-expressed in fp16.  A bf16 value has 8 significant bits, so
// X * 2^-shift is exact in fp16 once shift keeps the largest magnitude below 2^15
// (values more than 2^32 below that maximum lose low bits - far below anything the
// loss can see).  xmax_bits receives the bit pattern of max|X|; every consumer derives
// the same shift from it.  The folded weights carry the factor 2^shift, so the
// contraction is unchanged while its computed operand is rounded to 11 instead of 8
// significant bits.
hipError_t launch_xprep(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx, uint32_t* xmax_bits,
                        void* Xh, hipStream_t stream);
__host__ __device__ inline int shift_from_bf16_bits(uint32_t bits) {
  const int k = (int)((bits >> 7) & 0xffu) - 141;  // |x| < 2^(e-126); want < 2^15
  return k < 0 ? 0 : (k > 24 ? 24 : k);
}

// S2.  Quantises W*diag(s_k) for n_cand candidates (s_table row stride c_in).
// what:  folded operand deq/s as 16-bit [n_cand, c_out, c_in] (row stride c_in) or NULL
// codes/zp/delta/wdq: single-candidate auxiliary outputs or NULL
struct QuantArgs {
  const void* W; int64_t c_out, c_in, ldw; bool bf16;
  int bits, group, symmetric;
  const float* s_table;   // [n_cand, c_in] or NULL (ones)
  const float* inv_table; // [n_cand, c_in] or NULL (ones); used only for `what`
  int n_cand;
  void* what; int64_t what_cand_stride;  // elements between candidates
  bool what_f16;          // round `what` to fp16 even when W is bf16
  uint8_t* codes; uint8_t* zp; float* delta; void* wdq; int64_t ld_dq;
  // difference form: `what` receives deq*inv - W*2^shift (shift from xmax_bits, 0 when NULL)
  bool diff; const uint32_t* xmax_bits;
  const float* col_scale;   // [c_in] factor applied to `what` after everything else, or NULL
};
hipError_t launch_fake_quant(const QuantArgs& a, hipStream_t stream);

// Q_a: per-token symmetric activation fake-quant of X * diag(inv_k) for candidates k0 .. k0+nb-1.
// inv_table: [.., c_in] rows (row k used for candidate k) or NULL (ones).
// codes: fp16 integers [nb, n_tok, c_in]; sigma: float [nb, n_tok] (already offset to k0);
// rsigma: optional scratch of the same shape for the reciprocal steps.
hipError_t launch_act_quant(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx, bool bf16,
                            const float* inv_table, int k0, int nb, int act_bits, void* codes,
                            float* sigma, float* rsigma, hipStream_t stream);

// Wout[o,c] = round16(Win[o,c] * inv_s[c])
hipError_t launch_fold_scale(const void* Win, int64_t c_out, int64_t c_in, int64_t ldw, bool bf16,
                             const float* inv_s, const uint32_t* xmax_bits, bool out_f16, void* Wout,
                             hipStream_t stream);

// S3+S4 / plain GEMM with store epilogue.
struct GemmArgs {
  const void* X; int64_t n_tok, c_in, ldx;     // tokens  [n_tok, c_in]
  int64_t x_cand_stride;                        // elements between per-candidate token matrices (0 = shared)
  const float* tok_scale;                       // [n_cand, n_tok] factor on the accumulators or NULL
  const void* Wh; int64_t c_out, ldw;           // operand [n_cand, c_out, c_in]
  int64_t w_cand_stride; int n_cand; bool bf16;
  // loss epilogue
  const void* Yref; int64_t ldy; int yref_dtype; const float* token_w;
  int64_t y_cand_stride;   // launch_gemm_dot: elements between per-candidate Y matrices
  bool tri;                // launch_gemm_store of a symmetric product (X == Wh): tiles with tile row <= tile column only
  bool cand_outer;         // walk the candidates one after the other instead of inside every patch row
  bool wide_patch;         // L2 patches of 8 x 4 tiles (output rows x tokens) instead of 4 x 8
  bool sym_k;              // launch_gemm_dot: Wh is symmetric [c_in, c_in] and Y == X (a quadratic form)
  int64_t o_cand_stride;   // launch_gemm_store with n_cand > 1: elements between per-candidate outputs
  float* partial;          // [n_cand, tiles_o, tiles_t] float
  float* tok_partial;      // [tiles_o, n_tok] float or NULL (single candidate only)
  // store epilogue (n_cand == 1): Y[t,o]
  void* Yout; int64_t ldo; int yout_dtype;
};
void gemm_tile_counts(int64_t n_tok, int64_t c_out, int64_t* tiles_o, int64_t* tiles_t);
int64_t tile_map_defects(int64_t n_tok, int64_t c_in, int64_t c_out, int n_cand, int64_t* blocks_out);
hipError_t launch_gemm_loss(const GemmArgs& a, hipStream_t stream);
hipError_t launch_gemm_store(const GemmArgs& a, hipStream_t stream);
// partial[k, tile] = sum over the tile of (X_k Wh^T)[t,o] * Y_k[t,o]  (no token weights)
hipError_t launch_gemm_dot(const GemmArgs& a, hipStream_t stream);
// true when that launch uses the symmetry (sym_k: about half the flops, same partial sums)
bool gemm_dot_symmetric(const GemmArgs& a);

// Second-moment form (gram.hip).  out[c, t] = fp16(X[t,c] * sqrt(w_t / max w)) as [c_in, kp] with zero
// columns for n_tok <= t < kp; *wmax receives max_t w_t.
hipError_t launch_gram_operand(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx, bool bf16,
                               const float* token_w, float* wmax, void* out, int64_t kp, hipStream_t stream);
// H: n_split float [c_in, c_in] partial products of that operand with itself (tiles with column
// tile <= row tile), split_stride elements apart; they are summed into the first.  Writes the
// balanced fp16 matrix C, the per-channel factors of the weight errors and the factor that turns
// d'^T C d' into the loss; e is scratch [c_in].
hipError_t launch_gram_finish(float* H, int64_t c_in, int n_split, int64_t split_stride, const float* wmax,
                              int* e, double* factor, float* col_scale, void* C, hipStream_t stream);

// D[t,o] = Y[t,o] - D[t,o] (D float, row stride ldd)
hipError_t launch_sub_from_y(const void* Y, int64_t ldy, int ydt, float* D, int64_t ldd, int64_t n_tok,
                             int64_t c_out, hipStream_t stream);

// S4 final combine + S5 selection.
// `factor` (optional): device double multiplied into every loss
hipError_t launch_finalize(const float* partial, int n_cand, int64_t tiles_per_cand, int64_t c_out,
                           const float* s_table, int64_t c_in, float* losses, int32_t* best_idx,
                           float* best_scales, hipStream_t stream, const double* factor = nullptr);
hipError_t launch_token_err_reduce(const float* tok_partial, int64_t tiles_o, int64_t n_tok,
                                   int64_t c_out, float* per_token_err, hipStream_t stream);


// chain glue (glue.hip)
hipError_t launch_rmsnorm_mul(const void* Z, int64_t ldz, const void* Zb, int64_t ldzb, int64_t n_tok,
                              int64_t c, bool bf16, const float* m_a, const float* m_b, int period,
                              int split, void* out, int64_t ldo, hipStream_t stream);

// decoder-block glue (block.hip): head width 128, rows in blocks of seq_len
hipError_t launch_causal_attention(const void* Q, int64_t ldq, const void* K, int64_t ldk, const void* V,
                                   int64_t ldv, int64_t n_tok, int n_heads, int seq_len, bool bf16, void* O,
                                   int64_t ldo, hipStream_t stream);
// mode 0: out = SiLU(A) * B; mode 1: out = A + B (c % 8 == 0; out may alias A or B)
hipError_t launch_pairwise(int mode, const void* A, int64_t lda, const void* B, int64_t ldb, int64_t n_tok,
                           int64_t c, bool bf16, void* out, int64_t ldo, hipStream_t stream);

}  // namespace tlq
