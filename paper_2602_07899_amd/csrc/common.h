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
};

// ---- kernel launchers (each enqueues on `stream`, returns hipGetLastError) --
// S0: column mean/max of |X|; partial: double [n_chunks, c_in]
int xstat_chunks(int64_t n_tok);
hipError_t launch_xstat(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx, bool bf16,
                        int kind, double* partial, float* x_stat, hipStream_t stream);
// S1
hipError_t launch_scale_table(const float* x_stat, int64_t c_in, const float* alpha, int n_alpha,
                              float* s_table, float* inv_table, hipStream_t stream);

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
  uint8_t* codes; uint8_t* zp; float* delta; void* wdq; int64_t ld_dq;
};
hipError_t launch_fake_quant(const QuantArgs& a, hipStream_t stream);

// Wout[o,c] = round16(Win[o,c] * inv_s[c])
hipError_t launch_fold_scale(const void* Win, int64_t c_out, int64_t c_in, int64_t ldw, bool bf16,
                             const float* inv_s, void* Wout, hipStream_t stream);

// S3+S4 / plain GEMM with store epilogue.
struct GemmArgs {
  const void* X; int64_t n_tok, c_in, ldx;     // tokens  [n_tok, c_in]
  const void* Wh; int64_t c_out, ldw;           // operand [n_cand, c_out, c_in]
  int64_t w_cand_stride; int n_cand; bool bf16;
  // loss epilogue
  const void* Yref; int64_t ldy; int yref_dtype; const float* token_w;
  float* partial;          // [n_cand, tiles_o, tiles_t] float
  float* tok_partial;      // [tiles_o, n_tok] float or NULL (single candidate only)
  // store epilogue (n_cand == 1): Y[t,o]
  void* Yout; int64_t ldo; int yout_dtype;
};
void gemm_tile_counts(int64_t n_tok, int64_t c_out, int64_t* tiles_o, int64_t* tiles_t);
hipError_t launch_gemm_loss(const GemmArgs& a, hipStream_t stream);
hipError_t launch_gemm_store(const GemmArgs& a, hipStream_t stream);

// S4 final combine + S5 selection.
hipError_t launch_finalize(const float* partial, int n_cand, int64_t tiles_per_cand, int64_t c_out,
                           const float* s_table, int64_t c_in, float* losses, int32_t* best_idx,
                           float* best_scales, hipStream_t stream);
hipError_t launch_token_err_reduce(const float* tok_partial, int64_t tiles_o, int64_t n_tok,
                                   int64_t c_out, float* per_token_err, hipStream_t stream);

}  // namespace tlq
