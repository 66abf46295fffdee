// S0 (x_stat), S1 (scale table), the final loss combine and S5 (selection).
// All HBM-bound or tiny; none uses floating-point atomics, so results are
// bit-identical from run to run.
#include "common.h"

namespace tlq {

// ---------------------------------------------------------------- S0 x_stat
// Sec. 3.1.2 x_stat (mean variant of the ablation table, or max over all
// tokens).  Each lane owns 8 consecutive channels (one 16-byte load per row);
// the 4 waves of a block walk interleaved rows of the block's row chunk and
// are combined through LDS; chunks are combined by a second kernel.  Sums are
// carried in double: |fp16| values are multiples of 2^-24 below 2^16, so the
// sum over up to 2^37 tokens is exact and the order of addition is immaterial.
constexpr int kXsThreads = 256;
constexpr int kXsCols = 64 * 8;  // channels per block

int xstat_chunks(int64_t n_tok) {
  int64_t c = ceil_div(n_tok, 128);
  return (int)(c < 1 ? 1 : (c > 128 ? 128 : c));
}

template <typename T, int KIND>
__global__ __launch_bounds__(kXsThreads) void xstat_partial_kernel(
    const uint16_t* __restrict__ X, int64_t n_tok, int64_t c_in, int64_t ldx, int rows_per_chunk,
    double* __restrict__ partial, const uint8_t* __restrict__ pos_mask, int64_t period) {
  __shared__ double red[4][kXsCols];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c0 = (int64_t)blockIdx.x * kXsCols + lane * 8;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_chunk;
  int64_t r1 = r0 + rows_per_chunk;
  if (r1 > n_tok) r1 = n_tok;
  double acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.0;
  if (c0 < c_in) {
    for (int64_t r = r0 + wave; r < r1; r += 4) {
      if (pos_mask && !pos_mask[r % period]) continue;   // token position not in the selected set
      const uint4 v = *reinterpret_cast<const uint4*>(X + r * ldx + c0);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint16_t b = (uint16_t)((w[j >> 1] >> ((j & 1) * 16)) & 0x7fffu);  // |x|
        const double a = (double)T::to_float(b);
        if (KIND == 0) acc[j] += a; else acc[j] = a > acc[j] ? a : acc[j];
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) red[wave][lane * 8 + j] = acc[j];
  __syncthreads();
  for (int i = threadIdx.x; i < kXsCols; i += kXsThreads) {
    const int64_t c = (int64_t)blockIdx.x * kXsCols + i;
    if (c < c_in) {
      double s;
      if (KIND == 0) s = ((red[0][i] + red[1][i]) + red[2][i]) + red[3][i];
      else s = fmax(fmax(red[0][i], red[1][i]), fmax(red[2][i], red[3][i]));
      partial[(int64_t)blockIdx.y * c_in + c] = s;
    }
  }
}

template <int KIND>
__global__ void xstat_final_kernel(const double* __restrict__ partial, int n_chunks, int64_t c_in,
                                   int64_t n_tok, float* __restrict__ x_stat) {
  const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= c_in) return;
  double s = 0.0;
  for (int i = 0; i < n_chunks; ++i) {
    const double v = partial[(int64_t)i * c_in + c];
    if (KIND == 0) s += v; else s = v > s ? v : s;
  }
  x_stat[c] = (float)(KIND == 0 ? s / (double)n_tok : s);
}

hipError_t launch_xstat(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx, bool bf16,
                        int kind, double* partial, float* x_stat, hipStream_t stream,
                        const uint8_t* pos_mask, int64_t period) {
  const int chunks = xstat_chunks(n_tok);
  const int rows = (int)ceil_div(n_tok, chunks);
  dim3 grid((unsigned)ceil_div(c_in, kXsCols), (unsigned)chunks);
  const uint16_t* x = (const uint16_t*)X;
  {
    ProfScope ps("xstat_partial", stream, 2.0 * (double)n_tok * (double)c_in);
    if (!bf16 && kind == 0) xstat_partial_kernel<F16, 0><<<grid, kXsThreads, 0, stream>>>(x, n_tok, c_in, ldx, rows, partial, pos_mask, period);
    else if (!bf16) xstat_partial_kernel<F16, 1><<<grid, kXsThreads, 0, stream>>>(x, n_tok, c_in, ldx, rows, partial, pos_mask, period);
    else if (kind == 0) xstat_partial_kernel<BF16, 0><<<grid, kXsThreads, 0, stream>>>(x, n_tok, c_in, ldx, rows, partial, pos_mask, period);
    else xstat_partial_kernel<BF16, 1><<<grid, kXsThreads, 0, stream>>>(x, n_tok, c_in, ldx, rows, partial, pos_mask, period);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ProfScope ps("xstat_final", stream, 8.0 * (double)chunks * (double)c_in);
    const unsigned g2 = (unsigned)ceil_div(c_in, 256);
    if (kind == 0) xstat_final_kernel<0><<<g2, 256, 0, stream>>>(partial, chunks, c_in, n_tok, x_stat);
    else xstat_final_kernel<1><<<g2, 256, 0, stream>>>(partial, chunks, c_in, n_tok, x_stat);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------ S1 scale table
// Sec. 3.1.2 scale equation: s = x_stat^alpha, evaluated in double and rounded
// once; the reciprocal table feeds the folded GEMM operand deq / s.
__device__ __forceinline__ double pow2_shift(const uint32_t* xmax_bits) {
  const int k = xmax_bits ? shift_from_bf16_bits(*xmax_bits) : 0;
  return (double)__builtin_bit_cast(float, (uint32_t)(127 + k) << 23);
}

__global__ void scale_table_kernel(const float* __restrict__ x_stat, int64_t c_in,
                                   const float* __restrict__ alpha, int n_alpha,
                                   float* __restrict__ s_table, float* __restrict__ inv_table,
                                   const uint32_t* __restrict__ xmax_bits) {
  const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int k = blockIdx.y;
  if (c >= c_in || k >= n_alpha) return;
  float xs = x_stat[c];
  xs = xs > kXstatFloor ? xs : kXstatFloor;  // also maps NaN to the floor
  const float s = (float)pow((double)xs, (double)alpha[k]);
  s_table[(int64_t)k * c_in + c] = s;
  if (inv_table) inv_table[(int64_t)k * c_in + c] = (float)(pow2_shift(xmax_bits) / (double)s);
}

hipError_t launch_scale_table(const float* x_stat, int64_t c_in, const float* alpha, int n_alpha,
                              float* s_table, float* inv_table, const uint32_t* xmax_bits,
                              hipStream_t stream) {
  ProfScope ps("scale_table", stream, 8.0 * (double)n_alpha * (double)c_in);
  dim3 grid((unsigned)ceil_div(c_in, 256), (unsigned)n_alpha);
  scale_table_kernel<<<grid, 256, 0, stream>>>(x_stat, c_in, alpha, n_alpha, s_table, inv_table, xmax_bits);
  return hipGetLastError();
}

__global__ void recip_kernel(const float* __restrict__ s, int64_t n, const uint32_t* __restrict__ xmax_bits,
                             float* __restrict__ inv) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) inv[i] = (float)(pow2_shift(xmax_bits) / (double)s[i]);
}

hipError_t launch_recip(const float* s, int64_t c_in, const uint32_t* xmax_bits, float* inv,
                        hipStream_t stream) {
  recip_kernel<<<(unsigned)ceil_div(c_in, 256), 256, 0, stream>>>(s, c_in, xmax_bits, inv);
  return hipGetLastError();
}

// ------------------------------------------------ bf16 activations -> fp16 operand
__global__ void zero_u32_kernel(uint32_t* p) { *p = 0u; }

// max over the tensor of the magnitude bits; for bf16 the integer order of the
// magnitude bits is the order of the magnitudes, so an integer atomic max is exact
// and order independent
__global__ __launch_bounds__(256) void absmax_bits_kernel(const uint16_t* __restrict__ X, int64_t n_tok,
                                                          int64_t c_in, int64_t ldx,
                                                          uint32_t* __restrict__ out) {
  const int64_t chunks = c_in / 8, total = n_tok * chunks;
  uint32_t m = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const uint4 v = *reinterpret_cast<const uint4*>(X + (i / chunks) * ldx + (i % chunks) * 8);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t lo = w[j] & 0x7fffu, hi = (w[j] >> 16) & 0x7fffu;
      m = m > lo ? m : lo;
      m = m > hi ? m : hi;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const uint32_t o = __shfl_xor(m, off, 64);
    m = m > o ? m : o;
  }
  if ((threadIdx.x & 63) == 0) atomicMax(out, m);
}

__global__ __launch_bounds__(256) void bf16_to_f16_kernel(const uint16_t* __restrict__ X, int64_t n_tok,
                                                          int64_t c_in, int64_t ldx,
                                                          const uint32_t* __restrict__ xmax_bits,
                                                          uint16_t* __restrict__ Xh) {
  const int64_t chunks = c_in / 8, total = n_tok * chunks;
  const float scale = __builtin_bit_cast(float, (uint32_t)(127 - shift_from_bf16_bits(*xmax_bits)) << 23);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / chunks, c = (i % chunks) * 8;
    const uint4 v = *reinterpret_cast<const uint4*>(X + r * ldx + c);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float lo = BF16::to_float((uint16_t)w[j]) * scale, hi = BF16::to_float((uint16_t)(w[j] >> 16)) * scale;
      o[j] = (uint32_t)F16::from_float(lo) | ((uint32_t)F16::from_float(hi) << 16);
    }
    *reinterpret_cast<uint4*>(Xh + r * c_in + c) = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

hipError_t launch_xprep(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx, uint32_t* xmax_bits,
                        void* Xh, hipStream_t stream) {
  ProfScope ps("bf16_to_f16", stream, 6.0 * (double)n_tok * (double)c_in);
  const int64_t total = n_tok * (c_in / 8);
  const unsigned grid = (unsigned)(ceil_div(total, 256) < 4096 ? ceil_div(total, 256) : 4096);
  zero_u32_kernel<<<1, 1, 0, stream>>>(xmax_bits);
  absmax_bits_kernel<<<grid, 256, 0, stream>>>((const uint16_t*)X, n_tok, c_in, ldx, xmax_bits);
  bf16_to_f16_kernel<<<grid, 256, 0, stream>>>((const uint16_t*)X, n_tok, c_in, ldx, xmax_bits,
                                               (uint16_t*)Xh);
  return hipGetLastError();
}

// ------------------------------------------- final combine (S4) + select (S5)
// One block.  Wave k sums candidate k's tile partials in double in a fixed
// order (lane-strided, then a fixed butterfly), scales by 1/c_out, and stores
// the loss as float (+inf if not finite).  Thread 0 then picks the first
// minimum (Sec. 3.2.1 argmin) and the block copies that row of the table.
__global__ __launch_bounds__(1024) void finalize_kernel(
    const float* __restrict__ partial, int n_cand, int64_t tiles_per_cand, double inv_c_out,
    const double* __restrict__ factor, const float* __restrict__ s_table, int64_t c_in, float* __restrict__ losses,
    int32_t* __restrict__ best_idx, float* __restrict__ best_scales) {
  __shared__ float sl[TLQ_MAX_ALPHA];
  __shared__ int sbest;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  for (int k = wave; k < n_cand; k += nwaves) {
    double acc = 0.0;
    const float* p = partial + (int64_t)k * tiles_per_cand;
    for (int64_t i = lane; i < tiles_per_cand; i += 64) acc += (double)p[i];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) {
      float l = (float)(acc * inv_c_out * (factor ? *factor : 1.0));
      if (!(l == l) || l == __builtin_inff() || l == -__builtin_inff()) l = __builtin_inff();
      sl[k] = l;
      losses[k] = l;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int b = -1;
    float bl = __builtin_inff();
    for (int k = 0; k < n_cand; ++k)
      if (sl[k] < bl) { bl = sl[k]; b = k; }
    sbest = b;
    if (best_idx) *best_idx = b;
  }
  __syncthreads();
  if (best_scales) {
    const int b = sbest;
    for (int64_t c = threadIdx.x; c < c_in; c += blockDim.x)
      best_scales[c] = b >= 0 ? s_table[(int64_t)b * c_in + c] : __builtin_nanf("");
  }
}

hipError_t launch_finalize(const float* partial, int n_cand, int64_t tiles_per_cand, int64_t c_out,
                           const float* s_table, int64_t c_in, float* losses, int32_t* best_idx,
                           float* best_scales, hipStream_t stream, const double* factor) {
  ProfScope ps("finalize", stream, 4.0 * (double)n_cand * (double)tiles_per_cand);
  finalize_kernel<<<1, 1024, 0, stream>>>(partial, n_cand, tiles_per_cand, 1.0 / (double)c_out,
                                          factor, s_table, c_in, losses, best_idx, best_scales);
  return hipGetLastError();
}

// per_token_err[t] = (1/c_out) * sum over o-tiles of the tile row sums
__global__ void token_err_reduce_kernel(const float* __restrict__ tok_partial, int64_t tiles_o,
                                        int64_t n_tok, double inv_c_out, float* __restrict__ out) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_tok) return;
  double acc = 0.0;
  for (int64_t i = 0; i < tiles_o; ++i) acc += (double)tok_partial[i * n_tok + t];
  out[t] = (float)(acc * inv_c_out);
}

hipError_t launch_token_err_reduce(const float* tok_partial, int64_t tiles_o, int64_t n_tok,
                                   int64_t c_out, float* per_token_err, hipStream_t stream) {
  ProfScope ps("token_err_reduce", stream, 4.0 * (double)tiles_o * (double)n_tok);
  token_err_reduce_kernel<<<(unsigned)ceil_div(n_tok, 256), 256, 0, stream>>>(
      tok_partial, tiles_o, n_tok, 1.0 / (double)c_out, per_token_err);
  return hipGetLastError();
}

// D[t,o] = Y[t,o] - D[t,o]; one thread per element (used once per search in the difference form)
__global__ __launch_bounds__(256) void sub_from_y_kernel(const void* __restrict__ Y, int64_t ldy, int ydt,
                                                         float* __restrict__ D, int64_t ldd, int64_t n_tok,
                                                         int64_t c_out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_tok * c_out) return;
  const int64_t t = i / c_out, o = i % c_out;
  float y;
  if (ydt == TLQ_F32) y = ((const float*)Y)[t * ldy + o];
  else {
    const uint16_t b = ((const uint16_t*)Y)[t * ldy + o];
    y = ydt == TLQ_F16 ? F16::to_float(b) : BF16::to_float(b);
  }
  D[t * ldd + o] = y - D[t * ldd + o];
}

hipError_t launch_sub_from_y(const void* Y, int64_t ldy, int ydt, float* D, int64_t ldd, int64_t n_tok,
                             int64_t c_out, hipStream_t stream) {
  ProfScope ps("sub_from_y", stream, (double)n_tok * (double)c_out * 10.0);
  sub_from_y_kernel<<<(unsigned)ceil_div(n_tok * c_out, 256), 256, 0, stream>>>(Y, ldy, ydt, D, ldd, n_tok, c_out);
  return hipGetLastError();
}

}  // namespace tlq

