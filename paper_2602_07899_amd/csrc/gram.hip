// Second-moment form of the search objective (Sec. 3.2, eq. for r*; weight-only f_q).
//
// With no activation quantiser the quantised layer is linear in the tokens, so the weighted error
// of candidate k is a quadratic form in the weight error D_k = W - What_k:
//   sum_t w_t (1/C_out) ||x_t W^T - x_t What_k^T||^2 = (1/C_out) sum_o d_o^T G d_o,
//   G = sum_t w_t x_t x_t^T   (C_in x C_in, independent of the candidate and of the linear).
// G costs one pass of 2 N C_in^2 flops (half of it: G is symmetric) and every candidate
// 2 C_out C_in^2 instead of 2 N C_in C_out: N / C_in times fewer.  The kernels here prepare the
// operands; the two contractions run on the tile kernels of gemm.hip.
//
// Conditioning.  G is held in fp16 as C[i,j] = G'[i,j] 2^-(e_i + e_j) with G' = G / max_t w_t and
// e_c = round(log2(G'[c,c]) / 2): |C| <= 2 whatever the spread of the channel magnitudes, and the
// weight errors are emitted as D'[o,c] = D[o,c] 2^(e_c - m).  Both scalings are powers of two, so
// they change no rounding; d^T G d = max_t w_t 2^(2m) d'^T C d'.
#include <climits>

#include "common.h"

namespace tlq {
namespace {

__global__ __launch_bounds__(1024) void gram_wmax_kernel(const float* __restrict__ w, int64_t n,
                                                         float* __restrict__ out) {
  __shared__ float red[16];
  float m = 0.0f;
  for (int64_t i = threadIdx.x; i < n; i += 1024) m = fmaxf(m, w[i]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i < 16; ++i) m = fmaxf(m, red[i]);
    out[0] = m;
  }
}

// out[c, t] = fp16(X[t, c] * sqrt(w_t / wmax)) for t < n_tok, 0 for n_tok <= t < kp.
// One block transposes 64 tokens x 64 channels through LDS: 16-byte loads along the channels,
// 16-byte stores along the tokens.
constexpr int GT = 64, GLD = GT + 8;   // LDS row stride in halves (keeps 16-byte alignment)
template <typename T>
__global__ __launch_bounds__(256) void gram_operand_kernel(const uint16_t* __restrict__ X, int64_t n_tok,
                                                           int64_t c_in, int64_t ldx,
                                                           const float* __restrict__ w,
                                                           const float* __restrict__ wmax,
                                                           uint16_t* __restrict__ out, int64_t kp) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[GT * GLD];   // [channel][token]
  const int64_t t0 = (int64_t)blockIdx.x * GT, c0 = (int64_t)blockIdx.y * GT;
  const float wm = *wmax;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int idx = i * 256 + threadIdx.x;     // 64 token rows x 8 chunks of 8 channels
    const int tr = idx >> 3, ch = idx & 7;
    const int64_t t = t0 + tr, c = c0 + ch * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    float r = 0.0f;
    if (t < n_tok && c < c_in) {
      v = *reinterpret_cast<const uint4*>(X + t * ldx + c);
      r = wm > 0.0f ? sqrtf(w[t] / wm) : 0.0f;
    }
    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float x = T::to_float((uint16_t)(u[j >> 1] >> ((j & 1) * 16)));
      tile[(ch * 8 + j) * GLD + tr] = F16::from_float(x * r);
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int idx = i * 256 + threadIdx.x;     // 64 channel rows x 8 chunks of 8 tokens
    const int cr = idx >> 3, ch = idx & 7;
    const int64_t c = c0 + cr, t = t0 + ch * 8;
    if (c < c_in && t < kp)
      *reinterpret_cast<uint4*>(out + c * kp + t) = *reinterpret_cast<const uint4*>(tile + cr * GLD + ch * 8);
  }
}

// e[c] = round(log2(H[c,c]) / 2) (0 for an all-zero channel); m = max e - 10;
// col_scale[c] = 2^(e_c - m); factor = wmax * 2^(2m).
__global__ __launch_bounds__(1024) void gram_diag_kernel(const float* __restrict__ H, int64_t c_in,
                                                         const float* __restrict__ wmax, int* __restrict__ e,
                                                         float* __restrict__ col_scale, double* __restrict__ factor) {
  __shared__ int red[16];
  __shared__ int sm;
  int emax = INT_MIN;
  for (int64_t c = threadIdx.x; c < c_in; c += 1024) {
    const float h = H[c * c_in + c];
    int ec = 0;
    if (h > 0.0f && h < __builtin_inff()) {
      ec = (int)rintf(0.5f * log2f(h));
      emax = ec > emax ? ec : emax;
    }
    e[c] = ec;
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const int o = __shfl_xor(emax, off, 64);
    emax = o > emax ? o : emax;
  }
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = emax;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i < 16; ++i) emax = red[i] > emax ? red[i] : emax;
    if (emax == INT_MIN) emax = 0;
    sm = emax - 10;
    *factor = (double)*wmax * __builtin_ldexp(1.0, 2 * sm);
  }
  __syncthreads();
  const int m = sm;
  for (int64_t c = threadIdx.x; c < c_in; c += 1024) {
    int d = e[c] - m;
    d = d < -100 ? -100 : d;
    col_scale[c] = __builtin_ldexpf(1.0f, d);
  }
}

// H[0] += H[1] + ... + H[n_split - 1] in that order, over the 64 x 64 blocks of the computed
// triangle (split-k partial products, each [c_in, c_in] float, `stride` elements apart).
__global__ __launch_bounds__(256) void gram_reduce_kernel(float* __restrict__ H, int64_t c_in, int n_split,
                                                          int64_t stride) {
  const int64_t a0 = (int64_t)blockIdx.y * GT, b0 = (int64_t)blockIdx.x * GT;
  if ((b0 / 256) > (a0 / 256)) return;
  for (int i = threadIdx.x; i < GT * GT / 4; i += 256) {
    const int64_t a = a0 + i / (GT / 4), b = b0 + (i % (GT / 4)) * 4;
    if (a >= c_in || b >= c_in) continue;     // c_in % 4 == 0: whole groups of four
    float4 acc = *reinterpret_cast<const float4*>(H + a * c_in + b);
    for (int k = 1; k < n_split; ++k) {
      const float4 v = *reinterpret_cast<const float4*>(H + k * stride + a * c_in + b);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    *reinterpret_cast<float4*>(H + a * c_in + b) = acc;
  }
}

// C[a,b] = fp16(H[a,b] * 2^-(e_a + e_b)).  H holds the 256 x 256 tiles whose column tile is not
// beyond their row tile; the others are read from the mirrored position.  A 64 x 64 block lies
// inside one such tile, so the choice is uniform per block.
__global__ __launch_bounds__(256) void gram_convert_kernel(const float* __restrict__ H, int64_t c_in,
                                                           const int* __restrict__ e, uint16_t* __restrict__ C) {
  __shared__ float tile[GT][GT + 1];
  const int64_t a0 = (int64_t)blockIdx.y * GT, b0 = (int64_t)blockIdx.x * GT;
  const bool direct = (b0 / 256) <= (a0 / 256);
  const int64_t r0 = direct ? a0 : b0, q0 = direct ? b0 : a0;    // source rows / columns
  for (int i = threadIdx.x; i < GT * GT; i += 256) {
    const int r = i / GT, q = i % GT;
    float v = 0.0f;
    if (r0 + r < c_in && q0 + q < c_in) v = H[(r0 + r) * c_in + q0 + q];
    tile[r][q] = v;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < GT * GT; i += 256) {
    const int ar = i / GT, bq = i % GT;
    const int64_t a = a0 + ar, b = b0 + bq;
    if (a < c_in && b < c_in) {
      const float v = direct ? tile[ar][bq] : tile[bq][ar];
      C[a * c_in + b] = F16::from_float(__builtin_ldexpf(v, -(e[a] + e[b])));
    }
  }
}

}  // namespace

hipError_t launch_gram_operand(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx, bool bf16,
                               const float* token_w, float* wmax, void* out, int64_t kp, hipStream_t stream) {
  const int64_t bx = ceil_div(kp, GT), by = ceil_div(c_in, GT);
  if (bx > 0x7fffffffLL || by > 65535) return hipErrorInvalidValue;
  ProfScope ps("gram_operand", stream, 2.0 * (double)n_tok * (double)c_in + 2.0 * (double)kp * (double)c_in);
  gram_wmax_kernel<<<1, 1024, 0, stream>>>(token_w, n_tok, wmax);
  const dim3 grid((unsigned)bx, (unsigned)by);
  if (!bf16)
    gram_operand_kernel<F16><<<grid, 256, 0, stream>>>((const uint16_t*)X, n_tok, c_in, ldx, token_w, wmax,
                                                       (uint16_t*)out, kp);
  else
    gram_operand_kernel<BF16><<<grid, 256, 0, stream>>>((const uint16_t*)X, n_tok, c_in, ldx, token_w, wmax,
                                                        (uint16_t*)out, kp);
  return hipGetLastError();
}

hipError_t launch_gram_finish(float* H, int64_t c_in, int n_split, int64_t split_stride, const float* wmax,
                              int* e, double* factor, float* col_scale, void* C, hipStream_t stream) {
  const int64_t b = ceil_div(c_in, GT);
  if (b > 65535) return hipErrorInvalidValue;
  ProfScope ps("gram_scale", stream, (6.0 + 2.0 * n_split) * (double)c_in * (double)c_in);
  if (n_split > 1)
    gram_reduce_kernel<<<dim3((unsigned)b, (unsigned)b), 256, 0, stream>>>(H, c_in, n_split, split_stride);
  gram_diag_kernel<<<1, 1024, 0, stream>>>(H, c_in, wmax, e, col_scale, factor);
  gram_convert_kernel<<<dim3((unsigned)b, (unsigned)b), 256, 0, stream>>>(H, c_in, e, (uint16_t*)C);
  return hipGetLastError();
}

}  // namespace tlq
