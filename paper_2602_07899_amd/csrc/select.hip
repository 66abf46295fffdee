// Gradient-guided token selection (Sec. 3.1.2): the per-position gradient
// statistic sum_n = sum_b ||g_{b,n}||, the Top-K position set I, and (in
// stats.hip) the channel maximum over the selected positions.  Small,
// HBM-bound kernels; all reductions run in double in a fixed order.
#include "common.h"

namespace tlq {

// one wave per gradient row: mean_c |g| (the reading of the text) or the Euclidean norm
template <typename T>
__global__ __launch_bounds__(256) void row_norm_kernel(const uint16_t* __restrict__ G, int64_t rows, int64_t c,
                                                       int64_t ldg, int l2, double* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  double acc = 0.0;
  for (int64_t j = lane; j < c; j += 64) {
    const double v = (double)T::to_float(G[row * ldg + j]);
    acc += l2 ? v * v : fabs(v);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if (lane == 0) out[row] = l2 ? sqrt(acc) : acc / (double)c;
}

__global__ void position_sum_kernel(const double* __restrict__ row_norm, int64_t n_samples, int64_t n_pos,
                                    double* __restrict__ sum_n) {
  const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= n_pos) return;
  double s = 0.0;
  for (int64_t b = 0; b < n_samples; ++b) s += row_norm[b * n_pos + n];
  sum_n[n] = s;
}

hipError_t launch_token_importance(const void* G, int64_t n_samples, int64_t n_pos, int64_t c, int64_t ldg,
                                   bool bf16, bool l2, double* row_norm, double* sum_n, hipStream_t stream) {
  ProfScope ps("token_importance", stream, 2.0 * (double)n_samples * (double)n_pos * (double)c);
  const int64_t rows = n_samples * n_pos;
  const unsigned grid = (unsigned)ceil_div(rows, 4);
  if (!bf16) row_norm_kernel<F16><<<grid, 256, 0, stream>>>((const uint16_t*)G, rows, c, ldg, l2 ? 1 : 0, row_norm);
  else row_norm_kernel<BF16><<<grid, 256, 0, stream>>>((const uint16_t*)G, rows, c, ldg, l2 ? 1 : 0, row_norm);
  position_sum_kernel<<<(unsigned)ceil_div(n_pos, 256), 256, 0, stream>>>(row_norm, n_samples, n_pos, sum_n);
  return hipGetLastError();
}

// I = Top_k: position i is selected when fewer than k positions rank ahead of it
// (larger value, or equal value and lower index).  Rank by counting: O(n_pos^2), n_pos is
// a sequence length.
__global__ void topk_mask_kernel(const double* __restrict__ sum_n, int64_t n_pos, int64_t k,
                                 uint8_t* __restrict__ mask) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_pos) return;
  const double v = sum_n[i];
  int64_t ahead = 0;
  for (int64_t j = 0; j < n_pos; ++j) {
    const double u = sum_n[j];
    ahead += (u > v || (u == v && j < i)) ? 1 : 0;
  }
  mask[i] = ahead < k ? 1 : 0;
}

hipError_t launch_topk_mask(const double* sum_n, int64_t n_pos, int64_t k, uint8_t* mask, hipStream_t stream) {
  ProfScope ps("topk_mask", stream, 8.0 * (double)n_pos);
  topk_mask_kernel<<<(unsigned)ceil_div(n_pos, 256), 256, 0, stream>>>(sum_n, n_pos, k, mask);
  return hipGetLastError();
}

}  // namespace tlq
