// Glue of the synthetic sequential-calibration chain (not part of the paper's
// method): turns the quantised output of one linear into the exposed input of
// the next one (Sec. 3.2.1 PassAct2 feeds each layer the previous quantised
// layer's output; what sits between two linears of the synthetic stack is a
// row-wise RMS normalisation, an optional elementwise product of two branches
// and a fixed per-channel multiplier that re-imposes the outlier channels).
// HBM-bound, one wave per row, untuned on purpose.
#include "common.h"

namespace tlq {

// out[t,c] = round16( v[t,c] / sqrt(mean_c v[t,:]^2 + 1e-6) * m(t)[c] ),
// v = Z (or Z * Zb elementwise); m(t) = m_a when (t % period) < split, else m_b.
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_mul_kernel(const uint16_t* __restrict__ Z, int64_t ldz,
                                                          const uint16_t* __restrict__ Zb, int64_t ldzb,
                                                          int64_t n_tok, int64_t c, const float* __restrict__ m_a,
                                                          const float* __restrict__ m_b, int period, int split,
                                                          uint16_t* __restrict__ out, int64_t ldo) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n_tok) return;
  float ss = 0.0f;
  for (int64_t j = lane; j < c; j += 64) {
    float v = T::to_float(Z[row * ldz + j]);
    if (Zb) v *= T::to_float(Zb[row * ldzb + j]);
    ss += v * v;
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
  const float inv = 1.0f / sqrtf(ss / (float)c + 1e-6f);
  const float* m = (period > 0 && (int)(row % period) >= split) ? m_b : m_a;
  for (int64_t j = lane; j < c; j += 64) {
    float v = T::to_float(Z[row * ldz + j]);
    if (Zb) v *= T::to_float(Zb[row * ldzb + j]);
    out[row * ldo + j] = T::from_float(v * inv * (m ? m[j] : 1.0f));
  }
}

hipError_t launch_rmsnorm_mul(const void* Z, int64_t ldz, const void* Zb, int64_t ldzb, int64_t n_tok,
                              int64_t c, bool bf16, const float* m_a, const float* m_b, int period,
                              int split, void* out, int64_t ldo, hipStream_t stream) {
  ProfScope ps("rmsnorm_mul", stream, (Zb ? 6.0 : 4.0) * (double)n_tok * (double)c);
  const unsigned grid = (unsigned)ceil_div(n_tok, 4);
  if (!bf16)
    rmsnorm_mul_kernel<F16><<<grid, 256, 0, stream>>>((const uint16_t*)Z, ldz, (const uint16_t*)Zb, ldzb, n_tok,
                                                      c, m_a, m_b, period, split, (uint16_t*)out, ldo);
  else
    rmsnorm_mul_kernel<BF16><<<grid, 256, 0, stream>>>((const uint16_t*)Z, ldz, (const uint16_t*)Zb, ldzb, n_tok,
                                                       c, m_a, m_b, period, split, (uint16_t*)out, ldo);
  return hipGetLastError();
}

}  // namespace tlq
