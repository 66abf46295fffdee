// Glue of the synthetic decoder block that the calibrated linears sit in (not
// part of the paper's method; Sec. 3.2.1 only requires that activations are
// propagated through the model between two searches): causal self-attention per
// calibration sample, the SiLU gate and the residual addition.  Correct and
// reasonably quick, not tuned: the search kernels take > 90 % of a stack run.
#include "common.h"

namespace tlq {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));

#if defined(__HIP_DEVICE_COMPILE__)
template <typename T> __device__ __forceinline__ f32x16 mma16(u16x8 a, u16x8 b, f32x16 c);
template <> __device__ __forceinline__ f32x16 mma16<F16>(u16x8 a, u16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x16 mma16<BF16>(u16x8 a, u16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
#endif

constexpr int kAttDh = 128;   // head width
constexpr int kAttBq = 128;   // queries per block (32 per wave)
[[maybe_unused]] constexpr int kAttBk = 32;    // keys per step
[[maybe_unused]] constexpr int kAttVtLd = 40;  // 16-bit elements per row of the transposed V tile (80 B: 16-B aligned, off the bank period)

// out[t, head] = softmax_j<=t( q_t . k_j / sqrt(128) ) v_j, rows in blocks of seq_len.
// The matrix cores compute the TRANSPOSED products S^T = K Q^T and O^T = V^T P^T, so that
// a lane owns one query column: the running maximum and sum of the online softmax are
// per-lane scalars shared only with lane ^ 32.  The accumulator registers of S^T, taken
// in order, are a permutation of the 32 keys; the V tile is staged in LDS transposed and
// with its keys in that same permuted order, so P never has to be shuffled between lanes.
template <typename T>
__global__ __launch_bounds__(256) void causal_attention_kernel(
    const uint16_t* __restrict__ Q, int64_t ldq, const uint16_t* __restrict__ K, int64_t ldk,
    const uint16_t* __restrict__ V, int64_t ldv, uint16_t* __restrict__ O, int64_t ldo, int seq_len,
    float scale) {
#if defined(__HIP_DEVICE_COMPILE__)
  __shared__ __attribute__((aligned(16))) uint16_t vt[kAttDh * kAttVtLd];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, h = lane >> 5;
  const int qb = (int)gridDim.x - 1 - (int)blockIdx.x;  // longest rows first
  const int64_t row0 = (int64_t)blockIdx.z * seq_len;
  const int64_t col0 = (int64_t)blockIdx.y * kAttDh;
  const int q0 = qb * kAttBq + wave * 32;
  const int q = q0 + l32;                      // may lie past the end of the sample: computed, never stored
  const int qc = q < seq_len ? q : seq_len - 1;

  u16x8 qf[8];
  {
    const uint16_t* qp = Q + (row0 + qc) * ldq + col0 + 8 * h;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const u16x8*>(qp + 16 * s);
  }
  f32x16 acc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[dt][v] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;

  int last_q = qb * kAttBq + kAttBq - 1;
  if (last_q > seq_len - 1) last_q = seq_len - 1;
  const int n_kb = last_q / kAttBk + 1;
  int wave_last_q = q0 + 31;
  if (wave_last_q > seq_len - 1) wave_last_q = seq_len - 1;

  for (int kb = 0; kb < n_kb; ++kb) {
    __syncthreads();  // every wave is done with the previous V tile
    {
      const int key_local = tid >> 3, d0 = (tid & 7) * 16;
      int key = kb * kAttBk + key_local;
      if (key > seq_len - 1) key = seq_len - 1;  // masked below
      const uint16_t* vp = V + (row0 + key) * ldv + col0 + d0;
      const u16x8 a = *reinterpret_cast<const u16x8*>(vp);
      const u16x8 b = *reinterpret_cast<const u16x8*>(vp + 8);
      // key_local = 16 s + 8 jj + 4 hh + i  is stored at  16 s + 8 hh + 4 jj + i
      const int pos = (key_local & 16) | ((key_local & 4) << 1) | ((key_local & 8) >> 1) | (key_local & 3);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        vt[(d0 + e) * kAttVtLd + pos] = a[e];
        vt[(d0 + 8 + e) * kAttVtLd + pos] = b[e];
      }
    }
    __syncthreads();
    if (kb * kAttBk <= wave_last_q) {  // wave-uniform: some query of this wave sees this key block
      f32x16 s;
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] = 0.0f;
      {
        int kc = kb * kAttBk + l32;
        if (kc > seq_len - 1) kc = seq_len - 1;
        const uint16_t* kp = K + (row0 + kc) * ldk + col0 + 8 * h;
#pragma unroll
        for (int st = 0; st < 8; ++st) s = mma16<T>(*reinterpret_cast<const u16x8*>(kp + 16 * st), qf[st], s);
      }
      float mx = -INFINITY;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = kb * kAttBk + 8 * (v >> 2) + 4 * h + (v & 3);
        const float x = (key <= q && key < seq_len) ? s[v] * scale : -INFINITY;
        s[v] = x;
        mx = fmaxf(mx, x);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // key 0 is visible to every query and is part of the first block, so m_new is finite
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __expf(m_run - m_new);
      float ps = 0.0f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float pv = __expf(s[v] - m_new);
        ps += pv;
        s[v] = pv;
      }
      l_run = l_run * alpha + ps;
      m_run = m_new;
      u16x8 pf[2];
#pragma unroll
      for (int sl = 0; sl < 2; ++sl)
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[sl][e] = T::from_float(s[8 * sl + e]);
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[dt][v] *= alpha;
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
          const u16x8 a = *reinterpret_cast<const u16x8*>(&vt[(32 * dt + l32) * kAttVtLd + 16 * sl + 8 * h]);
          acc[dt] = mma16<T>(a, pf[sl], acc[dt]);
        }
      }
    }
  }
  l_run += __shfl_xor(l_run, 32, 64);
  if (q < seq_len) {
    const float inv = 1.0f / l_run;
    uint16_t* op = O + (row0 + q) * ldo + col0 + 4 * h;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        u16x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = T::from_float(acc[dt][4 * j + i] * inv);
        *reinterpret_cast<u16x4*>(op + 32 * dt + 8 * j) = o;
      }
  }
#endif
}

hipError_t launch_causal_attention(const void* Q, int64_t ldq, const void* K, int64_t ldk, const void* V,
                                   int64_t ldv, int64_t n_tok, int n_heads, int seq_len, bool bf16, void* O,
                                   int64_t ldo, hipStream_t stream) {
  const int64_t n_samples = n_tok / seq_len;
  // causal: half of the seq_len^2 score matrix; 2 products of 2*128 flop per score
  ProfScope ps("causal_attention", stream, 2.0 * (double)n_samples * n_heads * (double)seq_len * seq_len * kAttDh);
  const dim3 grid((unsigned)ceil_div(seq_len, kAttBq), (unsigned)n_heads, (unsigned)n_samples);
  const float scale = 0.08838834764831845f;  // 1 / sqrt(128)
  if (!bf16)
    causal_attention_kernel<F16><<<grid, 256, 0, stream>>>((const uint16_t*)Q, ldq, (const uint16_t*)K, ldk,
                                                           (const uint16_t*)V, ldv, (uint16_t*)O, ldo, seq_len, scale);
  else
    causal_attention_kernel<BF16><<<grid, 256, 0, stream>>>((const uint16_t*)Q, ldq, (const uint16_t*)K, ldk,
                                                            (const uint16_t*)V, ldv, (uint16_t*)O, ldo, seq_len, scale);
  return hipGetLastError();
}

// MODE 0: out = SiLU(a) * b;  MODE 1: out = a + b.  8 elements per thread; c % 8 == 0.
template <typename T, int MODE>
__global__ __launch_bounds__(256) void pairwise_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                       const uint16_t* __restrict__ B, int64_t ldb, int64_t n_tok,
                                                       int64_t c8, uint16_t* __restrict__ out, int64_t ldo) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_tok * c8) return;
  const int64_t row = i / c8, col = (i % c8) * 8;
  const u16x8 a = *reinterpret_cast<const u16x8*>(A + row * lda + col);
  const u16x8 b = *reinterpret_cast<const u16x8*>(B + row * ldb + col);
  u16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float x = T::to_float(a[e]), y = T::to_float(b[e]);
    o[e] = T::from_float(MODE == 0 ? x / (1.0f + __expf(-x)) * y : x + y);
  }
  *reinterpret_cast<u16x8*>(out + row * ldo + col) = o;
}

hipError_t launch_pairwise(int mode, const void* A, int64_t lda, const void* B, int64_t ldb, int64_t n_tok,
                           int64_t c, bool bf16, void* out, int64_t ldo, hipStream_t stream) {
  ProfScope ps(mode == 0 ? "silu_mul" : "residual_add", stream, 6.0 * (double)n_tok * (double)c);
  const int64_t c8 = c / 8;
  const unsigned grid = (unsigned)ceil_div(n_tok * c8, 256);
#define TLQ_PW(TT, M)                                                                                          \
  pairwise_kernel<TT, M><<<grid, 256, 0, stream>>>((const uint16_t*)A, lda, (const uint16_t*)B, ldb, n_tok, c8, \
                                                   (uint16_t*)out, ldo)
  if (mode == 0) { if (bf16) TLQ_PW(BF16, 0); else TLQ_PW(F16, 0); }
  else           { if (bf16) TLQ_PW(BF16, 1); else TLQ_PW(F16, 1); }
#undef TLQ_PW
  return hipGetLastError();
}

}  // namespace tlq
