// S2: group-wise fake quantisation of W * diag(s) (Sec. 2.2 quantiser in its
// min/max form; Sec. 3.2.1 Q_w(W * scale)).
//
// This file is compiled with floating-point contraction off: every float
// operation below rounds exactly once, in the order written, so the integer
// codes, zero points and steps are reproducible bit for bit.
//
// One pass reads W once and emits the operands of ALL candidates of the
// search: per candidate k the folded 16-bit matrix  What_k = deq_k / s_k  that
// the contraction kernel multiplies with the *unscaled* tokens (the smoothing
// identity of Sec. 2.2 moves diag(s)^-1 from X onto the dequantised weights).
// HBM traffic per weight element: 2 B read + 2 B written per candidate.
#include "common.h"

namespace tlq {

struct QuantDev {
  const uint16_t* W; int64_t c_out, c_in, ldw;
  float qmax, qlo, qhi; int half;  // asym: codes in [0,qmax]; sym: q in [qlo,qhi], half = 2^(bits-1)
  int group;                        // resolved group size (>= 8)
  const float* s_table; const float* inv_table; int n_cand;
  uint16_t* what; int64_t what_cand_stride; bool what_f16;
  uint8_t* codes; uint8_t* zp; float* delta; uint16_t* wdq; int64_t ld_dq;
  bool diff; const uint32_t* xmax_bits;  // what = deq*inv - W*2^shift
  const float* col_scale;                // [c_in] factor on `what` or NULL
};

template <bool SYM>
__device__ __forceinline__ void grid_params(float mx, float mn, const QuantDev& a, float& delta,
                                            float& zpf) {
  if (!SYM) {
    float rng = mx - mn;
    rng = fmaxf(rng, kRangeFloor);
    delta = rng / a.qmax;
    float z = rintf((-mn) / delta);
    zpf = fminf(fmaxf(z, 0.0f), a.qmax);
  } else {
    const float amax = fmaxf(mx, kRangeFloor);  // mx carries max|ws|
    delta = amax / a.qhi;
    zpf = (float)a.half;
  }
}

// rint(fl(ws / delta)) without a division per element.  With r = fl(1/delta),
// t = fl(ws * r) lies within 3 * 2^-24 * |Q| of the correctly rounded quotient q of
// Q = ws/delta, so rint(t) == rint(q) unless a half-integer sits inside that gap.  When t is
// that close to a half-integer (about one element in 10^5) the true division decides.
__device__ __forceinline__ float rint_quotient(float ws, float delta, float rdelta) {
  const float t = ws * rdelta;
  float n = rintf(t);
  const float gap = 0.5f - fabsf(t - n);                  // distance of t to the nearest tie
  if (!(gap > fabsf(t) * 4.8e-7f + 2.4e-7f)) n = rintf(ws / delta);   // also taken for NaN/inf
  return n;
}

template <bool SYM>
__device__ __forceinline__ void quant_one(float ws, float delta, float rdelta, float zpf,
                                          const QuantDev& a, float& code, float& deq) {
  if (!SYM) {
    float q = rint_quotient(ws, delta, rdelta) + zpf;
    q = fminf(fmaxf(q, 0.0f), a.qmax);
    code = q;
    deq = (q - zpf) * delta;
  } else {
    float q = rint_quotient(ws, delta, rdelta);
    q = fminf(fmaxf(q, a.qlo), a.qhi);
    code = q + zpf;
    deq = q * delta;
  }
}

// Fast path: group is a power of two in [8, 512].  A lane owns 8 consecutive
// input channels; a group is `group/8` adjacent lanes; a wave covers 512
// channels of one output row.  Min/max go through a butterfly inside the
// lane group; W stays in registers while the candidates are looped over.
// AUX = false drops the single-candidate outputs (codes, zero points, steps, dequantised
// weights) at compile time: the search only needs the folded operands.
template <typename T, bool SYM, bool AUX>
__global__ __launch_bounds__(256) void quant_pow2_kernel(QuantDev a) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t cblocks = (a.c_in + 511) / 512;
  const int64_t row = wave / cblocks;
  if (row >= a.c_out) return;
  const int64_t c = (wave % cblocks) * 512 + lane * 8;
  const bool active = c < a.c_in;
  const int lpg = a.group >> 3;

  float w[8];
  {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (active) v = *reinterpret_cast<const uint4*>(a.W + row * a.ldw + c);
    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) w[j] = T::to_float((uint16_t)(u[j >> 1] >> ((j & 1) * 16)));
  }
  const int64_t gidx = row * (a.c_in / a.group) + c / a.group;

  const float wsub = a.diff ? (a.xmax_bits ? __builtin_ldexpf(1.0f, shift_from_bf16_bits(*a.xmax_bits)) : 1.0f) : 0.0f;
  float cs[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) cs[j] = 1.0f;
  if (active && a.col_scale) {
    const float4 c0 = *reinterpret_cast<const float4*>(a.col_scale + c);
    const float4 c1 = *reinterpret_cast<const float4*>(a.col_scale + c + 4);
    cs[0] = c0.x; cs[1] = c0.y; cs[2] = c0.z; cs[3] = c0.w;
    cs[4] = c1.x; cs[5] = c1.y; cs[6] = c1.z; cs[7] = c1.w;
  }
  for (int k = 0; k < a.n_cand; ++k) {
    float s[8], inv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { s[j] = 1.0f; inv[j] = 1.0f; }
    if (active && a.s_table) {
      const float4 s0 = *reinterpret_cast<const float4*>(a.s_table + (int64_t)k * a.c_in + c);
      const float4 s1 = *reinterpret_cast<const float4*>(a.s_table + (int64_t)k * a.c_in + c + 4);
      s[0] = s0.x; s[1] = s0.y; s[2] = s0.z; s[3] = s0.w;
      s[4] = s1.x; s[5] = s1.y; s[6] = s1.z; s[7] = s1.w;
    }
    if (active && a.inv_table && a.what) {
      const float4 i0 = *reinterpret_cast<const float4*>(a.inv_table + (int64_t)k * a.c_in + c);
      const float4 i1 = *reinterpret_cast<const float4*>(a.inv_table + (int64_t)k * a.c_in + c + 4);
      inv[0] = i0.x; inv[1] = i0.y; inv[2] = i0.z; inv[3] = i0.w;
      inv[4] = i1.x; inv[5] = i1.y; inv[6] = i1.z; inv[7] = i1.w;
    }
    float ws[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) ws[j] = w[j] * s[j];
    float mx, mn;
    if (!SYM) {
      mx = ws[0]; mn = ws[0];
#pragma unroll
      for (int j = 1; j < 8; ++j) { mx = fmaxf(mx, ws[j]); mn = fminf(mn, ws[j]); }
    } else {
      mx = fabsf(ws[0]); mn = 0.0f;
#pragma unroll
      for (int j = 1; j < 8; ++j) mx = fmaxf(mx, fabsf(ws[j]));
    }
    for (int off = 1; off < lpg; off <<= 1) {
      mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      if (!SYM) mn = fminf(mn, __shfl_xor(mn, off, 64));
    }
    float delta, zpf;
    grid_params<SYM>(mx, mn, a, delta, zpf);
    const float rdelta = 1.0f / delta;

    uint32_t cw[2] = {0, 0};
    uint32_t hw[4] = {0, 0, 0, 0}, dw[4] = {0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float code, deq;
      quant_one<SYM>(ws[j], delta, rdelta, zpf, a, code, deq);
      float folded = deq * inv[j];
      if (a.diff) folded -= w[j] * wsub;
      if (a.col_scale) folded *= cs[j];
      hw[j >> 1] |= (uint32_t)(a.what_f16 ? F16::from_float(folded) : T::from_float(folded)) << ((j & 1) * 16);
      if (AUX) {
        cw[j >> 2] |= ((uint32_t)code & 0xffu) << ((j & 3) * 8);
        dw[j >> 1] |= (uint32_t)T::from_float(deq) << ((j & 1) * 16);
      }
    }
    if (!active) continue;
    if (a.what)
      *reinterpret_cast<uint4*>(a.what + (int64_t)k * a.what_cand_stride + row * a.c_in + c) =
          make_uint4(hw[0], hw[1], hw[2], hw[3]);
    if (AUX && k == 0) {  // auxiliary outputs describe a single candidate
      if (a.codes) *reinterpret_cast<uint2*>(a.codes + row * a.c_in + c) = make_uint2(cw[0], cw[1]);
      if (a.wdq)
        *reinterpret_cast<uint4*>(a.wdq + row * a.ld_dq + c) = make_uint4(dw[0], dw[1], dw[2], dw[3]);
      if ((lane & (lpg - 1)) == 0) {
        if (a.zp) a.zp[gidx] = (uint8_t)zpf;
        if (a.delta) a.delta[gidx] = delta;
      }
    }
  }
}

// General path: any group size that is a multiple of 8 (including the whole
// row).  One wave per (row, group); two sweeps over the group per candidate.
template <typename T, bool SYM>
__global__ __launch_bounds__(256) void quant_any_kernel(QuantDev a) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t G = a.c_in / a.group;
  if (wave >= a.c_out * G) return;
  const int64_t row = wave / G;
  const int64_t c0 = (wave % G) * a.group;
  const float wsub = a.diff ? (a.xmax_bits ? __builtin_ldexpf(1.0f, shift_from_bf16_bits(*a.xmax_bits)) : 1.0f) : 0.0f;
  for (int k = 0; k < a.n_cand; ++k) {
    const float* sk = a.s_table ? a.s_table + (int64_t)k * a.c_in : nullptr;
    const float* ik = (a.inv_table && a.what) ? a.inv_table + (int64_t)k * a.c_in : nullptr;
    float mx = SYM ? 0.0f : -__builtin_inff(), mn = __builtin_inff();
    for (int64_t c = c0 + lane; c < c0 + a.group; c += 64) {
      const float ws = T::to_float(a.W[row * a.ldw + c]) * (sk ? sk[c] : 1.0f);
      if (!SYM) { mx = fmaxf(mx, ws); mn = fminf(mn, ws); } else mx = fmaxf(mx, fabsf(ws));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      if (!SYM) mn = fminf(mn, __shfl_xor(mn, off, 64));
    }
    float delta, zpf;
    grid_params<SYM>(mx, mn, a, delta, zpf);
    const float rdelta = 1.0f / delta;
    for (int64_t c = c0 + lane; c < c0 + a.group; c += 64) {
      const float ws = T::to_float(a.W[row * a.ldw + c]) * (sk ? sk[c] : 1.0f);
      float code, deq;
      quant_one<SYM>(ws, delta, rdelta, zpf, a, code, deq);
      if (a.what)
        {
          float folded = deq * (ik ? ik[c] : 1.0f);
          if (a.diff) folded -= T::to_float(a.W[row * a.ldw + c]) * wsub;
          if (a.col_scale) folded *= a.col_scale[c];
          a.what[(int64_t)k * a.what_cand_stride + row * a.c_in + c] =
              a.what_f16 ? F16::from_float(folded) : T::from_float(folded);
        }
      if (k == 0) {
        if (a.codes) a.codes[row * a.c_in + c] = (uint8_t)code;
        if (a.wdq) a.wdq[row * a.ld_dq + c] = T::from_float(deq);
      }
    }
    if (k == 0 && lane == 0) {
      if (a.zp) a.zp[wave] = (uint8_t)zpf;
      if (a.delta) a.delta[wave] = delta;
    }
  }
}

// ---------------------------------------------------------------------------
// Q_a (Sec. 3.2.1 f_q; quantiser of Sec. 2.2 applied per token row):
//   xt = x * inv ; sigma = max(max_c |xt|, 1e-5) / (2^(n-1) - 1) ;
//   code = clip(rint(xt / sigma), -2^(n-1), 2^(n-1) - 1).
// Two tiled passes so that a tile of X (8 rows x 8 channels per lane) stays in
// registers for all candidates and a candidate's reciprocal scales are loaded
// once per 8 rows: (1) row maxima, combined across the channel strips with an
// integer atomic max on the float bit pattern (non-negative floats order like
// integers, so the result is exact and order independent); (2) the codes,
// written as fp16 integers (exact), so the contraction runs on the same MFMA
// path and the per-token step is applied to the accumulators in its epilogue.
constexpr int kAqRows = 8;      // rows per wave
constexpr int kAqCols = 512;    // channels per block strip (64 lanes x 8)

template <typename T>
__device__ __forceinline__ void aq_load_tile(const uint16_t* __restrict__ X, int64_t n_tok, int64_t c_in,
                                             int64_t ldx, int64_t r0, int64_t c, float (&x)[kAqRows][8]) {
#pragma unroll
  for (int r = 0; r < kAqRows; ++r) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r0 + r < n_tok && c < c_in) v = *reinterpret_cast<const uint4*>(X + (r0 + r) * ldx + c);
    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) x[r][j] = T::to_float((uint16_t)(u[j >> 1] >> ((j & 1) * 16)));
  }
}
__device__ __forceinline__ void aq_load_inv(const float* __restrict__ inv, int64_t c, int64_t c_in, float (&iv)[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j) iv[j] = 1.0f;
  if (inv && c < c_in) {
    const float4 a = *reinterpret_cast<const float4*>(inv + c), b = *reinterpret_cast<const float4*>(inv + c + 4);
    iv[0] = a.x; iv[1] = a.y; iv[2] = a.z; iv[3] = a.w; iv[4] = b.x; iv[5] = b.y; iv[6] = b.z; iv[7] = b.w;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void act_amax_kernel(const uint16_t* __restrict__ X, int64_t n_tok,
                                                       int64_t c_in, int64_t ldx,
                                                       const float* __restrict__ inv_table, int k0, int nb,
                                                       uint32_t* __restrict__ amax_bits) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c = (int64_t)blockIdx.x * kAqCols + lane * 8;
  const int64_t r0 = ((int64_t)blockIdx.y * 4 + wave) * kAqRows;
  if (r0 >= n_tok) return;
  float x[kAqRows][8];
  aq_load_tile<T>(X, n_tok, c_in, ldx, r0, c, x);
  for (int kb = 0; kb < nb; ++kb) {
    float iv[8];
    aq_load_inv(inv_table ? inv_table + (int64_t)(k0 + kb) * c_in : nullptr, c, c_in, iv);
#pragma unroll
    for (int r = 0; r < kAqRows; ++r) {
      float m = 0.0f;
#pragma unroll
      for (int j = 0; j < 8; ++j) m = fmaxf(m, fabsf(x[r][j] * iv[j]));
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
      if (lane == 0 && r0 + r < n_tok)
        atomicMax(amax_bits + (int64_t)kb * n_tok + r0 + r, __builtin_bit_cast(uint32_t, m));
    }
  }
}

// in place: amax bit pattern -> sigma; optional reciprocal table
__global__ void act_sigma_kernel(float* __restrict__ sig, int64_t n, float qa, float* __restrict__ rsig) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float sg = fmaxf(sig[i], kRangeFloor) / qa;   // the stored bits are the float maximum
  sig[i] = sg;
  if (rsig) rsig[i] = 1.0f / sg;
}

__global__ void fill_zero_u32_kernel(uint32_t* __restrict__ p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

template <typename T>
__global__ __launch_bounds__(256) void act_codes_kernel(const uint16_t* __restrict__ X, int64_t n_tok,
                                                        int64_t c_in, int64_t ldx,
                                                        const float* __restrict__ inv_table, int k0, int nb,
                                                        const float* __restrict__ sig,
                                                        const float* __restrict__ rsig, float qa,
                                                        uint16_t* __restrict__ codes) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c = (int64_t)blockIdx.x * kAqCols + lane * 8;
  const int64_t r0 = ((int64_t)blockIdx.y * 4 + wave) * kAqRows;
  if (r0 >= n_tok || c >= c_in) return;
  float x[kAqRows][8];
  aq_load_tile<T>(X, n_tok, c_in, ldx, r0, c, x);
  for (int kb = 0; kb < nb; ++kb) {
    float iv[8];
    aq_load_inv(inv_table ? inv_table + (int64_t)(k0 + kb) * c_in : nullptr, c, c_in, iv);
#pragma unroll
    for (int r = 0; r < kAqRows; ++r) {
      if (r0 + r >= n_tok) break;
      const float sg = sig[(int64_t)kb * n_tok + r0 + r];
      const float rs = rsig ? rsig[(int64_t)kb * n_tok + r0 + r] : 1.0f / sg;
      uint32_t o[4] = {0, 0, 0, 0};
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float q = rint_quotient(x[r][j] * iv[j], sg, rs);
        q = fminf(fmaxf(q, -qa - 1.0f), qa);
        o[j >> 1] |= (uint32_t)F16::from_float(q) << ((j & 1) * 16);
      }
      *reinterpret_cast<uint4*>(codes + ((int64_t)kb * n_tok + r0 + r) * c_in + c) = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
}

hipError_t launch_act_quant(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx, bool bf16,
                            const float* inv_table, int k0, int nb, int act_bits, void* codes,
                            float* sigma, float* rsigma, hipStream_t stream) {
  ProfScope ps("act_quant", stream, (double)n_tok * (double)c_in * (4.0 + 2.0 * nb));
  const float qa = (float)((1 << (act_bits - 1)) - 1);
  const uint16_t* x = (const uint16_t*)X;
  const int64_t n = (int64_t)nb * n_tok;
  dim3 grid((unsigned)ceil_div(c_in, kAqCols), (unsigned)ceil_div(n_tok, 4 * kAqRows));
  fill_zero_u32_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, stream>>>((uint32_t*)sigma, n);
  if (!bf16) act_amax_kernel<F16><<<grid, 256, 0, stream>>>(x, n_tok, c_in, ldx, inv_table, k0, nb, (uint32_t*)sigma);
  else act_amax_kernel<BF16><<<grid, 256, 0, stream>>>(x, n_tok, c_in, ldx, inv_table, k0, nb, (uint32_t*)sigma);
  act_sigma_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, stream>>>(sigma, n, qa, rsigma);
  if (!bf16) act_codes_kernel<F16><<<grid, 256, 0, stream>>>(x, n_tok, c_in, ldx, inv_table, k0, nb, sigma, rsigma, qa, (uint16_t*)codes);
  else act_codes_kernel<BF16><<<grid, 256, 0, stream>>>(x, n_tok, c_in, ldx, inv_table, k0, nb, sigma, rsigma, qa, (uint16_t*)codes);
  return hipGetLastError();
}

hipError_t launch_fake_quant(const QuantArgs& q, hipStream_t stream) {
  QuantDev d;
  d.W = (const uint16_t*)q.W; d.c_out = q.c_out; d.c_in = q.c_in; d.ldw = q.ldw;
  d.qmax = (float)((1 << q.bits) - 1);
  d.half = 1 << (q.bits - 1);
  d.qlo = -(float)d.half; d.qhi = (float)(d.half - 1);
  d.group = q.group == 0 ? (int)q.c_in : q.group;
  d.s_table = q.s_table; d.inv_table = q.inv_table; d.n_cand = q.n_cand;
  d.what = (uint16_t*)q.what; d.what_cand_stride = q.what_cand_stride; d.what_f16 = q.what_f16;
  d.codes = q.codes; d.zp = q.zp; d.delta = q.delta; d.wdq = (uint16_t*)q.wdq; d.ld_dq = q.ld_dq;
  d.diff = q.diff; d.xmax_bits = q.xmax_bits; d.col_scale = q.col_scale;
  const bool pow2 = d.group >= 8 && d.group <= 512 && (d.group & (d.group - 1)) == 0;
  const double bytes = (double)q.c_out * (double)q.c_in * (2.0 + 2.0 * (q.what ? q.n_cand : 0) +
                                                           (q.codes ? 1.0 : 0.0) + (q.wdq ? 2.0 : 0.0));
  ProfScope ps("fake_quant", stream, bytes);
  const bool sym = q.symmetric != 0;
  if (pow2) {
    const int64_t waves = q.c_out * ceil_div(q.c_in, 512);
    const unsigned grid = (unsigned)ceil_div(waves, 4);
    const bool aux = q.codes || q.zp || q.delta || q.wdq;
    auto go = [&](auto kern) { kern<<<grid, 256, 0, stream>>>(d); };
    if (aux) {
      if (!q.bf16 && !sym) go(quant_pow2_kernel<F16, false, true>);
      else if (!q.bf16) go(quant_pow2_kernel<F16, true, true>);
      else if (!sym) go(quant_pow2_kernel<BF16, false, true>);
      else go(quant_pow2_kernel<BF16, true, true>);
    } else {
      if (!q.bf16 && !sym) go(quant_pow2_kernel<F16, false, false>);
      else if (!q.bf16) go(quant_pow2_kernel<F16, true, false>);
      else if (!sym) go(quant_pow2_kernel<BF16, false, false>);
      else go(quant_pow2_kernel<BF16, true, false>);
    }
  } else {
    const int64_t waves = q.c_out * (q.c_in / d.group);
    const unsigned grid = (unsigned)ceil_div(waves, 4);
    if (!q.bf16 && !sym) quant_any_kernel<F16, false><<<grid, 256, 0, stream>>>(d);
    else if (!q.bf16) quant_any_kernel<F16, true><<<grid, 256, 0, stream>>>(d);
    else if (!sym) quant_any_kernel<BF16, false><<<grid, 256, 0, stream>>>(d);
    else quant_any_kernel<BF16, true><<<grid, 256, 0, stream>>>(d);
  }
  return hipGetLastError();
}

// Wout[o,c] = round16(Win[o,c] * inv_s[c]); dense output, row stride c_in.
template <typename T, typename TO>
__global__ __launch_bounds__(256) void fold_scale_kernel(const uint16_t* __restrict__ Win,
                                                         int64_t c_out, int64_t c_in, int64_t ldw,
                                                         const float* __restrict__ inv_s,
                                                         const uint32_t* __restrict__ xmax_bits,
                                                         uint16_t* __restrict__ Wout) {
  const int64_t chunks = c_in / 8;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= c_out * chunks) return;
  const int64_t row = i / chunks, c = (i % chunks) * 8;
  const uint4 v = *reinterpret_cast<const uint4*>(Win + row * ldw + c);
  const uint32_t u[4] = {v.x, v.y, v.z, v.w};
  uint32_t o[4] = {0, 0, 0, 0};
  const float up = xmax_bits
      ? __builtin_bit_cast(float, (uint32_t)(127 + shift_from_bf16_bits(*xmax_bits)) << 23) : 1.0f;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float f = T::to_float((uint16_t)(u[j >> 1] >> ((j & 1) * 16))) * (inv_s ? inv_s[c + j] : 1.0f);
    o[j >> 1] |= (uint32_t)TO::from_float(f * up) << ((j & 1) * 16);
  }
  *reinterpret_cast<uint4*>(Wout + row * c_in + c) = make_uint4(o[0], o[1], o[2], o[3]);
}

hipError_t launch_fold_scale(const void* Win, int64_t c_out, int64_t c_in, int64_t ldw, bool bf16,
                             const float* inv_s, const uint32_t* xmax_bits, bool out_f16, void* Wout,
                             hipStream_t stream) {
  ProfScope ps("fold_scale", stream, 4.0 * (double)c_out * (double)c_in);
  const unsigned grid = (unsigned)ceil_div(c_out * (c_in / 8), 256);
  const uint16_t* in = (const uint16_t*)Win;
  uint16_t* out = (uint16_t*)Wout;
  if (!bf16) fold_scale_kernel<F16, F16><<<grid, 256, 0, stream>>>(in, c_out, c_in, ldw, inv_s, xmax_bits, out);
  else if (out_f16) fold_scale_kernel<BF16, F16><<<grid, 256, 0, stream>>>(in, c_out, c_in, ldw, inv_s, xmax_bits, out);
  else fold_scale_kernel<BF16, BF16><<<grid, 256, 0, stream>>>(in, c_out, c_in, ldw, inv_s, xmax_bits, out);
  return hipGetLastError();
}

}  // namespace tlq
