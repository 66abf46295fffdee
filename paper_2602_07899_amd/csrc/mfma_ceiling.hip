// Register-only fp16 MFMA loop: what the chip sustains on its matrix cores when
// nothing but MFMAs issue, (a) 32x32x16 with constant operands, (b) 32x32x16 and
// (c) 16x16x32 with pseudo-random operands whose bit patterns toggle like real
// activations and weights.  (b) and (c) are the practical ceilings for an fp16
// contraction on this device: the matrix cores are power-limited well below the
// nominal peak when the operands carry real data, and the shader clock (read from
// the ratio of the shader cycle counter to the constant 100 MHz counter) drops
// accordingly.  The 16x16x32 shape reads and writes half the accumulator registers
// per flop and sustains about 16 % more.  Prints one JSON line.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <vector>

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

template <int RANDOM>
__global__ __launch_bounds__(512) void mfma_loop(float* out, long long* clk, int iters) {
  f16x8 a[8], b[8];
  unsigned s = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  for (int n = 0; n < 8; ++n)
    for (int i = 0; i < 8; ++i) {
      s = s * 1664525u + 1013904223u;
      a[n][i] = (_Float16)(RANDOM ? ((int)(s >> 8) % 2001 - 1000) * 0.001f : 0.5f);
      s = s * 1664525u + 1013904223u;
      b[n][i] = (_Float16)(RANDOM ? ((int)(s >> 8) % 2001 - 1000) * 0.00002f : 0.01f);
    }
  float t = 0;
  const long long c0 = clock64(), w0 = wall_clock64();
  if (RANDOM < 2) {
    f32x16 acc[8];
    for (int n = 0; n < 8; ++n)
      for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
    for (int it = 0; it < iters / 8; ++it) {
#pragma unroll
      for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int n = 0; n < 8; ++n)
          acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[n], b[(n + r) & 7], acc[n], 0, 0, 0);
    }
    for (int n = 0; n < 8; ++n) t += acc[n][0] + acc[n][7];
  } else {   // same flops per iteration: 16 MFMAs of 16x16x32 for 8 of 32x32x16
    f32x4 acc[32];
    for (int n = 0; n < 32; ++n)
      for (int v = 0; v < 4; ++v) acc[n][v] = 0.f;
    for (int it = 0; it < iters / 16; ++it) {
#pragma unroll
      for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int n = 0; n < 32; ++n)
          acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[n & 7], b[(n + r + (n >> 3)) & 7], acc[n], 0, 0, 0);
    }
    for (int n = 0; n < 32; ++n) t += acc[n][0] + acc[n][3];
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  out[blockIdx.x * blockDim.x + threadIdx.x] = t;
  if (threadIdx.x == 0) {
    clk[blockIdx.x * 2] = c1 - c0;
    clk[blockIdx.x * 2 + 1] = w1 - w0;
  }
}

template <int RANDOM>
static bool run(float* out, long long* clk, double* tflops, double* ghz) {
  const int blocks = 256 * 4, threads = 512, iters = 4000, reps = 24;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return false;
  double best = 0, clock = 0;
  for (int rep = 0; rep < reps; ++rep) {  // the clock settles after a few launches
    if (hipEventRecord(e0) != hipSuccess) return false;
    mfma_loop<RANDOM><<<blocks, threads>>>(out, clk, iters);
    if (hipEventRecord(e1) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) return false;
    float ms = 0;
    if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return false;
    if (rep < reps - 8) continue;  // average the last eight launches
    const double flops = 2.0 * 32 * 32 * 16 * 8.0 * iters * (threads / 64) * blocks;
    std::vector<long long> h(blocks * 2);
    if (hipMemcpy(h.data(), clk, blocks * 16, hipMemcpyDeviceToHost) != hipSuccess) return false;
    double sc = 0, wc = 0;
    for (int i = 0; i < blocks; ++i) { sc += (double)h[2 * i]; wc += (double)h[2 * i + 1]; }
    best += flops / ms / 1e9 / 8.0;
    clock += sc / wc * 0.1 / 8.0;  // shader cycles per 100 MHz tick -> GHz
  }
  *tflops = best;
  *ghz = clock;
  return true;
}

int main() {
  float* out = nullptr;
  long long* clk = nullptr;
  if (hipMalloc(&out, 1024 * 512 * 4) != hipSuccess || hipMalloc(&clk, 1024 * 16) != hipSuccess) {
    fprintf(stderr, "mfma_ceiling: no device memory\n");
    return 1;
  }
  double t0, g0, t1, g1, t2, g2;
  if (!run<0>(out, clk, &t0, &g0) || !run<1>(out, clk, &t1, &g1) || !run<2>(out, clk, &t2, &g2)) {
    fprintf(stderr, "mfma_ceiling: HIP error\n");
    return 1;
  }
  printf("{\"constant_operands\": {\"tflops\": %.1f, \"shader_clock_ghz\": %.3f}, "
         "\"random_operands\": {\"tflops\": %.1f, \"shader_clock_ghz\": %.3f}, "
         "\"random_operands_16x16x32\": {\"tflops\": %.1f, \"shader_clock_ghz\": %.3f}}\n", t0, g0, t1, g1, t2, g2);
  return hipDeviceSynchronize() == hipSuccess ? 0 : 1;
}
