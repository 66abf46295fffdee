// Entry point for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc): tlq_x_stat with its
// partial sums kept in a fixed device array of this library instead of a caller
// workspace.  Nothing here allocates or frees device or host memory.
#include <mutex>

#include "common.h"

using namespace tlq;

namespace {

// 128 row chunks (the most launch_xstat ever uses) x TLQ_X_STAT_STATIC_MAX_C_IN channels
// of double partial sums: 16 MiB on every GPU the library runs on, held until the
// process ends.
constexpr size_t kScratchDoubles = (size_t)128 * TLQ_X_STAT_STATIC_MAX_C_IN;
static __device__ __align__(256) double scratch[kScratchDoubles];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
double* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU

// The array's name is only a host-side handle; the address a kernel can use comes from
// hipGetSymbolAddress, once per device, with that device current.
tlq_status scratch_for_current_device(double** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TLQ_ERR_LAUNCH;
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TLQ_ERR_LAUNCH;
    g_scratch_ptr[dev] = (double*)p;
  }
  *out = g_scratch_ptr[dev];
  return TLQ_OK;
}

}  // namespace

extern "C" tlq_status tlq_x_stat_static(const void* X, int64_t n_tok, int64_t c_in, int64_t ldx,
                                        const tlq_params* p, float* x_stat, void* stream) {
  if (!X || !x_stat || !p) return TLQ_ERR_NULL;
  if (p->struct_size != sizeof(tlq_params)) return TLQ_ERR_UNSUPPORTED;
  if (p->xstat_kind != 0 && p->xstat_kind != 1) return TLQ_ERR_UNSUPPORTED;
  if (p->x_dtype != TLQ_F16 && p->x_dtype != TLQ_BF16) return TLQ_ERR_UNSUPPORTED;
  if (n_tok <= 0 || c_in <= 0 || ldx < c_in || n_tok >= (1LL << 31) || (c_in % 8) != 0) return TLQ_ERR_SHAPE;
  if (c_in > TLQ_X_STAT_STATIC_MAX_C_IN) return TLQ_ERR_WORKSPACE;   // beyond the fixed scratch
  if (((uintptr_t)X % 16) != 0 || (ldx % 8) != 0) return TLQ_ERR_ALIGN;
  if (tlq_profile_enabled()) return TLQ_ERR_UNSUPPORTED;            // timing creates HIP events
  if ((size_t)xstat_chunks(n_tok) * (size_t)c_in > kScratchDoubles) return TLQ_ERR_WORKSPACE;
  double* partial = nullptr;
  const tlq_status st = scratch_for_current_device(&partial);
  if (st != TLQ_OK) return st;
  // every partial entry that xstat_final reads is written by xstat_partial in the same
  // call, so the array needs no clearing between calls
  return launch_xstat(X, n_tok, c_in, ldx, p->x_dtype == TLQ_BF16, p->xstat_kind, partial, x_stat,
                      (hipStream_t)stream) == hipSuccess ? TLQ_OK : TLQ_ERR_LAUNCH;
}
