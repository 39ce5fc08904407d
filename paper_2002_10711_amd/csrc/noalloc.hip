// wino_conv2d_fwd_noalloc: the forward for callers that cannot allocate device memory (HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  The workspace of
// wino_conv2d_fwd -- the transformed input V and, for the three-kernel sequence, the
// Hadamard/GEMM result M -- lives in a buffer that is part of the library's device image
// instead of coming from the caller.
#include <mutex>

#include "wino_internal.h"

namespace {

// One copy per GPU the library is loaded on, held until the process ends.
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[WINO_NOALLOC_SCRATCH_BYTES];

// The name `scratch` is a host-side stand-in in host code, not a device address: each
// device's copy has its own address, looked up once with that device current.
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

hipError_t scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" wino_status wino_conv2d_fwd_noalloc(const wino_desc* d, const wino_quant* q,
                                               const void* x_dev, const void* U_dev,
                                               void* y_dev, void* stream) {
  // every argument check of wino_conv2d_fwd first, so that error paths never touch the
  // GPU; then the size against the built-in buffer
  wino::Geom g;
  const wino_status st = wino::fwd_check(d, q, x_dev, U_dev, y_dev, WINO_STAGE_ALL, &g);
  if (st != WINO_OK) return st;
  const size_t need = wino::fwd_workspace_touched(d);
  if (need > (size_t)WINO_NOALLOC_SCRATCH_BYTES) return WINO_E_SCRATCH_LIMIT;
  void* ws = nullptr;
  if (scratch_of_current_device(&ws) != hipSuccess) return WINO_E_HIP;
  // (the kernels never read workspace bytes that this call has not written: padding rows
  // and channels of V are written by the input stage, padding tiles only feed sums that
  // are dropped -- nothing has to be cleared between calls)
  return wino::fwd_stages(d, q, x_dev, U_dev, y_dev, ws, (size_t)WINO_NOALLOC_SCRATCH_BYTES,
                          WINO_STAGE_ALL, stream, true, wino::kSeqAuto);
}
