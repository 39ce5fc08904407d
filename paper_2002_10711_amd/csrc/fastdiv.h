// Division by a run-time constant as one multiply-high: the host stores
// inv(d) = ceil(2^32 / d) (0 stands for d == 1) in the launch plan; the quotient is exact
// whenever numerator * d < 2^32, which the host checks for every use.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wino {

__host__ __device__ inline uint32_t make_inv(uint32_t d) {
  return d <= 1 ? 0u : (uint32_t)((0x100000000ull + d - 1) / d);
}

#if defined(__HIPCC__)
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t inv) {
  return __umulhi(n, inv) + (inv ? 0u : n);           // branch-free: inv == 0 means d == 1
}
#endif

}  // namespace wino
