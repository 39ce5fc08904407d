// Loads from global memory straight into LDS, the waits that go with them (the compiler does
// not track such loads), and a barrier that orders LDS traffic only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wino {

#if defined(__HIPCC__)

// One wavefront load of 1 KB from global memory straight into LDS: lane l's 16 bytes
// (base + lane_off) land at LDS byte address lds_byte + 16 l.
__device__ __forceinline__ void dma_1k(uint32_t lds_byte, const void* base, uint32_t lane_off) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_byte), "v"(lane_off), "s"(base)
      : "memory");
}

// (the compiler knows nothing of those loads: their completion is waited for by hand)
template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  // gfx9 encoding: vmcnt low bits [3:0], high bits [15:14]; expcnt [6:4] and lgkmcnt [11:8]
  // left at their maxima (no wait)
  constexpr int imm = (N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8);
  __builtin_amdgcn_s_waitcnt(imm);
  asm volatile("" ::: "memory");
}
// ... at most `chunks` * LPW loads outstanding, chunks (uniform) in 0 .. MAXC
template <int LPW, int MAXC>
__device__ __forceinline__ void wait_vm_chunks(int chunks) {
  if constexpr (MAXC == 0) {
    wait_vm<0>();
  } else {
    if (chunks >= MAXC) wait_vm<MAXC * LPW>();
    else wait_vm_chunks<LPW, MAXC - 1>(chunks);
  }
}

__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

#endif  // __HIPCC__

}  // namespace wino
