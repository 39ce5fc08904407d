// Matrix-core peak probe: a loop of independent MFMAs and nothing else, the measured
// counterpart of the datasheet peaks that the rooflines quote (int8 5 POP/s, fp32
// 157.3 TFLOP/s dense).  Eight accumulator sets per wavefront keep the pipe full; operands
// never change, the sums are stored once so that nothing is optimised away.
#include "wino_internal.h"
#include "wino.h"

namespace wino {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

template <bool I8>
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, float* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  if constexpr (I8) {
    const v4i a = v4i{lane, lane + 1, lane + 2, lane + 3}, b = v4i{lane ^ 5, lane ^ 9, 1, 2};
    v4i acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = v4i{j, 0, 0, 0};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[j], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += acc[j].x + acc[j].y + acc[j].z + acc[j].w;
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = (float)s;
  } else {
    const float a = 1.0f + lane * 1e-3f, b = 1.0f - lane * 1e-3f;
    v4f acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = v4f{(float)j, 0.0f, 0.0f, 0.0f};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += acc[j].x + acc[j].y + acc[j].z + acc[j].w;
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
  }
}

// Vector-memory-path probe: every wavefront walks its own slice of a buffer with one load
// form and nothing else (eight loads in flight per wavefront), round and round: a slice
// that fits the L1 measures the L1, one that fits the XCD's L2 the L2 -> L1 path, a larger
// one whatever lies behind the L2.  kMode 0: 16 bytes per lane into registers, 1: 8 bytes,
// 2: 4 bytes, 3: 16 bytes per lane straight into LDS (global_load_lds_dwordx4).
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

template <int kMode, int kWaves>
__global__ __launch_bounds__(kWaves * 64) void load_loop_kernel(const char* __restrict__ buf,
                                                                size_t wg_bytes, int iters,
                                                                float* __restrict__ out) {
  __shared__ __attribute__((aligned(1024))) char lds[kWaves * 8 * 1024];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  constexpr int BPL = (kMode == 0 || kMode == 3) ? 16 : kMode == 1 ? 8 : 4;   // bytes per lane
  constexpr uint32_t chunk = 64 * BPL;                     // bytes per wavefront load
  const size_t wave_bytes = wg_bytes / kWaves;
  const char* base = buf + (size_t)blockIdx.x * wg_bytes + (size_t)wave * wave_bytes;
  const uint32_t nchunks = (uint32_t)(wave_bytes / chunk);
  uint32_t acc = 0, c = 0;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const uint32_t off = c * chunk + (uint32_t)lane * BPL;
      if constexpr (kMode == 0) {
        const v4u v = *(const v4u*)(base + off);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
      } else if constexpr (kMode == 1) {
        const v2u v = *(const v2u*)(base + off);
        acc ^= v.x ^ v.y;
      } else if constexpr (kMode == 2) {
        acc ^= *(const uint32_t*)(base + off);
      } else {
        const uint32_t ldsb =
            (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds + (uint32_t)(wave * 8 + u) * 1024u;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :
                     : "s"(ldsb), "v"(off), "s"(base)
                     : "memory");
      }
      c = c + 1 == nchunks ? 0 : c + 1;
    }
    if constexpr (kMode == 3) {
      // (the compiler does not track loads into LDS: all eight have landed before the next
      // round overwrites their slots; vmcnt = 0, the other counters left alone)
      __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));
      asm volatile("" ::: "memory");
    }
  }
  if constexpr (kMode == 3) acc = *(const uint32_t*)(lds + threadIdx.x * 4);
  out[(size_t)blockIdx.x * kWaves * 64 + threadIdx.x] = (float)acc;
}

template <int kMode>
hipError_t launch_load_loop(int waves, int workgroups, const char* buf, size_t wg_bytes, int iters,
                            float* out, hipStream_t s) {
  switch (waves) {
    case 4: load_loop_kernel<kMode, 4><<<workgroups, 256, 0, s>>>(buf, wg_bytes, iters, out); break;
    case 8: load_loop_kernel<kMode, 8><<<workgroups, 512, 0, s>>>(buf, wg_bytes, iters, out); break;
    default: load_loop_kernel<kMode, 16><<<workgroups, 1024, 0, s>>>(buf, wg_bytes, iters, out); break;
  }
  return hipGetLastError();
}

}  // namespace
}  // namespace wino

extern "C" wino_status wino_debug_load_loop(int mode, int waves, int workgroups,
                                            size_t workgroup_bytes, int iters,
                                            const void* buf_dev, float* out_dev,
                                            double* bytes_per_launch, void* stream) {
  if (!buf_dev || !out_dev) return WINO_E_NULL;
  if (mode < 0 || mode > 3 || (waves != 4 && waves != 8 && waves != 16)) return WINO_E_BAD_ARG;
  // (a wavefront's slice: whole 1 KB chunks, at least one, 32-bit offsets)
  if (workgroups < 1 || workgroups > 65535 || iters < 1 || workgroup_bytes % ((size_t)waves * 1024) != 0 ||
      workgroup_bytes < (size_t)waves * 1024 || workgroup_bytes / waves >= (1ull << 31))
    return WINO_E_BAD_SHAPE;
  const int bpl = (mode == 0 || mode == 3) ? 16 : mode == 1 ? 8 : 4;
  if (bytes_per_launch) *bytes_per_launch = (double)workgroups * waves * 64.0 * bpl * 8.0 * iters;
  hipStream_t s = (hipStream_t)stream;
  const char* b = (const char*)buf_dev;
  hipError_t e;
  switch (mode) {
    case 0: e = wino::launch_load_loop<0>(waves, workgroups, b, workgroup_bytes, iters, out_dev, s); break;
    case 1: e = wino::launch_load_loop<1>(waves, workgroups, b, workgroup_bytes, iters, out_dev, s); break;
    case 2: e = wino::launch_load_loop<2>(waves, workgroups, b, workgroup_bytes, iters, out_dev, s); break;
    default: e = wino::launch_load_loop<3>(waves, workgroups, b, workgroup_bytes, iters, out_dev, s); break;
  }
  return e == hipSuccess ? WINO_OK : WINO_E_HIP;
}

extern "C" wino_status wino_debug_mfma_loop(int dtype, int workgroups, int iters,
                                            float* out_dev, double* ops_per_launch,
                                            void* stream) {
  if (!out_dev) return WINO_E_NULL;
  if (workgroups < 1 || workgroups > 65535 || iters < 1) return WINO_E_BAD_SHAPE;
  if (dtype != WINO_I8 && dtype != WINO_F32) return WINO_E_BAD_DTYPE;
  hipStream_t s = (hipStream_t)stream;
  const double per_mfma = dtype == WINO_I8 ? 2.0 * 16 * 16 * 64 : 2.0 * 16 * 16 * 4;
  if (ops_per_launch) *ops_per_launch = per_mfma * 8.0 * iters * 4.0 * workgroups;
  if (dtype == WINO_I8)
    wino::mfma_loop_kernel<true><<<workgroups, 256, 0, s>>>(iters, out_dev);
  else
    wino::mfma_loop_kernel<false><<<workgroups, 256, 0, s>>>(iters, out_dev);
  return hipGetLastError() == hipSuccess ? WINO_OK : WINO_E_HIP;
}
