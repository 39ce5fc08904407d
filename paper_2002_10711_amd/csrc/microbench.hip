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

}  // namespace
}  // namespace wino

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
