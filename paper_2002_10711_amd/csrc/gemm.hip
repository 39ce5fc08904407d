// Hadamard stage of Eq. 1 summed over input channels, written as one GEMM per
// Winograd position (paper, Sec. 5.3: "Winograd convolutions using GEMMs"):
//
//     M[p][t][k] = sum_c A[p][t][c] * B[p][k][c]
//
// Both operands are channel-contiguous, which is the operand order the gfx950
// matrix cores want: a lane of v_mfma_i32_16x16x64_i8 supplies 16 consecutive
// bytes of the reduction axis for one row.  int8 x int8 -> int32 is exact;
// the float variant accumulates in fp32.  The same kernels serve the im2row
// baseline with P = 1 and a reduction length of 9*C.
#include "wino_internal.h"

namespace wino {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

// Block = 4 wavefronts = 64 tiles x 64 output channels of one position.
// Wave w owns tiles [16w, 16w+16) and four 16x16 MFMA accumulators along k.
// The weights are the MFMA "A" operand (rows = k) and the activations the "B"
// operand (columns = t), so a lane ends up with four consecutive k of one tile
// and stores 16 bytes at once.  Whatever order the instruction assigns to the 64
// reduction elements inside a lane group, it is the same for both operands, so
// the sum is over matching channels.
__global__ __launch_bounds__(256) void gemm_i8_kernel(const int8_t* __restrict__ A,
                                                      const int8_t* __restrict__ B,
                                                      int32_t* __restrict__ M, int Tp, int Kp,
                                                      int Cp) {
  const int p = blockIdx.z, tb = blockIdx.x * 64, kb = blockIdx.y * 64;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 15, grp = lane >> 4;
  const int t = tb + wave * 16 + r;
  const int8_t* vrow = A + ((size_t)p * Tp + t) * Cp + grp * 16;
  const int8_t* urow = B + ((size_t)p * Kp + kb + r) * Cp + grp * 16;
  v4i acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) acc[j] = (v4i){0, 0, 0, 0};
  for (int c0 = 0; c0 < Cp; c0 += 64) {
    const v4i bv = *(const v4i*)(vrow + c0);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const v4i au = *(const v4i*)(urow + (size_t)j * 16 * Cp + c0);
      acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(au, bv, acc[j], 0, 0, 0);
    }
  }
  int32_t* mrow = M + ((size_t)p * Tp + t) * Kp + kb + grp * 4;
#pragma unroll
  for (int j = 0; j < 4; ++j) *(v4i*)(mrow + j * 16) = acc[j];
}

// Same blocking with v_mfma_f32_16x16x4_f32: a lane loads four consecutive
// channels and feeds them to four MFMA steps; the step order permutes the
// channels inside a chunk of 16, identically for both operands.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A,
                                                       const float* __restrict__ B,
                                                       float* __restrict__ M, int Tp, int Kp,
                                                       int Cp) {
  const int p = blockIdx.z, tb = blockIdx.x * 64, kb = blockIdx.y * 64;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 15, grp = lane >> 4;
  const int t = tb + wave * 16 + r;
  const float* vrow = A + ((size_t)p * Tp + t) * Cp + grp * 4;
  const float* urow = B + ((size_t)p * Kp + kb + r) * Cp + grp * 4;
  v4f acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) acc[j] = (v4f){0.f, 0.f, 0.f, 0.f};
  for (int c0 = 0; c0 < Cp; c0 += 16) {
    const v4f bv = *(const v4f*)(vrow + c0);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const v4f au = *(const v4f*)(urow + (size_t)j * 16 * Cp + c0);
      acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(au.x, bv.x, acc[j], 0, 0, 0);
      acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(au.y, bv.y, acc[j], 0, 0, 0);
      acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(au.z, bv.z, acc[j], 0, 0, 0);
      acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(au.w, bv.w, acc[j], 0, 0, 0);
    }
  }
  float* mrow = M + ((size_t)p * Tp + t) * Kp + kb + grp * 4;
#pragma unroll
  for (int j = 0; j < 4; ++j) *(v4f*)(mrow + j * 16) = acc[j];
}

}  // namespace

hipError_t launch_gemm(int P, int Tp, int Kp, int Cp, int i8, const void* A, const void* B, void* M,
                       hipStream_t s) {
  // Tp, Kp are multiples of 64; Cp of 64 (int8) or 16 (float): the host API rounds them.
  if (Tp % 64 || Kp % 64 || Cp % (i8 ? 64 : 16) || P < 1 || P > 65535 || Kp / 64 > 65535)
    return hipErrorInvalidValue;
  dim3 grid(Tp / 64, Kp / 64, P);
  if (i8)
    gemm_i8_kernel<<<grid, 256, 0, s>>>((const int8_t*)A, (const int8_t*)B, (int32_t*)M, Tp, Kp,
                                        Cp);
  else
    gemm_f32_kernel<<<grid, 256, 0, s>>>((const float*)A, (const float*)B, (float*)M, Tp, Kp, Cp);
  return hipGetLastError();
}

}  // namespace wino
