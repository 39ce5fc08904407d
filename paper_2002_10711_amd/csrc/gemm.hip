// Hadamard stage of Eq. 1 summed over input channels, written as one GEMM per
// Winograd position (the GEMM formulation of Winograd convolutions, paper Sec. 5.3):
//
//     M[p][t][k] = sum_c A[p][t][c] * B[p][k][c]
//
// Both operands are channel-contiguous, which is the operand order the gfx950
// matrix cores want: a lane of v_mfma_i32_16x16x64_i8 supplies 16 consecutive bytes
// of the reduction axis for one row (v_mfma_f32_16x16x4_f32: 4 consecutive floats,
// fed one at a time).  int8 x int8 -> int32 is exact; the float variant accumulates
// in fp32.  This stand-alone GEMM (M goes to memory) serves the layers whose
// accumulators do not fit the fused kernels, the per-stage calls and parity taps, and
// the im2row baseline with P = 1 and a reduction length of 9*C.
//
// Tiling: workgroup = 2 x 2 wavefronts; a wavefront owns WT x WK MFMA tiles of
// 16 x 16, so the block is (32 WT) tiles x (32 WK) output channels.  The reduction
// runs in steps of 64 bytes per row: the block's A rows and B rows of a step are
// copied to LDS once (16 bytes per thread and row piece, double buffered, the next
// step's global loads in flight during the MFMAs) and every wave reads its
// operands from there with 16-byte LDS reads, each reused WK (resp. WT) times from
// registers.  The weights are the MFMA "A" operand (rows = k) and the activations
// the "B" operand (columns = t), so a lane ends up with four consecutive k of one
// tile and stores 16 bytes at once.  Whatever order the instruction assigns to the
// reduction elements inside a lane group, it is the same for both operands.
#include "wino_internal.h"

namespace wino {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

template <bool I8> struct AccT { typedef v4i type; };
template <> struct AccT<false> { typedef v4f type; };

// kBlockedB: B is in the block layout of u_byte_index (1 KB blocks of 16 rows x 64
// bytes, piece (16-byte segment seg, row kr) at piece index seg*16 + kr): a thread's
// pieces are then taken in block order, so the global reads stay contiguous, and are put
// into the same LDS places as in the plain layout.
template <int WT, int WK, bool I8, bool kBlockedB = false>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(const char* __restrict__ A,
                                                         const char* __restrict__ B,
                                                         char* __restrict__ M, int Tp, int Kp,
                                                         int row_bytes) {
  constexpr int BT = 32 * WT, BK = 32 * WK;            // block tile
  constexpr int LA = BT * 4 / 256, LB = BK * 4 / 256;  // 16-byte pieces per thread and step
  typedef typename AccT<I8>::type acc_t;
  __shared__ __attribute__((aligned(16))) char As[2][BT * 64];
  __shared__ __attribute__((aligned(16))) char Bs[2][BK * 64];
  const int p = blockIdx.z, tb = blockIdx.x * BT, kb = blockIdx.y * BK;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, grp = lane >> 4;
  const int wt = wave >> 1, wk = wave & 1;             // position of the wave in the block
  const char* Ag = A + ((size_t)p * Tp + tb) * row_bytes;
  const char* Bg = B + ((size_t)p * Kp + kb) * row_bytes;
  const int nstep = row_bytes >> 6;
  // piece q of the block's B tile at reduction step st: where it comes from, where it goes
  auto b_src = [&](int q, int st) -> const char* {
    if constexpr (kBlockedB)
      return Bg + ((size_t)(q >> 6) * nstep + st) * 1024 + (q & 63) * 16;   // block q/64 of 16 rows
    else
      return Bg + (size_t)(q >> 2) * row_bytes + (size_t)st * 64 + (q & 3) * 16;
  };
  auto b_dst = [&](int q) -> int {
    if constexpr (kBlockedB)
      return (((q >> 6) * 16 + (q & 15)) * 4 + ((q >> 4) & 3)) * 16;        // row, segment
    else
      return q * 16;
  };

  acc_t acc[WT][WK];
#pragma unroll
  for (int i = 0; i < WT; ++i)
#pragma unroll
    for (int j = 0; j < WK; ++j) acc[i][j] = acc_t{0, 0, 0, 0};

  // piece q of a tile: row q / 4, bytes (q % 4) * 16 .. + 15 of the step
  v4i ra[LA], rb[LB];
#pragma unroll
  for (int u = 0; u < LA; ++u) {
    const int q = tid + u * 256;
    ra[u] = *(const v4i*)(Ag + (size_t)(q >> 2) * row_bytes + (q & 3) * 16);
  }
#pragma unroll
  for (int u = 0; u < LB; ++u) rb[u] = *(const v4i*)b_src(tid + u * 256, 0);
#pragma unroll
  for (int u = 0; u < LA; ++u) *(v4i*)(As[0] + (tid + u * 256) * 16) = ra[u];
#pragma unroll
  for (int u = 0; u < LB; ++u) *(v4i*)(Bs[0] + b_dst(tid + u * 256)) = rb[u];
  __syncthreads();

  for (int st = 0; st < nstep; ++st) {
    const int cur = st & 1;
    const bool more = st + 1 < nstep;
    if (more) {
      const size_t co = (size_t)(st + 1) * 64;
#pragma unroll
      for (int u = 0; u < LA; ++u) {
        const int q = tid + u * 256;
        ra[u] = *(const v4i*)(Ag + (size_t)(q >> 2) * row_bytes + co + (q & 3) * 16);
      }
#pragma unroll
      for (int u = 0; u < LB; ++u) rb[u] = *(const v4i*)b_src(tid + u * 256, st + 1);
    }
    acc_t va[WT], vb[WK];
#pragma unroll
    for (int i = 0; i < WT; ++i)
      va[i] = *(const acc_t*)(As[cur] + ((wt * WT + i) * 16 + r) * 64 + grp * 16);
#pragma unroll
    for (int j = 0; j < WK; ++j)
      vb[j] = *(const acc_t*)(Bs[cur] + ((wk * WK + j) * 16 + r) * 64 + grp * 16);
#pragma unroll
    for (int i = 0; i < WT; ++i)
#pragma unroll
      for (int j = 0; j < WK; ++j) {
        if constexpr (I8) {
          acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(vb[j], va[i], acc[i][j], 0, 0, 0);
        } else {
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(vb[j].x, va[i].x, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(vb[j].y, va[i].y, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(vb[j].z, va[i].z, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(vb[j].w, va[i].w, acc[i][j], 0, 0, 0);
        }
      }
    if (more) {
#pragma unroll
      for (int u = 0; u < LA; ++u) *(v4i*)(As[cur ^ 1] + (tid + u * 256) * 16) = ra[u];
#pragma unroll
      for (int u = 0; u < LB; ++u) *(v4i*)(Bs[cur ^ 1] + b_dst(tid + u * 256)) = rb[u];
    }
    __syncthreads();
  }

  // lane holds, per tile (i, j): t = tb + (wt*WT + i)*16 + r, k = kb + (wk*WK + j)*16 + grp*4 .. +3
#pragma unroll
  for (int i = 0; i < WT; ++i) {
    const int t = tb + (wt * WT + i) * 16 + r;
    char* mrow = M + (((size_t)p * Tp + t) * Kp + kb + wk * WK * 16 + grp * 4) * 4;
#pragma unroll
    for (int j = 0; j < WK; ++j) *(acc_t*)(mrow + j * 64) = acc[i][j];
  }
}

}  // namespace

hipError_t launch_gemm(int P, int Tp, int Kp, int Cp, int i8, int b_blocked, const void* A,
                       const void* B, void* M, hipStream_t s) {
  // Tp, Kp are multiples of 64; Cp of 64 (int8) or 16 (float): the host API rounds them.
  if (Tp % 64 || Kp % 64 || Cp % (i8 ? 64 : 16) || P < 1 || P > 65535)
    return hipErrorInvalidValue;
  const int row_bytes = Cp * (i8 ? 1 : 4);
  const char* a = (const char*)A;
  const char* b = (const char*)B;
  char* m = (char*)M;
  // 128 x 128 blocks when both extents allow it and the grid still fills the chip
  const bool big = Tp % 128 == 0 && Kp % 128 == 0 && (long long)(Tp / 128) * (Kp / 128) * P >= 512;
  if (big) {
    if (Kp / 128 > 65535) return hipErrorInvalidValue;
    dim3 grid(Tp / 128, Kp / 128, P);
    if (i8 && b_blocked)
      gemm_tiled_kernel<4, 4, true, true><<<grid, 256, 0, s>>>(a, b, m, Tp, Kp, row_bytes);
    else if (i8)
      gemm_tiled_kernel<4, 4, true><<<grid, 256, 0, s>>>(a, b, m, Tp, Kp, row_bytes);
    else if (b_blocked)
      gemm_tiled_kernel<4, 4, false, true><<<grid, 256, 0, s>>>(a, b, m, Tp, Kp, row_bytes);
    else
      gemm_tiled_kernel<4, 4, false><<<grid, 256, 0, s>>>(a, b, m, Tp, Kp, row_bytes);
  } else {
    if (Kp / 64 > 65535) return hipErrorInvalidValue;
    dim3 grid(Tp / 64, Kp / 64, P);
    if (i8 && b_blocked)
      gemm_tiled_kernel<2, 2, true, true><<<grid, 256, 0, s>>>(a, b, m, Tp, Kp, row_bytes);
    else if (i8)
      gemm_tiled_kernel<2, 2, true><<<grid, 256, 0, s>>>(a, b, m, Tp, Kp, row_bytes);
    else if (b_blocked)
      gemm_tiled_kernel<2, 2, false, true><<<grid, 256, 0, s>>>(a, b, m, Tp, Kp, row_bytes);
    else
      gemm_tiled_kernel<2, 2, false><<<grid, 256, 0, s>>>(a, b, m, Tp, Kp, row_bytes);
  }
  return hipGetLastError();
}

}  // namespace wino
