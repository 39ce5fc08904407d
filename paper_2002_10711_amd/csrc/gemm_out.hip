// Hadamard/GEMM stage fused with the output transform (Eq. 1, Sec. 3.1; GEMM
// formulation of Sec. 5.3): a wavefront keeps the accumulators of ALL n*n Winograd
// positions of a 16-tile x 16-channel block in registers, so M never travels
// through memory -- the int32 M tensor is 4x the size of everything else the layer
// moves and is what makes the separate kernels bandwidth-bound.
//
//     M[p][t][k] = sum_c V[p][t][c] * U[p][k][c]      (MFMA, exact in int8 mode)
//     Yt         = A^T M[., t, k] A                   (lane-local, fp32 chains)
//     y          = sat(rne(Yt * r_y))  -> NCHW
//
// Every position uses the same MFMA lane mapping (lane = (tile t, 4 consecutive
// k)), so after the last position a lane holds the complete n x n matrix M[., t, k]
// of four (t, k) pairs and transforms them without any exchange.
#include "output_stage.h"

namespace wino {
namespace {

// Workgroup = 4 wavefronts = 16 tiles x 64 output channels; wave w owns channels
// [16w, 16w+16) of the block, so the four waves read the same V rows (served by
// the L1) and different U rows.  Operands go straight from global memory / L2 into
// the MFMA: a lane loads 16 bytes of the reduction axis of one row, which is the
// operand layout of v_mfma_i32_16x16x64_i8 (int8, 64 channels per instruction) and,
// taken one float at a time, of v_mfma_f32_16x16x4_f32.  The weights are the "A"
// operand (rows = k) and the activations the "B" operand (columns = t).
template <int M, bool I8, bool kSparse, bool kMQ>
__global__ __launch_bounds__(256) void gemm_out_kernel(Geom g, MatAT at,
                                                       const void* __restrict__ Vv,
                                                       const void* __restrict__ Uv,
                                                       void* __restrict__ yv, float r_m, float r_y,
                                                       float qmax) {
  constexpr int n = M + 2, P = n * n;
  constexpr int ESZ = I8 ? 1 : 4;           // bytes per element
  constexpr int CHUNK = I8 ? 64 : 16;       // reduction elements per load step
  typedef typename Acc<I8>::type acc_t;
  const int tb = blockIdx.x * 16, kb = blockIdx.y * 64;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 15, grp = lane >> 4;
  const int t = tb + r;
  // Addresses = uniform 64-bit base (position, channel chunk: scalar registers) + a
  // 32-bit per-lane offset (row, lane group): no per-position 64-bit vector pointers,
  // which would not fit next to n*n accumulator sets.  The host checks the 32-bit range.
  const size_t vp = (size_t)g.Tp * g.Cp * ESZ, up = (size_t)g.Kp * g.Cp * ESZ;
  const uint32_t voff = (uint32_t)t * (uint32_t)(g.Cp * ESZ) + (uint32_t)grp * 16u;
  // (the weights are in the blocked layout of u_byte_index: the wavefront's 16 channels x
  // 64 bytes of a chunk are 1 KB of consecutive bytes, this lane's piece at grp*16 + r)
  const uint32_t uoff = (uint32_t)((kb + wave * 16) >> 4) * (uint32_t)((g.Cp * ESZ) >> 6) * 1024u +
                        (uint32_t)(grp * 16 + r) * 16u;
  constexpr int kUChunk = 1024;                        // bytes from one chunk of U to the next
  const char* vrow = (const char*)Vv;
  const char* urow = (const char*)Uv;
  const int nchunk = g.Cp / CHUNK;

  // Operand stream: step (ch, p) needs 16 bytes of V and 16 bytes of U per lane.  With
  // one or two wavefronts per SIMD nothing else hides the load latency, so the loads
  // run kDepth steps ahead of the MFMAs in a register ring (kDepth divides P, so ring
  // slot p % kDepth is the same in every pass over the channels).
  constexpr int kDepth = M == 4 ? 9 : 8;
  static_assert(P % kDepth == 0, "ring depth must divide the number of positions");
  typedef typename Acc<I8>::type op_t;      // 16 bytes either way
  op_t bufV[kDepth], bufU[kDepth];
#pragma unroll
  for (int p = 0; p < kDepth; ++p) {
    bufV[p] = *(const op_t*)(vrow + p * vp + voff);
    bufU[p] = *(const op_t*)(urow + p * up + uoff);
  }
  static_assert(CHUNK * ESZ == 64, "V advances 64 bytes per chunk");
  acc_t acc[P];
#pragma unroll
  for (int p = 0; p < P; ++p) acc[p] = acc_t{0, 0, 0, 0};
  // Running (uniform) byte offsets of the next loads, advanced by one position per step
  // and wrapped to the next channel chunk after the last position: a loop-carried scalar
  // each, instead of one precomputed base per position.
  size_t vchunk = 0, uchunk = 0;
  size_t vld = kDepth * vp, uld = kDepth * up;
  for (int ch = 0; ch < nchunk; ++ch) {
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const op_t bv = bufV[p % kDepth], au = bufU[p % kDepth];
      // refill the slot with the operands of step p + kDepth (of the next chunk, if any,
      // once the positions of this one are all on their way)
      if (p + kDepth < P || ch + 1 < nchunk) {
        bufV[p % kDepth] = *(const op_t*)(vrow + vld + voff);
        bufU[p % kDepth] = *(const op_t*)(urow + uld + uoff);
      }
      if (p + kDepth + 1 == P) {
        vchunk += 64;
        uchunk += kUChunk;
        vld = vchunk;
        uld = uchunk;
      } else {
        vld += vp;
        uld += up;
      }
      // (empty statement: keeps the two offsets in scalar registers as they are; without
      // it the optimiser rewrites the chain as one 64-bit vector pointer per position)
      asm volatile("" : "+s"(vld), "+s"(uld));
      if constexpr (I8) {
        acc[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(au, bv, acc[p], 0, 0, 0);
      } else {
        acc[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(au.x, bv.x, acc[p], 0, 0, 0);
        acc[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(au.y, bv.y, acc[p], 0, 0, 0);
        acc[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(au.z, bv.z, acc[p], 0, 0, 0);
        acc[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(au.w, bv.w, acc[p], 0, 0, 0);
      }
    }
  }

  // lane holds M[., t, k] for k = kb + wave*16 + grp*4 + rr, rr = 0..3
  if (t >= g.T) return;
  const int tw = t % g.TW, th = (t / g.TW) % g.TH, img = t / (g.TW * g.TH);
  finish_lane<M, I8, kSparse, kMQ>(g, at, acc, yv, img, th, tw, kb + wave * 16 + grp * 4, r_m, r_y, qmax);
}

template <int M, bool I8>
hipError_t launch_m(const Geom& g, const MatAT& at, const void* V, const void* U, void* y,
                    float r_m, float r_y, float qmax, hipStream_t s) {
  const size_t esz = I8 ? 1 : 4;
  if (g.Kp / 64 > 65535 || (size_t)g.Tp * g.Cp * esz >= 0xffffffffull ||
      (size_t)g.Kp * g.Cp * esz >= 0xffffffffull)
    return hipErrorInvalidValue;
  dim3 grid(g.Tp / 16, g.Kp / 64);
  const bool sparse = sparse_at<M>(at.v);
  if (I8 && r_m > 0.0f) {
    if (sparse)
      gemm_out_kernel<M, I8, true, I8><<<grid, 256, 0, s>>>(g, at, V, U, y, r_m, r_y, qmax);
    else
      gemm_out_kernel<M, I8, false, I8><<<grid, 256, 0, s>>>(g, at, V, U, y, r_m, r_y, qmax);
  } else {
    if (sparse)
      gemm_out_kernel<M, I8, true, false><<<grid, 256, 0, s>>>(g, at, V, U, y, r_m, r_y, qmax);
    else
      gemm_out_kernel<M, I8, false, false><<<grid, 256, 0, s>>>(g, at, V, U, y, r_m, r_y, qmax);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_out(const Geom& g, const MatAT& at, const void* V, const void* U, void* y,
                           float r_m, float r_y, float qmax, hipStream_t s) {
  if (g.i8) {
    switch (g.m) {
      case 2: return launch_m<2, true>(g, at, V, U, y, r_m, r_y, qmax, s);
      case 4: return launch_m<4, true>(g, at, V, U, y, r_m, r_y, qmax, s);
      default: return launch_m<6, true>(g, at, V, U, y, r_m, r_y, qmax, s);
    }
  }
  switch (g.m) {
    case 2: return launch_m<2, false>(g, at, V, U, y, r_m, r_y, qmax, s);
    case 4: return launch_m<4, false>(g, at, V, U, y, r_m, r_y, qmax, s);
    default: return launch_m<6, false>(g, at, V, U, y, r_m, r_y, qmax, s);
  }
}

}  // namespace wino
