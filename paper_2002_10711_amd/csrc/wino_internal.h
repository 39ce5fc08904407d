// Internal declarations shared by the host API and the kernel files of libwino.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wino.h"

namespace wino {

// Derived sizes of one layer problem.  Private device layouts:
//   V [P][Tp][Cp]   transformed input, int8 or float, channel fastest
//   U [P][Kp][Cp]   transformed weights, int8 or float, channel fastest
//   M [P][Tp][Kp]   Hadamard/GEMM result, int32 or float
// with Tp, Kp rounded up to 64 and Cp rounded up to 64 (int8) / 16 (float).
// Padding channels are written as zero by the transform kernels; padding tiles
// and padding output channels are computed on and never read back.
struct Geom {
  int N, C, K, H, W, pad, m, n, P;
  int Ho, Wo, TH, TW, T;
  int Tp, Cp, Kp;
  int i8;
  int w16;   // 16-bit codes in the Winograd domain (WINO_I16, WINO_I8W16): own kernels, own layouts
  int x16;   // ... and int16 containers for X and Y (WINO_I16)
  int bf16;  // float path with bf16 GEMM operands (WINO_BF16): own U layout, one-kernel forward only
};

struct MatBT { float v[64]; };   // n x n, row-major, n <= 8
struct MatG  { float v[24]; };   // n x 3
struct MatAT { float v[48]; };   // m x n, m <= 6
struct PosScale { float r[64]; };   // one factor per Winograd position (n*n <= 64)

inline int round_up(int a, int b) { return (a + b - 1) / b * b; }

// Private layout of the transformed weights U: per position, blocks of 16 output channels
// x 64 bytes of the reduction axis (64 int8 or 16 fp32 input channels), [p][Kp/16][row
// bytes/64] blocks of 1 KB, each in the order in which an MFMA wavefront loads it -- the
// 16-byte piece (segment q of the 64 bytes, output channel k) sits at piece index
// q*16 + k, which is the lane that needs it.  A wavefront's operand load is then 1 KB of
// consecutive bytes (8 cache lines) instead of 16 bytes from each of up to 64 lines.
// Byte offset of element U[p][k][c], esz = bytes per element:
__host__ __device__ inline size_t u_byte_index(int Kp, int Cp, int esz, int p, int k, int c) {
  const int cb = c * esz;                               // byte position in the row
  const size_t blk = ((size_t)p * (Kp >> 4) + (k >> 4)) * ((Cp * esz) >> 6) + (cb >> 6);
  return (blk * 64 + (size_t)(((cb & 63) >> 4) * 16 + (k & 15))) * 16 + (cb & 15);
}

// Host-side pieces shared by the entry points (api.cpp).
size_t fwd_workspace_touched(const wino_desc* d);
wino_status fwd_check(const wino_desc* d, const wino_quant* q, const void* x_dev,
                      const void* U_dev, const void* y_dev, int stages, Geom* g);
wino_status fwd_stages(const wino_desc* d, const wino_quant* q, const void* x_dev,
                       const void* U_dev, void* y_dev, void* workspace_dev,
                       size_t workspace_bytes, int stages, void* stream, bool exact_need,
                       int forced_seq);

// Kernel launchers (each enqueues on `s` and returns hipGetLastError()).
// (the optional PosScale arguments switch a stage to per-position factors: r_v[p], r_u[p],
// and w[p] = s_u[p] * s_v[p] applied to the accumulators before the output transform)
hipError_t launch_input_transform(const Geom& g, const MatBT& bt, const void* x, void* V,
                                  float r_v, float qmax, hipStream_t s,
                                  const PosScale* rv_pos = nullptr);
hipError_t launch_weight_transform(const Geom& g, const MatG& mg, const float* w, void* U,
                                   float r_u, float qmax, hipStream_t s,
                                   const PosScale* ru_pos = nullptr);
// Batched GEMM  M[p][t][k] = sum_c A[p][t][c] * B[p][k][c]; rows padded as above.
// Used with P = n*n for the Winograd domain and P = 1 for the im2row baseline.
// b_blocked: B is in the block layout of u_byte_index.
hipError_t launch_gemm(int P, int Tp, int Kp, int Cp, int i8, int b_blocked, const void* A,
                       const void* B, void* M, hipStream_t s);
hipError_t launch_output_transform(const Geom& g, const MatAT& at, const void* M, void* y,
                                   float r_m, float r_y, float qmax, hipStream_t s,
                                   const PosScale* w_pos = nullptr);
// Kernel sequences of the int8 forward (which one runs is looked up in a table of measured
// times, see fwd_sequence_auto):
enum FwdSeq {
  kSeqAuto = 0,
  kSeqFused = 1,    // one kernel: matrix-core input transform, per-position MFMAs, output transform
  kSeqCol = 2,      // input stage; GEMM + column-wise output transform (gemm_out_col_kernel)
  kSeqCol2 = 3,     // ... with two tile blocks per wavefront
  kSeqLds = 4,      // input stage; GEMM + output transform with 32 x 64 workgroup tiles
  kSeqRegs = 5,     // input stage; GEMM + output transform, all accumulators in registers
  kSeqStaged = 6,   // input stage; LDS-tiled GEMM writing M; output transform
  kSeqTrow = 7,     // input stage; GEMM + output transform on whole rows of tiles (F6)
  kSeqCount = 8
};
// Can sequence `seq` run this problem at all (shape and matrices only)?
bool fwd_sequence_supported(const Geom& g, const MatBT* bt, int seq);
// The sequence wino_conv2d_fwd takes: the fastest supported one at the nearest point of the
// measured grid (dispatch_table.h, written by paper_2002_10711_amd/tune.py).
// allow_fused: the call runs the whole forward (a stage-by-stage call cannot fuse it).
int fwd_sequence_auto(const Geom& g, const MatBT* bt, bool allow_fused);
// fp32: GEMM + output transform in one kernel (gemm_out_kernel) while the reduction is short
// enough for the operand stream to stay ahead of the matrix cores.
inline bool gemm_out_f32_preferred(const Geom& g) {
  return !g.i8 && !g.w16 && g.Cp * 4 <= (g.m == 6 ? 64 : 128);
}

// GEMM and output transform in one kernel (M stays in registers, operands straight
// from global memory).
hipError_t launch_gemm_out(const Geom& g, const MatAT& at, const void* V, const void* U, void* y,
                           float r_m, float r_y, float qmax, hipStream_t s);
// The same for long int8 reductions (64 .. 512 padded channels in steps of 64; per-tensor
// or per-position scales): column-by-column output transform, V shared through LDS.
// two_blocks: two tile blocks per wavefront (every U operand feeds two MFMAs, half the
// workgroups), built for F(2x2,3x3) at 256 and F(4x4,3x3) at 512 padded channels.
bool gemm_out_col_supported(const Geom& g);
bool gemm_out_col2_supported(const Geom& g);
hipError_t launch_gemm_out_col(const Geom& g, const MatAT& at, const void* V, const void* U,
                               void* y, const PosScale* w_pos, float r_m, float r_y, float qmax,
                               hipStream_t s, bool two_blocks);
// The same for F(2x2,3x3) with 512 padded input channels: workgroup tiles of 32 tiles x 64
// channels (fewer operand bytes per compute unit), 32x32x32 MFMAs.
bool gemm_out_lds_supported(const Geom& g);
hipError_t launch_gemm_out_lds(const Geom& g, const MatAT& at, const void* V, const void* U,
                               void* y, const PosScale* w_pos, float r_m, float r_y, float qmax,
                               hipStream_t s);
// The same for F(6x6,3x3) with 64, 128 or 256 padded input channels and output rows of a
// multiple of 16 pixels: workgroups of 32 tiles x 32 channels that own whole rows of tiles,
// both operands staged through LDS, output codes stored as 16-byte pieces of plane rows.
// (y must be 16-byte aligned: the launcher returns hipErrorInvalidValue otherwise.)
bool gemm_out_trow_supported(const Geom& g);
hipError_t launch_gemm_out_trow(const Geom& g, const MatAT& at, const void* V, const void* U,
                                void* y, const PosScale* w_pos, float r_m, float r_y, float qmax,
                                hipStream_t s);
// Whole int8 forward in one kernel (neither V nor M stored); only where supported.
bool fused_fwd_supported(const Geom& g);
// ... and worth it with the vector-ALU input transform, which a second block of output
// channels would have to repeat in full.
// Measured against the separate input stage plus GEMM + output kernel: a single block of
// input channels always wins; two blocks only for F2 with few tiles (12.5 vs 16.9 us at 4 k
// tiles, 44 vs 37 at 16 k); longer reductions lose (F4, 256 channels: 44.5 vs 28.6 us).
inline bool fused_fwd_generic_preferred(const Geom& g) {
  return g.Kp <= 64 && g.W >= 8 && (g.Cp == 64 || (g.m == 2 && g.Cp == 128 && g.T < 8192));
}
hipError_t launch_fused_fwd(const Geom& g, const MatBT& bt, const MatAT& at, const void* x,
                            const void* U, void* y, float r_v, float r_m, float r_y, float qmax,
                            const PosScale* rv_pos, const PosScale* w_pos, hipStream_t s);
// Whole fp32 forward in one kernel; only where supported.
bool fused_fwd_f32_supported(const Geom& g);
hipError_t launch_fused_fwd_f32(const Geom& g, const MatBT& bt, const MatAT& at, const void* x,
                                const void* U, void* y, hipStream_t s);
// The same with bf16 operands in the per-position GEMM (WINO_BF16): U in the layout of
// ubf_index, written by launch_weight_transform when g.bf16 is set.
bool fused_fwd_bf16_supported(const Geom& g);
hipError_t launch_fused_fwd_bf16(const Geom& g, const MatBT& bt, const MatAT& at, const void* x,
                                 const void* U, void* y, hipStream_t s);
// Element index of U[p][k][c] in the bf16 layout: per position, blocks of 16 output channels
// x 16 input channels (512 bytes), each in the order in which an MFMA wavefront loads it --
// lane (k % 16, c % 16 / 4) takes the four consecutive channels c % 4 = 0 .. 3 as one 8-byte
// piece at piece index (c % 16 / 4) * 16 + k % 16.
__host__ __device__ inline size_t ubf_index(int Kp, int Cp, int p, int k, int c) {
  const size_t blk = ((size_t)p * (Kp >> 4) + (k >> 4)) * (Cp >> 4) + (c >> 4);
  return blk * 256 + (size_t)((((c & 15) >> 2) * 16 + (k & 15)) * 4 + (c & 3));
}
// The fp32 input stage alone, LDS-staged (coalesced row loads); only where supported.
bool input_f32_staged_supported(const Geom& g);
hipError_t launch_input_f32_staged(const Geom& g, const MatBT& bt, const void* x, void* V,
                                   hipStream_t s);
// The same for F(4x4,3x3) with an exact (dyadic) B^T: input transform on the matrix cores.
bool fused_fwd_exact_supported(const Geom& g, const MatBT& bt);
// The input stage alone with the same exact transform (any number of output channels).
bool input_exact_supported(const Geom& g, const MatBT& bt);
// (smallest s <= 3 with 2^s B^T integral and int8 products; -1 if none)
int exact_input_shift(const Geom& g, const MatBT& bt);
bool input_exact_preferred(const Geom& g, const MatBT& bt, const void* x);
hipError_t launch_input_exact(const Geom& g, const MatBT& bt, const void* x, void* V, float r_v,
                              float qmax, hipStream_t s, const PosScale* rv_pos = nullptr);
// (rv_pos, w_pos: per-position quantizer factors of V and factors of the accumulators,
// both or neither; nullptr = per-tensor scales)
hipError_t launch_fused_fwd_exact(const Geom& g, const MatBT& bt, const MatAT& at, const void* x,
                                  const void* U, void* y, float r_v, float r_m, float r_y,
                                  float qmax, const PosScale* rv_pos, const PosScale* w_pos,
                                  hipStream_t s);
hipError_t launch_export(const Geom& g, int which, const void* src, void* out, hipStream_t s);

// The path with up to 16-bit codes after every stage (g.w16): weight stage, input stage,
// exact int64 GEMM on int8 digit planes, output stage; layouts private to these kernels.
hipError_t launch_w16_weights(const Geom& g, const MatG& mg, const float* w, void* U,
                              const PosScale& ru, float qmax, hipStream_t s);
hipError_t launch_w16_input(const Geom& g, const MatBT& bt, const void* x, void* V,
                            const PosScale& rv, float qmax, hipStream_t s);
hipError_t launch_w16_gemm(const Geom& g, const void* V, const void* U, void* M, hipStream_t s);
hipError_t launch_w16_output(const Geom& g, const MatAT& at, const void* M, void* y,
                             const PosScale* w_pos, float r_m, float r_y, float qmax_m,
                             float qmax_y, hipStream_t s);
// GEMM and output stage in one kernel (M stays in registers); only where supported.
bool w16_gemm_out_supported(const Geom& g, const MatAT& at);
hipError_t launch_w16_gemm_out(const Geom& g, const MatAT& at, const void* V, const void* U,
                               void* y, const PosScale* w_pos, float r_m, float r_y, float qmax_m,
                               float qmax_y, hipStream_t s);
hipError_t launch_w16_export(const Geom& g, int which, const void* src, void* out, hipStream_t s);

// im2row baseline pieces.
struct RefGeom {
  int N, C, K, H, W, stride, pad, Ho, Wo, T, Tp, Cp, Kp, i8;
};
// Packed weights: rows of 9*Cp values per output channel (tap-major); for int8 a second copy
// in MFMA operand order follows at this byte offset (a multiple of 256).
__host__ __device__ inline size_t ref_operand_weights_offset(int Cp, int Kp) { return (size_t)Kp * 9 * Cp; }
hipError_t launch_ref_pack_weights(int C, int K, int Cp, int Kp, int i8, const void* w, void* wp,
                                   hipStream_t s);
hipError_t launch_im2row(const RefGeom& g, const void* x, void* rows, hipStream_t s);
hipError_t launch_ref_epilogue(const RefGeom& g, const void* M, void* y, float r_y, float qmax,
                               hipStream_t s);
// The same convolution as one kernel that gathers its rows in LDS (int8 only).
bool conv_implicit_supported(const RefGeom& g);
hipError_t launch_conv_implicit(const RefGeom& g, const void* x, const void* wp, void* y, float r_y,
                                float qmax, hipStream_t s);

}  // namespace wino
