// The whole int8 forward of the Winograd-aware layer in ONE kernel (Sec. 3.2, Fig. 2):
// input transform B^T d B + quantizer, per-position GEMM over the input channels,
// output transform A^T M A + quantizer, NCHW store.  Neither the transformed input V
// nor the GEMM result M ever goes to memory; per layer the kernel reads X and U and
// writes Y.  On the small layers this path is made for (64..128 channels), a separate
// kernel costs several microseconds of launch and memory latency before it does any
// work, which is as long as the work itself.
//
// Workgroup = 256 threads = 16 tiles x (4 waves x 16 output channels).  For every
// block of 64 input channels:
//   1. stage the input rows of the 16 tiles into LDS (input_stage.h, phase 1);
//   2. thread (tile, channel quad) transforms and quantizes its four channels and
//      writes the int8 codes to LDS as Vl[p][tile][64 channels] -- exactly the
//      channel-contiguous "B" operand rows of v_mfma_i32_16x16x64_i8.  Vl reuses the
//      staging area (every thread has its patch in registers before anyone writes);
//   3. wave w multiplies: for every position p one MFMA with U[p][16 k of w][64 c] as
//      the "A" operand, loaded straight from global memory / L2 through a register
//      ring, accumulating into acc[p].
// After the last channel block a lane holds M[., tile, 4 consecutive k] and finishes
// with the lane-local output transform (output_stage.h).
//
// If K > 64 the grid's y dimension repeats the input transform for every 64 output
// channels, so the host uses this kernel only while that repetition is cheaper than
// writing and re-reading V.
#include "input_stage.h"
#include "output_stage.h"

namespace wino {
namespace {

// kFast: whole tiles and K % 4 == 0 (branch-free output side, see output_stage.h).
// kOneBlock: C <= 64, a single channel block; the accumulators then start life at the
// MFMAs (zero "C" operand) instead of occupying registers during staging and transform.
// That variant is held to 256 registers per lane, i.e. at least two workgroups per compute
// unit: one's memory and LDS latencies hide behind the other's arithmetic.
// pos != 0: per-position scales -- rv[p] is the quantizer factor of V at position p (else
// r_v everywhere) and w[p] brings accumulator p to real units.  The quantizer
// after the Hadamard stage (r_m > 0) and `pos` are run-time options (output_stage.h).
template <int M, bool kSparseB, bool kSparseA, bool kWide, bool kFast, bool kOneBlock>
__global__ __launch_bounds__(256, kOneBlock ? 2 : 1) void fused_fwd_i8_kernel(
    Geom g, MatBT bt, MatAT at, const int8_t* __restrict__ x, const int8_t* __restrict__ U,
    void* __restrict__ y, float r_v, float r_m, float r_y, float qmax, int RB, int TWB, int pos,
    PosScale rv, PosScale w) {
  constexpr int n = M + 2, P = n * n, CBQ = InCfg<M>::kCBQ;
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  uint32_t* Vl = lds;                                 // [P][16 tiles][16 dwords], aliases staging
  const int Wc = stage_cols(M, TWB);
  const int ntwb = (g.TW + TWB - 1) / TWB;
  const int twb = blockIdx.x % ntwb, rb = blockIdx.x / ntwb;
  const int r0 = rb * RB, tw0 = twb * TWB, kb = blockIdx.y * 64;
  const int R = g.N * g.TH;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, grp = lane >> 4;
  const float lo = kMagic - qmax, hi = kMagic + qmax;

  // phase-2 role: tile tl of the workgroup, channel quad cq
  const int cq = tid & 15, tl = tid >> 4;
  const int rs2 = tl / TWB, twl2 = tl - rs2 * TWB;
  const bool has_tile = rs2 < RB;                      // RB * TWB may be less than 16

  // MFMA role: "A" rows = output channels kb + wave*16 + r, 16 bytes at channel grp*16: in
  // the blocked layout of the weights (u_byte_index) the wavefront's 16 x 64 block of a
  // channel block is 1 KB of consecutive bytes, this lane's piece at (grp*16 + r) * 16
  const int8_t* urow = U + (size_t)((kb + wave * 16) >> 4) * (g.Cp >> 6) * 1024 + (grp * 16 + r) * 16;
  const size_t up = (size_t)g.Kp * g.Cp;

  v4i acc[P];
  if constexpr (!kOneBlock) {
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p] = v4i{0, 0, 0, 0};
  }

  const int nblk = kOneBlock ? 1 : (g.Cp >> 6);
  for (int cb = 0; cb < nblk; ++cb) {
    if (cb) __syncthreads();                           // previous block's Vl fully consumed
    stage_strips<M, kWide>(g, x, lds, cb * 64, r0, tw0, RB, TWB);
    __syncthreads();
    uint32_t raw[n][n];
    if (has_tile) {
      load_quad_patch<M>(lds + ((size_t)rs2 * n * Wc + twl2 * M) * CBQ + cq, Wc, raw);
    } else {
#pragma unroll
      for (int j = 0; j < n; ++j)
#pragma unroll
        for (int l = 0; l < n; ++l) raw[j][l] = 0u;
    }
    __syncthreads();                                   // staging area is free: Vl may overwrite it
    {
      uint32_t out[P];
      // (one copy per kind of scale: 36 factors in scalar registers would crowd out the
      // per-tensor path's matrix entries)
      if (pos) transform_raw<M, kSparseB, true>(raw, bt, 0.0f, lo, hi, out, &rv);
      else transform_raw<M, kSparseB, false>(raw, bt, r_v, lo, hi, out);
#pragma unroll
      for (int p = 0; p < P; ++p) Vl[(p * 16 + tl) * 16 + cq] = out[p];
    }
    __syncthreads();

    // one MFMA per position; U through a register ring kDepth positions deep
    constexpr int kDepth = M == 4 ? 9 : 8;
    static_assert(P % kDepth == 0, "ring depth must divide the number of positions");
    const int8_t* ub = urow + (size_t)cb * 1024;
    v4i bufU[kDepth];
#pragma unroll
    for (int p = 0; p < kDepth; ++p) bufU[p] = *(const v4i*)(ub + p * up);
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const v4i au = bufU[p % kDepth];
      if (p + kDepth < P) bufU[p % kDepth] = *(const v4i*)(ub + (p + kDepth) * up);
      const v4i bv = *(const v4i*)(Vl + (p * 16 + r) * 16 + grp * 4);
      if constexpr (kOneBlock)
        acc[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(au, bv, v4i{0, 0, 0, 0}, 0, 0, 0);
      else
        acc[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(au, bv, acc[p], 0, 0, 0);
    }
  }

  // lane holds M[., tile r, k] for k = kb + wave*16 + grp*4 + rr
  const int rs = r / TWB, twl = r - rs * TWB;
  const int rr_ = r0 + rs, tw = tw0 + twl;
  const int k0 = kb + wave * 16 + grp * 4;
  if (rs >= RB || rr_ >= R || tw >= g.TW || k0 >= g.K) return;
  const int img = rr_ / g.TH, th = rr_ - img * g.TH;
  finish_lane_any<M, kSparseA, kFast>(g, at, acc, y, img, th, tw, k0, r_m, r_y, qmax, pos != 0, w.r);
}

template <int M, bool kSparseB, bool kSparseA>
hipError_t launch_k(const Geom& g, const MatBT& bt, const MatAT& at, const int8_t* x,
                    const int8_t* U, void* y, float r_v, float r_m, float r_y, float qmax,
                    const PosScale* rv_pos, const PosScale* w_pos, hipStream_t s) {
  constexpr int n = M + 2, P = n * n;
  const int R = g.N * g.TH;
  int TWB = g.TW < 16 ? g.TW : 16;
  int RB = 16 / TWB;
  if (RB > R) RB = R;
  const size_t stage_b = (size_t)stage_dwords<M>(RB, TWB) * 4, vl_b = (size_t)P * 16 * 16 * 4;
  const size_t lb = stage_b > vl_b ? stage_b : vl_b;
  const int ntwb = (g.TW + TWB - 1) / TWB, nrb = (R + RB - 1) / RB;
  if (lb > 65536 || (long long)ntwb * nrb > 0x7fffffffLL || g.Kp / 64 > 65535 ||
      n * (stage_cols(M, TWB) / 4) > 256 || (rv_pos == nullptr) != (w_pos == nullptr))
    return hipErrorInvalidValue;
  PosScale rv, w;
  for (int p = 0; p < 64; ++p) {
    rv.r[p] = rv_pos ? rv_pos->r[p] : r_v;
    w.r[p] = w_pos ? w_pos->r[p] : 1.0f;
  }
  const int pos = w_pos != nullptr;
  dim3 grid((unsigned)(ntwb * nrb), (unsigned)(g.Kp / 64));
#define WINO_LAUNCH_FUSED1(WIDE, FAST, ONE)                                           \
  fused_fwd_i8_kernel<M, kSparseB, kSparseA, WIDE, FAST, ONE><<<grid, 256, lb, s>>>(   \
      g, bt, at, x, U, y, r_v, r_m, r_y, qmax, RB, TWB, pos, rv, w)
  // What the dispatch sends here (fused_fwd_generic_preferred): images at least 8 wide, one
  // block of input channels, or two for F2 -- nothing else is instantiated.
  if (g.W < 8 || (g.Cp != 64 && !(M == 2 && g.Cp == 128))) return hipErrorInvalidValue;
#define WINO_LAUNCH_FUSED(WIDE, FAST)                                                 \
  do { if (g.Cp == 64) WINO_LAUNCH_FUSED1(WIDE, FAST, true);                          \
       else if constexpr (M == 2) WINO_LAUNCH_FUSED1(WIDE, FAST, false); } while (0)
  // whole tiles and K % 4 == 0: no guards on the output side
  // (the branch-free output side stores 2 or 4 codes at a time: y must be aligned for that)
  const bool fast = g.Ho % M == 0 && g.Wo % M == 0 && g.K % 4 == 0 && ((uintptr_t)y & 3) == 0;
  if (fast) WINO_LAUNCH_FUSED(true, true); else WINO_LAUNCH_FUSED(true, false);
#undef WINO_LAUNCH_FUSED
#undef WINO_LAUNCH_FUSED1
  return hipGetLastError();
}

template <int M>
hipError_t launch_m(const Geom& g, const MatBT& bt, const MatAT& at, const int8_t* x,
                    const int8_t* U, void* y, float r_v, float r_m, float r_y, float qmax,
                    const PosScale* rv_pos, const PosScale* w_pos, hipStream_t s) {
  const bool sb = fits_mask(bt.v, g.n * g.n, CookToomMask<M>::bt);
  const bool sa = sparse_at<M>(at.v);
#define WINO_ARGS g, bt, at, x, U, y, r_v, r_m, r_y, qmax, rv_pos, w_pos, s
  if (sb && sa) return launch_k<M, true, true>(WINO_ARGS);
  if (sb) return launch_k<M, true, false>(WINO_ARGS);
  if (sa) return launch_k<M, false, true>(WINO_ARGS);
  return launch_k<M, false, false>(WINO_ARGS);
#undef WINO_ARGS
}

}  // namespace

bool fused_fwd_supported(const Geom& g) {
  // int8, F2 or F4 (F6 needs 256 accumulator registers per lane on top of the input
  // transform's working set), and few enough output-channel blocks that repeating the
  // input transform per block stays cheaper than a round trip of V through memory.
  return g.i8 && (g.m == 2 || g.m == 4) && g.Kp <= 128;
}

hipError_t launch_fused_fwd(const Geom& g, const MatBT& bt, const MatAT& at, const void* x,
                            const void* U, void* y, float r_v, float r_m, float r_y, float qmax,
                            const PosScale* rv_pos, const PosScale* w_pos, hipStream_t s) {
  if (!fused_fwd_supported(g)) return hipErrorInvalidValue;
  if (g.m == 2)
    return launch_m<2>(g, bt, at, (const int8_t*)x, (const int8_t*)U, y, r_v, r_m, r_y, qmax,
                       rv_pos, w_pos, s);
  return launch_m<4>(g, bt, at, (const int8_t*)x, (const int8_t*)U, y, r_v, r_m, r_y, qmax, rv_pos,
                     w_pos, s);
}

}  // namespace wino
