// The whole fp32 forward of the layer (Eq. 1 with the channel sum in the Winograd
// domain, Sec. 3.1 and 5.3; quantizers off) in ONE kernel: input transform B^T d B,
// per-position GEMM over the input channels on v_mfma_f32_16x16x4_f32, output transform
// A^T M A, NCHW store.  V and M never go to memory.
//
// Workgroup = 256 threads = 16 tiles x (4 waves x 16 output channels).  For every block of
// 16 input channels:
//   1. the input rows of the 16 tiles are staged in LDS as floats, Xs[channel][row][col],
//      with coalesced loads along the image rows (zero outside the image);
//   2. thread (tile, channel) takes its n x n patch to registers, transforms it with the
//      pinned fmaf chains and writes V to LDS as Vl[p][tile][16 channels] -- a lane of the
//      MFMA then reads four consecutive channels (16 bytes) and feeds them to four MFMAs;
//      Vl reuses the staging area (every patch is in registers before anyone writes);
//   3. wave w multiplies: per position four MFMAs with U[p][16 k of w][4 x 4 channels] as
//      the "A" operand, streamed from global memory / L2 through a register ring.
// Whatever order the instruction gives the four reduction elements of a lane group, it is
// the same for both operands.  After the last block a lane holds M[., tile, 4 consecutive k]
// and finishes with the lane-local output transform.
//
// The matrix pipe bounds this kernel: fp32 MFMA peak is 1/32 of the int8 one.
#include "fastdiv.h"
#include "output_stage.h"

#if defined(WINO_PROFILE_PHASES)
// Development build only: shader-clock timestamps per wavefront and phase.
__device__ unsigned long long wino_phase_ts_f32[4096 * 16];
#define WINO_TSF(slot)                                                                    \
  if ((threadIdx.x & 63) == 0 && blockIdx.y == 0 && blockIdx.z == 0 && blockIdx.x < 1024)   \
    wino_phase_ts_f32[(blockIdx.x * 4 + (threadIdx.x >> 6)) * 16 + (slot)] = __builtin_amdgcn_s_memtime()
extern "C" int wino_debug_read_phases_f32(unsigned long long* host, size_t count) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(wino_phase_ts_f32), count * sizeof(unsigned long long));
}
#else
#define WINO_TSF(slot)
#endif

namespace wino {
namespace {

struct FPlan {
  int RB, TWB;               // tile rows and tiles per row of a workgroup (RB * TWB <= 16)
  int Wc;                    // staged columns per row: TWB * m + 2
  int rows;                  // staged rows per channel: RB * n
  int plane;                 // floats per channel in LDS (rows * Wc, made odd)
  int total, iters;          // staged elements per channel block, and ceil(total / 256)
  uint32_t inv_twb, inv_wc, inv_rows, inv_th;
};

template <int M, bool kSparseB, bool kSparseA>
__global__ __launch_bounds__(256) void fused_fwd_f32_kernel(const float* __restrict__ x,
                                                            const float* __restrict__ U,
                                                            float* __restrict__ y, Geom g, FPlan pl,
                                                            MatBT bt, MatAT at) {
  constexpr int n = M + 2, P = n * n, CB = 16;
  constexpr int kMaxIters = 32;                        // staged elements per thread and block
  extern __shared__ __attribute__((aligned(16))) float ldsf[];
  float* Xs = ldsf;
  float* Vl = ldsf;                                    // aliases Xs
  const int area = CB * pl.plane > P * 256 ? CB * pl.plane : P * 256;
  // ldsf[area .. area + 3]: 4 floats nobody reads (target of surplus staging lanes)
  int* rowinfo = (int*)(ldsf + area + 4);              // [rows]
  const int RB = pl.RB, TWB = pl.TWB, Wc = pl.Wc, rows = pl.rows, plane = pl.plane;
  const int r0 = blockIdx.x * RB, tw0 = blockIdx.y * TWB, kb = blockIdx.z * 64;
  const int R = g.N * g.TH, HW = g.H * g.W;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, grp = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // Row table: element offset of (image, channel 0, row h, column 0) for every staged row
  // of the workgroup, or -1 for rows outside the image / beyond the last tile row.
  if (tid < rows) {
    const int rs = tid / n, j = tid - rs * n;
    const int rr = r0 + rs;
    const int rc = rr < R ? rr : R - 1;
    const int img = (int)fast_div(rc, pl.inv_th), th = rc - img * g.TH;
    const int h = th * M - g.pad + j;
    rowinfo[tid] = (rr < R && h >= 0 && h < g.H) ? (img * g.C * g.H + h) * g.W : -1;
  }

  // phase-2 role: tile tl of the workgroup, channel c2 of the block
  const int c2 = tid & 15, tl = tid >> 4;
  const int rs2 = (int)fast_div(tl, pl.inv_twb), twl2 = tl - rs2 * TWB;
  const float* patch = Xs + c2 * plane + ((rs2 < RB ? rs2 : 0) * n) * Wc + twl2 * M;

  // MFMA role: "A" rows = output channels kb + wave*16 + r, 4 floats at channel grp*4
  const uint32_t uoff = ((uint32_t)(kb + wave * 16 + r) * (uint32_t)g.Cp + (uint32_t)grp * 4u) * 4u;
  const size_t up = (size_t)g.Kp * g.Cp * 4;
  const char* Ub = (const char*)U;

  v4f acc[P];
#pragma unroll
  for (int p = 0; p < P; ++p) acc[p] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

  // Staging plan of this thread, the same for every channel block: element e = tid + 256 i
  // of the block's [16 channels][rows][Wc] array -> element offset in x relative to the
  // block's first channel (-1: outside the image) and (channel << 16 | LDS index).
  const int wbase = tw0 * M - g.pad;
  int goff[kMaxIters];
  uint32_t lpk[kMaxIters];
  __syncthreads();                                     // row table complete
#pragma unroll
  for (int i = 0; i < kMaxIters; ++i) {
    const int e = tid + i * 256;
    const int ec = e < pl.total ? e : pl.total - 1;
    const int rowidx = (int)fast_div(ec, pl.inv_wc), col = ec - rowidx * Wc;
    const int c = (int)fast_div(rowidx, pl.inv_rows), rj = rowidx - c * rows;
    const int info = rowinfo[rj];
    const int w = wbase + col;
    const bool ok = e < pl.total && info >= 0 && w >= 0 && w < g.W;
    goff[i] = ok ? info + c * HW + w : -1;
    lpk[i] = ((uint32_t)c << 16) | (uint32_t)(e < pl.total ? c * plane + rj * Wc + col : area + (tid & 3));
  }
  // The loads of a block are all issued at once, one block ahead of its use: they are in
  // flight during the transform and the MFMAs of the block before.
  // (validity travels as one bit per element in a vector register: 32 lane masks kept
  // alive across the load latency would not fit the scalar registers)
  float xv[kMaxIters];
  uint32_t okbits = 0u;
  auto issue_loads = [&](int cbase) {
    okbits = 0u;
#pragma unroll
    for (int i = 0; i < kMaxIters; ++i) {
      if (i < pl.iters) {
        const bool ok = goff[i] >= 0 && cbase + (int)(lpk[i] >> 16) < g.C;
        xv[i] = x[ok ? goff[i] + cbase * HW : 0];
        okbits |= ok ? (1u << i) : 0u;
      }
    }
  };
  WINO_TSF(0);
  issue_loads(0);
  WINO_TSF(1);

  const int nblk = g.Cp / CB;
  for (int cb = 0; cb < nblk; ++cb) {
    if (cb) __syncthreads();                           // previous block's Vl consumed
    if (cb == 1) WINO_TSF(2);
    const int cbase = cb * CB;
#pragma unroll
    for (int i = 0; i < kMaxIters; ++i)
      if (i < pl.iters) ldsf[lpk[i] & 0xffffu] = (okbits & (1u << i)) ? xv[i] : 0.0f;
    __syncthreads();
    if (cb == 1) WINO_TSF(3);
    float d[n][n];
#pragma unroll
    for (int j = 0; j < n; ++j)
#pragma unroll
      for (int l = 0; l < n; ++l) d[j][l] = patch[j * Wc + l];
    __syncthreads();                                   // staging area is free: Vl may overwrite it
    if (cb == 1) WINO_TSF(4);
    if (cb + 1 < nblk) issue_loads(cbase + CB);
    if (cb == 1) WINO_TSF(5);
    {
      float Vt[n][n];
      transform_patch<M, kSparseB>(d, bt, Vt);
#pragma unroll
      for (int p = 0; p < P; ++p) Vl[(p * 16 + tl) * 16 + c2] = Vt[p / n][p % n];
    }
    __syncthreads();
    if (cb == 1) WINO_TSF(6);

    // four MFMAs per position; U through a register ring kDepth positions deep
    constexpr int kDepth = M == 4 ? 9 : 8;
    static_assert(P % kDepth == 0, "ring depth must divide the number of positions");
    const uint32_t ub = uoff + (uint32_t)cbase * 4u;
    v4f bufU[kDepth];
    // (uniform running pointer, one position per step; the empty statement keeps it in
    // scalar registers instead of one precomputed 64-bit base per position)
    const char* uld = Ub;
#pragma unroll
    for (int p = 0; p < kDepth; ++p) {
      bufU[p] = *(const v4f*)(uld + ub);
      uld += up;
      asm volatile("" : "+s"(uld));
    }
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const v4f au = bufU[p % kDepth];
      if (p + kDepth < P) {
        bufU[p % kDepth] = *(const v4f*)(uld + ub);
        uld += up;
        asm volatile("" : "+s"(uld));
      }
      const v4f bv = *(const v4f*)(Vl + (p * 16 + r) * 16 + grp * 4);
      acc[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(au.x, bv.x, acc[p], 0, 0, 0);
      acc[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(au.y, bv.y, acc[p], 0, 0, 0);
      acc[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(au.z, bv.z, acc[p], 0, 0, 0);
      acc[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(au.w, bv.w, acc[p], 0, 0, 0);
    }
    if (cb == 1) WINO_TSF(7);
  }

  WINO_TSF(8);
  // lane holds M[., tile r, k] for k = kb + wave*16 + grp*4 + rr
  const int rs = (int)fast_div(r, pl.inv_twb), twl = r - rs * TWB;
  const int rr_ = r0 + rs, tw = tw0 + twl;
  if (rs < RB && rr_ < R && tw < g.TW) {
    const int img = (int)fast_div(rr_, pl.inv_th), th = rr_ - img * g.TH;
    finish_lane<M, false, kSparseA, false>(g, at, acc, y, img, th, tw, kb + wave * 16 + grp * 4,
                                           0.0f, 0.0f, 0.0f);
  }
  WINO_TSF(9);
}

// Launch plan and dynamic LDS size; false if the shape does not fit the kernel's limits.
bool make_fplan(const Geom& g, FPlan* plp, size_t* lds_bytes, int* nrb, int* ntwb) {
  FPlan& pl = *plp;
  const int M = g.m, n = g.n, P = n * n;
  const int R = g.N * g.TH;
  pl.TWB = g.TW < 16 ? g.TW : 16;
  pl.RB = 16 / pl.TWB;
  if (pl.RB > R) pl.RB = R;
  pl.Wc = pl.TWB * M + 2;
  pl.rows = pl.RB * n;
  pl.plane = (pl.rows * pl.Wc) | 1;
  pl.total = 16 * pl.rows * pl.Wc;
  pl.iters = (pl.total + 255) / 256;
  pl.inv_twb = make_inv(pl.TWB);
  pl.inv_wc = make_inv(pl.Wc);
  pl.inv_rows = make_inv(pl.rows);
  pl.inv_th = make_inv(g.TH);
  const size_t area = (size_t)(16 * pl.plane > P * 256 ? 16 * pl.plane : P * 256);
  *lds_bytes = (area + 4 + pl.rows) * 4;
  *ntwb = (g.TW + pl.TWB - 1) / pl.TWB;
  *nrb = (R + pl.RB - 1) / pl.RB;
  // 32 = kMaxIters of the kernel; 65536 floats: the packed LDS index has 16 bits
  return *lds_bytes <= 65536 && *ntwb <= 65535 && g.Kp / 64 <= 65535 && pl.rows <= 256 &&
         pl.iters <= 32;
}

template <int M>
hipError_t launch_m(const Geom& g, const MatBT& bt, const MatAT& at, const float* x, const float* U,
                    float* y, hipStream_t s) {
  FPlan pl;
  size_t lb;
  int nrb, ntwb;
  if (!make_fplan(g, &pl, &lb, &nrb, &ntwb)) return hipErrorInvalidValue;
  dim3 grid((unsigned)nrb, (unsigned)ntwb, (unsigned)(g.Kp / 64));
  const bool sb = fits_mask(bt.v, g.n * g.n, CookToomMask<M>::bt);
  const bool sa = fits_mask(at.v, g.m * g.n, CookToomMask<M>::at);
#define WINO_LAUNCH_F32(SB, SA) \
  fused_fwd_f32_kernel<M, SB, SA><<<grid, 256, lb, s>>>(x, U, y, g, pl, bt, at)
  if (sb && sa) WINO_LAUNCH_F32(true, true);
  else if (sb) WINO_LAUNCH_F32(true, false);
  else if (sa) WINO_LAUNCH_F32(false, true);
  else WINO_LAUNCH_F32(false, false);
#undef WINO_LAUNCH_F32
  return hipGetLastError();
}

}  // namespace

bool fused_fwd_f32_supported(const Geom& g) {
  // fp32, F2 or F4 (the 8 x 8 accumulator sets of F6 leave no room for the transforms), few
  // enough output-channel blocks that repeating the input transform per block is cheaper
  // than a round trip of V through memory; 32-bit element offsets into X and U, and exact
  // reciprocals (fastdiv.h) for the tile row index.
  const unsigned long long R = (unsigned long long)g.N * g.TH;
  FPlan pl;
  size_t lb;
  int nrb, ntwb;
  return !g.i8 && (g.m == 2 || g.m == 4) && g.Kp <= 128 && make_fplan(g, &pl, &lb, &nrb, &ntwb) &&
         (unsigned long long)g.N * g.C * g.H * g.W < 0x7fffffffull &&
         (unsigned long long)g.Kp * g.Cp * 4 < 0xffffffffull && R * g.TH < 0x100000000ull;
}

hipError_t launch_fused_fwd_f32(const Geom& g, const MatBT& bt, const MatAT& at, const void* x,
                                const void* U, void* y, hipStream_t s) {
  if (!fused_fwd_f32_supported(g)) return hipErrorInvalidValue;
  if (g.m == 2) return launch_m<2>(g, bt, at, (const float*)x, (const float*)U, (float*)y, s);
  return launch_m<4>(g, bt, at, (const float*)x, (const float*)U, (float*)y, s);
}

}  // namespace wino
