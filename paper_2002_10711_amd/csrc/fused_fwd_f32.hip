// The whole fp32 forward of the layer (Eq. 1 with the channel sum in the Winograd
// domain, Sec. 3.1 and 5.3; quantizers off) in ONE kernel: input transform B^T d B,
// per-position GEMM over the input channels on v_mfma_f32_16x16x4_f32, output transform
// A^T M A, NCHW store.  V and M never go to memory.
//
// The fp32 matrix pipe is slow (1/32 of the int8 rate) and every wavefront streams its
// own slice of U from L2 once per 16 tiles (8 flop per operand byte), so the MFMAs and
// their operand stream bound this kernel and everything else is arranged to run beside them.  A workgroup (16 tiles x 64 output
// channels) has EIGHT wavefronts in two roles, one of each per SIMD:
//   * wavefronts 0-3, "consumers": wave w owns output channels 16 w .. 16 w + 15; for every
//     block of 16 input channels and every position, four MFMAs with U[p][k][4 x 4
//     channels] (streamed from global memory / L2 through a register ring) as the "A"
//     operand and V (from LDS) as the "B" operand.  After the last block a lane holds
//     M[., tile, 4 consecutive k] and finishes with the lane-local output transform.
//   * wavefronts 4-7, "producers": while block s is multiplied they prepare block s + 1:
//     the input rows of the 16 tiles, staged in LDS as Xs[channel][row][col] with coalesced
//     loads along the image rows (issued a whole block ahead), then thread (tile, channel)
//     transforms its n x n patch with the pinned fmaf chains and writes it to the other
//     half of the double-buffered Vl[2][p][tile][16 channels].
// Both roles meet at two barriers per block (the consumers' first one sits a third of the
// way into their MFMA loop): every wavefront executes exactly 3 + 2 * (number of blocks)
// barriers, whatever its role.  A lane of the MFMA reads four consecutive channels
// (16 bytes) of V and of U and feeds them to four MFMAs: whatever order the instruction
// gives the four reduction elements of a lane group, it is the same for both operands.
#include "fastdiv.h"
#include "output_stage.h"

#if defined(WINO_PROFILE_PHASES)
// Development build only: shader-clock timestamps per wavefront and phase.
__device__ unsigned long long wino_phase_ts_f32[4096 * 16];
#define WINO_TSF(slot)                                                                    \
  if ((threadIdx.x & 63) == 0 && blockIdx.y == 0 && blockIdx.z == 0 && blockIdx.x < 512)    \
    wino_phase_ts_f32[(blockIdx.x * 8 + (threadIdx.x >> 6)) * 16 + (slot)] = __builtin_amdgcn_s_memtime()
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

// Workgroup barrier that orders LDS traffic only: the writers' LDS stores are complete
// before anyone passes, while global loads stay in flight across it (a full
// __syncthreads() would also wait for them, which is the latency this kernel hides).
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// kSparse: B^T and A^T both have the Cook-Toom zero pattern.
// kFast: whole tiles, K % 4 == 0, y 16-byte aligned (vector stores, no guards).
// kIters: staged elements per producer thread and block (>= ceil(total / 256)).
// kBF: bf16 operands in the per-position GEMM (WINO_BF16): the producers round V to bf16
// (nearest even) as they store it, U arrives as bf16 in the layout of ubf_index, and a
// block of 16 channels is one v_mfma_f32_16x16x16_bf16 per position instead of four fp32
// MFMAs at an eighth of the rate -- the consumers then wait for the producers, whose loads
// of the next block of X are no longer covered by a long MFMA phase (running them several
// blocks ahead was tried and measured slower: the waits the compiler places at the loop's
// joins drain every block in flight).  Everything else (staging, transforms, barriers,
// output side) is the fp32 kernel's.
template <int M, bool kSparse, bool kFast, int kIters, bool kBF = false>
__global__ __launch_bounds__(512) void fused_fwd_f32_kernel(const float* __restrict__ x,
                                                            const float* __restrict__ U,
                                                            float* __restrict__ y, Geom g, FPlan pl,
                                                            MatBT bt, MatAT at) {
  constexpr int n = M + 2, P = n * n, CB = 16;
  extern __shared__ __attribute__((aligned(16))) float ldsf[];
  float* Vl = ldsf;                                    // [2][P][16 tiles][16 channels]
  float* Xs = ldsf + 2 * P * 256;                      // [16 channels][plane]
  const int dumpi = 2 * P * 256 + CB * pl.plane;       // 4 floats nobody reads
  int* rowinfo = (int*)(ldsf + dumpi + 4);             // [rows]
  const int RB = pl.RB, TWB = pl.TWB, Wc = pl.Wc, rows = pl.rows, plane = pl.plane;
  const int r0 = blockIdx.x * RB, tw0 = blockIdx.y * TWB, kb = blockIdx.z * 64;
  const int R = g.N * g.TH, HW = g.H * g.W;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nblk = g.Cp / CB;

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
  lds_barrier();                                       // barrier 0: row table complete

  if (wave >= 4) {
    // ------------------------------------------------------------------ producers
    const int ptid = tid - 256;
    const int c2 = ptid & 15, tl = ptid >> 4;          // transform role: (tile, channel)
    const int rs2 = (int)fast_div(tl, pl.inv_twb), twl2 = tl - rs2 * TWB;
    const float* patch = Xs + c2 * plane + ((rs2 < RB ? rs2 : 0) * n) * Wc + twl2 * M;
    // Staging plan of this thread, the same for every channel block: element
    // e = ptid + 256 i of the block's [16 channels][rows][Wc] array -> element offset in x
    // relative to the block's first channel, LDS index, channel.  Elements outside the
    // image are zero in every block: their Xs slots are cleared once, here, and from then
    // on such lanes load x[0] (any valid address) and store to the dump area, so the
    // per-block work is one address add, one load and one LDS store per element, with no
    // decisions.  The loads of block 0 go out as soon as their offsets are known.
    const int wbase = tw0 * M - g.pad;
    const bool full_c = g.C % CB == 0;                 // no ragged last channel block
    int goff[kIters];
    uint32_t lpk[kIters];
    float xv[kIters];
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
      const int e = ptid + i * 256;
      const int ec = e < pl.total ? e : pl.total - 1;
      const int rowidx = (int)fast_div(ec, pl.inv_wc), col = ec - rowidx * Wc;
      const int c = (int)fast_div(rowidx, pl.inv_rows), rj = rowidx - c * rows;
      const int info = rowinfo[rj];
      const int w = wbase + col;
      const bool inside = info >= 0 && w >= 0 && w < g.W;
      const bool ok = e < pl.total && inside && c < g.C;          // (c < C: block 0)
      const int xs = 2 * P * 256 + c * plane + rj * Wc + col;
      goff[i] = ok ? info + c * HW + w : 0;
      xv[i] = x[goff[i]];
      if (e < pl.total && !ok) ldsf[xs] = 0.0f;
      lpk[i] = ((uint32_t)c << 16) | (uint32_t)(ok ? xs : dumpi + (ptid & 3));
    }
    // every block but a ragged last one: channel c of the block exists
    auto issue_loads = [&](int cbase) {
      const float* xb = x + (size_t)cbase * HW;
#pragma unroll
      for (int i = 0; i < kIters; ++i) xv[i] = xb[goff[i]];
    };
    // ragged last block: channels beyond C read x[0] and are stored as zero
    auto issue_loads_ragged = [&](int cbase) {
      const float* xb = x + (size_t)cbase * HW;
#pragma unroll
      for (int i = 0; i < kIters; ++i) {
        const bool ok = cbase + (int)(lpk[i] >> 16) < g.C;
        xv[i] = ok ? xb[goff[i]] : 0.0f;
      }
    };
    for (int nb = 0; nb < nblk; ++nb) {                // prepares block nb during step nb - 1
      const int cbase = nb * CB;
      if (nb == 1) WINO_TSF(6);
      // phase A: X of block nb into Xs (last read before the previous step's barrier 2)
#pragma unroll
      for (int i = 0; i < kIters; ++i) ldsf[lpk[i] & 0xffffu] = xv[i];
      if (nb == 1) WINO_TSF(7);
      lds_barrier();                                   // barrier 1 of step nb - 1
      if (nb == 1) WINO_TSF(8);
      // phase B: patch to registers, loads of the block after, transform, V to
      // Vl[nb & 1] (last read by the consumers before the previous step's barrier 2)
      float d[n][n];
#pragma unroll
      for (int j = 0; j < n; ++j)
#pragma unroll
        for (int l = 0; l < n; ++l) d[j][l] = patch[j * Wc + l];
      if (nb == 1) WINO_TSF(9);
      if (nb + 1 < nblk) {
        if (full_c || nb + 2 < nblk) issue_loads(cbase + CB);
        else issue_loads_ragged(cbase + CB);
      }
      if (nb == 1) WINO_TSF(10);
      {
        float Vt[n][n];
        transform_patch<M, kSparse>(d, bt, Vt);
        if constexpr (kBF) {
          __bf16* vdst = (__bf16*)Vl + (nb & 1) * P * 256 + tl * 16 + c2;
#pragma unroll
          for (int p = 0; p < P; ++p) vdst[p * 256] = (__bf16)Vt[p / n][p % n];
        } else {
          float* vdst = Vl + (nb & 1) * P * 256 + tl * 16 + c2;
#pragma unroll
          for (int p = 0; p < P; ++p) vdst[p * 256] = Vt[p / n][p % n];
        }
      }
      if (nb == 1) WINO_TSF(11);
      lds_barrier();                                   // barrier 2 of step nb - 1
      if (nb == 1) WINO_TSF(12);
    }
    // the consumers' last step: nothing left to prepare
    lds_barrier();
    lds_barrier();
    return;
  }

  // -------------------------------------------------------------------- consumers
  const int lane = tid & 63, r = lane & 15, grp = lane >> 4;
  v4f acc[P];
#pragma unroll
  for (int p = 0; p < P; ++p) acc[p] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
  constexpr int kVRing = 4;                            // V operands: LDS reads 4 positions ahead
  static_assert(P % kVRing == 0 && P % 2 == 0, "ring depths must divide the number of positions");
  constexpr int kSplit = (P / 3) & ~1;                 // barrier 1 after this many positions
  if constexpr (kBF) {
    // "A" rows = output channels kb + wave*16 + r, four bf16 at channel grp*4: in the layout
    // of ubf_index the wavefront's 16 x 16 block of a channel block is 512 consecutive
    // bytes, this lane's piece at (grp*16 + r) * 8
    typedef short v4s __attribute__((ext_vector_type(4)));
    const uint32_t uoff = (uint32_t)((kb + wave * 16) >> 4) * (uint32_t)(g.Cp >> 4) * 512u +
                          (uint32_t)(grp * 16 + r) * 8u;
    const size_t up = (size_t)g.Kp * g.Cp * 2;
    constexpr int kDepth = M == 4 ? 12 : 8;
    static_assert(P % kDepth == 0, "ring depth must divide the number of positions");
    v4s bufU[kDepth];
    const char* Ub = (const char*)U;
    size_t ublk = 0, uld = 0;
#pragma unroll
    for (int p = 0; p < kDepth; ++p) {
      bufU[p] = *(const v4s*)(Ub + uld + uoff);
      uld += up;
      asm volatile("" : "+s"(uld));
    }
    lds_barrier();                                     // step -1: the producers prepare block 0
    lds_barrier();
    for (int s = 0; s < nblk; ++s) {
      const __bf16* vb = (const __bf16*)Vl + (s & 1) * P * 256 + r * 16 + grp * 4;
      v4s bufV[kVRing];
#pragma unroll
      for (int p = 0; p < kVRing; ++p) bufV[p] = *(const v4s*)(vb + p * 256);
#pragma unroll
      for (int p0 = 0; p0 < P; p0 += 2) {
        if (p0 == kSplit) lds_barrier();               // barrier 1 of step s
        v4s au[2], bv[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int p = p0 + q;
          au[q] = bufU[p % kDepth];
          bv[q] = bufV[p % kVRing];
          if (p + kVRing < P) bufV[p % kVRing] = *(const v4s*)(vb + (p + kVRing) * 256);
          if (p + kDepth < P || s + 1 < nblk) bufU[p % kDepth] = *(const v4s*)(Ub + uld + uoff);
          if (p + kDepth + 1 == P) {
            ublk += 512;                               // next 16-channel block of U
            uld = ublk;
          } else {
            uld += up;
          }
          asm volatile("" : "+s"(uld));
        }
        acc[p0] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(au[0], bv[0], acc[p0], 0, 0, 0);
        acc[p0 + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(au[1], bv[1], acc[p0 + 1], 0, 0, 0);
      }
      lds_barrier();                                   // barrier 2 of step s
    }
  } else {
  // "A" rows = output channels kb + wave*16 + r, 4 floats at channel grp*4: in the blocked
  // layout of the fp32 weights (u_byte_index) the wavefront's 16 x 16 block of a channel
  // block is 1 KB of consecutive bytes, this lane's piece at (grp*16 + r) * 16
  const uint32_t uoff = (uint32_t)((kb + wave * 16) >> 4) * (uint32_t)(g.Cp >> 4) * 1024u +
                        (uint32_t)(grp * 16 + r) * 16u;
  const size_t up = (size_t)g.Kp * g.Cp * 4;

  // U through a register ring kDepth positions deep that runs on across the channel
  // blocks (uniform running byte offset, one position per step; the empty statement keeps
  // it in scalar registers instead of one precomputed 64-bit base per position)
  constexpr int kDepth = M == 4 ? 12 : 8;
  static_assert(P % kDepth == 0, "ring depth must divide the number of positions");
  v4f bufU[kDepth];
  const char* Ub = (const char*)U;
  size_t ublk = 0;                                     // byte offset of position 0, current block
  size_t uld = 0;
#pragma unroll
  for (int p = 0; p < kDepth; ++p) {
    bufU[p] = *(const v4f*)(Ub + uld + uoff);
    uld += up;
    asm volatile("" : "+s"(uld));
  }
  WINO_TSF(0);
  lds_barrier();                                       // step -1: the producers prepare block 0
  lds_barrier();
  WINO_TSF(1);

  for (int s = 0; s < nblk; ++s) {
    const float* vb = Vl + (s & 1) * P * 256 + r * 16 + grp * 4;
    v4f bufV[kVRing];
#pragma unroll
    for (int p = 0; p < kVRing; ++p) bufV[p] = *(const v4f*)(vb + p * 256);
    __builtin_amdgcn_sched_group_barrier(0x100, kVRing, 0);
#pragma unroll
    for (int p0 = 0; p0 < P; p0 += 2) {
      if (p0 == kSplit) {
        if (s == 0) WINO_TSF(13);
        lds_barrier();                                 // barrier 1 of step s
        if (s == 0) WINO_TSF(14);
      }
      v4f au[2], bv[2];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int p = p0 + q;
        au[q] = bufU[p % kDepth];
        bv[q] = bufV[p % kVRing];
        if (p + kVRing < P) bufV[p % kVRing] = *(const v4f*)(vb + (p + kVRing) * 256);
        // refill the U slot with position p + kDepth (of the next block, if any, once the
        // positions of this one are all on their way)
        if (p + kDepth < P || s + 1 < nblk) bufU[p % kDepth] = *(const v4f*)(Ub + uld + uoff);
        if (p + kDepth + 1 == P) {
          ublk += 1024;                                // next 16-channel block of U
          uld = ublk;
        } else {
          uld += up;
        }
        asm volatile("" : "+s"(uld));
      }
      // two positions interleaved: consecutive MFMAs never wait for each other's result
      acc[p0] = __builtin_amdgcn_mfma_f32_16x16x4f32(au[0].x, bv[0].x, acc[p0], 0, 0, 0);
      acc[p0 + 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(au[1].x, bv[1].x, acc[p0 + 1], 0, 0, 0);
      acc[p0] = __builtin_amdgcn_mfma_f32_16x16x4f32(au[0].y, bv[0].y, acc[p0], 0, 0, 0);
      acc[p0 + 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(au[1].y, bv[1].y, acc[p0 + 1], 0, 0, 0);
      acc[p0] = __builtin_amdgcn_mfma_f32_16x16x4f32(au[0].z, bv[0].z, acc[p0], 0, 0, 0);
      acc[p0 + 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(au[1].z, bv[1].z, acc[p0 + 1], 0, 0, 0);
      acc[p0] = __builtin_amdgcn_mfma_f32_16x16x4f32(au[0].w, bv[0].w, acc[p0], 0, 0, 0);
      acc[p0 + 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(au[1].w, bv[1].w, acc[p0 + 1], 0, 0, 0);
      // Scheduling groups, in this order: the two LDS reads and the two U loads issued
      // above (operands of later positions), then this pair's eight MFMAs.  Left to
      // itself the scheduler sinks every operand load to just before its use, which
      // undoes the rings and leaves the matrix pipe idle for each load's latency.
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    }
    if (s == 0) WINO_TSF(15);
    lds_barrier();                                     // barrier 2 of step s
    if (s == 0) WINO_TSF(2);
    if (s == 1) WINO_TSF(3);
  }
  }
  WINO_TSF(4);

  // lane holds M[., tile r, k] for k = kb + wave*16 + grp*4 + rr
  const int rs = (int)fast_div(r, pl.inv_twb), twl = r - rs * TWB;
  const int rr_ = r0 + rs, tw = tw0 + twl, k0 = kb + wave * 16 + grp * 4;
  if (rs < RB && rr_ < R && tw < g.TW && k0 < g.K) {
    const int img = (int)fast_div(rr_, pl.inv_th), th = rr_ - img * g.TH;
    finish_lane<M, false, kSparse, false, kFast>(g, at, acc, y, img, th, tw, k0, 0.0f, 0.0f, 0.0f);
  }
  WINO_TSF(5);
}

// The fp32 input stage alone (V to memory, for the unfused sequences): the same staging
// and per-(tile, channel) transform as the producers above, one 16-channel block per
// workgroup.  Grid: x = blocks of RB tile rows, y = blocks of TWB tiles, z = Cp / 16.
template <int M, bool kSparse>
__global__ __launch_bounds__(256) void input_transform_f32_staged(const float* __restrict__ x,
                                                                  float* __restrict__ V, Geom g,
                                                                  FPlan pl, MatBT bt) {
  constexpr int n = M + 2, P = n * n, CB = 16;
  extern __shared__ __attribute__((aligned(16))) float ldsf[];
  float* Xs = ldsf;                                    // [16 channels][plane]
  int* rowinfo = (int*)(ldsf + CB * pl.plane);         // [rows]
  const int RB = pl.RB, TWB = pl.TWB, Wc = pl.Wc, rows = pl.rows, plane = pl.plane;
  const int r0 = blockIdx.x * RB, tw0 = blockIdx.y * TWB, cbase = blockIdx.z * CB;
  const int R = g.N * g.TH, HW = g.H * g.W;
  const int tid = threadIdx.x;
  if (tid < rows) {
    const int rs = tid / n, j = tid - rs * n;
    const int rr = r0 + rs;
    const int rc = rr < R ? rr : R - 1;
    const int img = (int)fast_div(rc, pl.inv_th), th = rc - img * g.TH;
    const int h = th * M - g.pad + j;
    rowinfo[tid] = (rr < R && h >= 0 && h < g.H) ? (img * g.C * g.H + h) * g.W : -1;
  }
  __syncthreads();
  const int wbase = tw0 * M - g.pad;
  const float* xb = x + (size_t)cbase * HW;
  constexpr int kBatch = 8;
  for (int i0 = 0; i0 < pl.iters; i0 += kBatch) {
    float v[kBatch];
    int dst[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int e = tid + (i0 + u) * 256;
      const int ec = e < pl.total ? e : pl.total - 1;
      const int rowidx = (int)fast_div(ec, pl.inv_wc), col = ec - rowidx * Wc;
      const int c = (int)fast_div(rowidx, pl.inv_rows), rj = rowidx - c * rows;
      const int info = rowinfo[rj];
      const int w = wbase + col;
      const bool ok = info >= 0 && w >= 0 && w < g.W && cbase + c < g.C;
      const float f = xb[ok ? info + c * HW + w : 0];
      v[u] = ok ? f : 0.0f;
      dst[u] = c * plane + rj * Wc + col;              // surplus lanes repeat the last element
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) Xs[dst[u]] = v[u];
  }
  __syncthreads();
  const int c2 = tid & 15, tl = tid >> 4;
  const int rs2 = (int)fast_div(tl, pl.inv_twb), twl2 = tl - rs2 * TWB;
  const int rr = r0 + rs2, tw = tw0 + twl2;
  if (rs2 >= RB || rr >= R || tw >= g.TW) return;
  const float* patch = Xs + c2 * plane + (rs2 * n) * Wc + twl2 * M;
  float d[n][n], Vt[n][n];
#pragma unroll
  for (int j = 0; j < n; ++j)
#pragma unroll
    for (int l = 0; l < n; ++l) d[j][l] = patch[j * Wc + l];
  transform_patch<M, kSparse>(d, bt, Vt);
  const size_t pstride = (size_t)g.Tp * g.Cp;
  float* vp = V + ((size_t)rr * g.TW + tw) * g.Cp + cbase + c2;
#pragma unroll
  for (int p = 0; p < P; ++p) vp[p * pstride] = Vt[p / n][p % n];
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
  const size_t lds_floats = (size_t)2 * P * 256 + (size_t)16 * pl.plane + 4 + pl.rows;
  *lds_bytes = lds_floats * 4;
  *ntwb = (g.TW + pl.TWB - 1) / pl.TWB;
  *nrb = (R + pl.RB - 1) / pl.RB;
  // 32 = the largest kIters of the fused kernel; its packed LDS index has 16 bits;
  // 160 KB of LDS per workgroup on gfx950
  return lds_floats <= 65536 && *lds_bytes <= 160 * 1024 && *ntwb <= 65535 &&
         g.Kp / 64 <= 65535 && pl.rows <= 256 && pl.iters <= 32;
}

template <int M>
hipError_t launch_input_staged_m(const Geom& g, const MatBT& bt, const float* x, float* V,
                                 hipStream_t s) {
  FPlan pl;
  size_t lb_fused;
  int nrb, ntwb;
  make_fplan(g, &pl, &lb_fused, &nrb, &ntwb);            // the plan itself; limits checked here
  const size_t lb = ((size_t)16 * pl.plane + pl.rows) * 4;
  if (lb > 65536 || ntwb > 65535 || g.Cp / 16 > 65535 || pl.rows > 256) return hipErrorInvalidValue;
  dim3 grid((unsigned)nrb, (unsigned)ntwb, (unsigned)(g.Cp / 16));
  if (fits_mask(bt.v, g.n * g.n, CookToomMask<M>::bt))
    input_transform_f32_staged<M, true><<<grid, 256, lb, s>>>(x, V, g, pl, bt);
  else
    input_transform_f32_staged<M, false><<<grid, 256, lb, s>>>(x, V, g, pl, bt);
  return hipGetLastError();
}

template <int M, bool kSparse, bool kFast, int kIters, bool kBF = false>
hipError_t launch_k(const Geom& g, const FPlan& pl, size_t lb, dim3 grid, const MatBT& bt,
                    const MatAT& at, const float* x, const float* U, float* y, hipStream_t s) {
  if (lb > 65536) {
    // more dynamic LDS than the default limit: raise it for this kernel (cheap, idempotent)
    const hipError_t e =
        hipFuncSetAttribute((const void*)fused_fwd_f32_kernel<M, kSparse, kFast, kIters, kBF>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lb);
    if (e != hipSuccess) return e;
  }
  fused_fwd_f32_kernel<M, kSparse, kFast, kIters, kBF><<<grid, 512, lb, s>>>(x, U, y, g, pl, bt, at);
  return hipGetLastError();
}

// WINO_BF16: the same launch with bf16 GEMM operands (fewer staging-loop sizes are built)
template <int M>
hipError_t launch_m_bf16(const Geom& g, const MatBT& bt, const MatAT& at, const float* x,
                         const float* U, float* y, hipStream_t s) {
  FPlan pl;
  size_t lb;
  int nrb, ntwb;
  if (!make_fplan(g, &pl, &lb, &nrb, &ntwb)) return hipErrorInvalidValue;
  dim3 grid((unsigned)nrb, (unsigned)ntwb, (unsigned)(g.Kp / 64));
  const bool sparse = fits_mask(bt.v, g.n * g.n, CookToomMask<M>::bt) &&
                      sparse_at<M>(at.v);
  const bool fast = g.Ho % M == 0 && g.Wo % M == 0 && g.K % 4 == 0 && ((uintptr_t)y & 15) == 0;
#define WINO_LAUNCH_BF(SP, FA, IT) \
  return launch_k<M, SP, FA, IT, true>(g, pl, lb, grid, bt, at, x, U, y, s)
  if (sparse && fast) {
    if (pl.iters <= 8) WINO_LAUNCH_BF(true, true, 8);
    if (pl.iters <= 16) WINO_LAUNCH_BF(true, true, 16);
    WINO_LAUNCH_BF(true, true, 32);
  }
  if (sparse) WINO_LAUNCH_BF(true, false, 32);
  if (fast) WINO_LAUNCH_BF(false, true, 32);
  WINO_LAUNCH_BF(false, false, 32);
#undef WINO_LAUNCH_BF
}

template <int M>
hipError_t launch_m(const Geom& g, const MatBT& bt, const MatAT& at, const float* x, const float* U,
                    float* y, hipStream_t s) {
  FPlan pl;
  size_t lb;
  int nrb, ntwb;
  if (!make_fplan(g, &pl, &lb, &nrb, &ntwb)) return hipErrorInvalidValue;
  dim3 grid((unsigned)nrb, (unsigned)ntwb, (unsigned)(g.Kp / 64));
  const bool sparse = fits_mask(bt.v, g.n * g.n, CookToomMask<M>::bt) &&
                      sparse_at<M>(at.v);
  const bool fast = g.Ho % M == 0 && g.Wo % M == 0 && g.K % 4 == 0 && ((uintptr_t)y & 15) == 0;
  // The common case (Cook-Toom pattern, whole tiles) gets the staging loop sized to the
  // shape, in steps of 4 elements per thread; everything else the full 32.
#define WINO_LAUNCH_F32(SP, FA, IT) \
  return launch_k<M, SP, FA, IT>(g, pl, lb, grid, bt, at, x, U, y, s)
  if (sparse && fast) {
    switch ((pl.iters + 3) / 4) {
      case 1: WINO_LAUNCH_F32(true, true, 4);
      case 2: WINO_LAUNCH_F32(true, true, 8);
      case 3: WINO_LAUNCH_F32(true, true, 12);
      case 4: WINO_LAUNCH_F32(true, true, 16);
      case 5: WINO_LAUNCH_F32(true, true, 20);
      case 6: WINO_LAUNCH_F32(true, true, 24);
      case 7: WINO_LAUNCH_F32(true, true, 28);
      default: WINO_LAUNCH_F32(true, true, 32);
    }
  }
  if (sparse) WINO_LAUNCH_F32(true, false, 32);
  if (fast) WINO_LAUNCH_F32(false, true, 32);
  WINO_LAUNCH_F32(false, false, 32);
#undef WINO_LAUNCH_F32
}

}  // namespace

bool fused_fwd_f32_supported(const Geom& g) {
  // fp32, F2 or F4 (the 8 x 8 accumulator sets of F6 leave no room beside the operand
  // rings), few enough output-channel blocks that repeating the input transform per block
  // is cheaper than a round trip of V through memory; 32-bit element offsets into X and
  // byte offsets into U, and exact reciprocals (fastdiv.h) for the tile row index.
  const unsigned long long R = (unsigned long long)g.N * g.TH;
  FPlan pl;
  size_t lb;
  int nrb, ntwb;
  // With fewer than 128 workgroups of 16 tiles a long reduction leaves most of the chip idle
  // for the whole of it: the separate stages (more, smaller workgroups) then measure faster
  // (256 channels, F4, 512 tiles: 69 vs 35 us; at 2 k tiles the two tie).
  if (g.Cp > 128 && g.T < 2048) return false;
  return !g.i8 && (g.m == 2 || g.m == 4) && g.Kp <= 128 && make_fplan(g, &pl, &lb, &nrb, &ntwb) &&
         (unsigned long long)g.N * g.C * g.H * g.W < 0x7fffffffull &&
         (unsigned long long)g.Kp * g.Cp * 4 < 0xffffffffull && R * g.TH < 0x100000000ull;
}

bool fused_fwd_bf16_supported(const Geom& g) {
  // what the kernel can run: F2 or F4, the staging plan within its limits, 32-bit offsets
  const unsigned long long R = (unsigned long long)g.N * g.TH;
  FPlan pl;
  size_t lb;
  int nrb, ntwb;
  return g.bf16 && (g.m == 2 || g.m == 4) && make_fplan(g, &pl, &lb, &nrb, &ntwb) &&
         (unsigned long long)g.N * g.C * g.H * g.W < 0x7fffffffull &&
         (unsigned long long)g.Kp * g.Cp * 2 < 0xffffffffull && R * g.TH < 0x100000000ull;
}

hipError_t launch_fused_fwd_bf16(const Geom& g, const MatBT& bt, const MatAT& at, const void* x,
                                 const void* U, void* y, hipStream_t s) {
  if (!fused_fwd_bf16_supported(g)) return hipErrorInvalidValue;
  if (g.m == 2) return launch_m_bf16<2>(g, bt, at, (const float*)x, (const float*)U, (float*)y, s);
  return launch_m_bf16<4>(g, bt, at, (const float*)x, (const float*)U, (float*)y, s);
}

bool input_f32_staged_supported(const Geom& g) {
  // 32-bit element offsets into X, exact reciprocal for the tile row index, LDS within the
  // default limit (checked again by the launcher)
  const unsigned long long R = (unsigned long long)g.N * g.TH;
  FPlan pl;
  size_t lb;
  int nrb, ntwb;
  make_fplan(g, &pl, &lb, &nrb, &ntwb);
  return !g.i8 && (unsigned long long)g.N * g.C * g.H * g.W < 0x7fffffffull &&
         R * g.TH < 0x100000000ull && ((size_t)16 * pl.plane + pl.rows) * 4 <= 65536 &&
         ntwb <= 65535 && g.Cp / 16 <= 65535 && pl.rows <= 256 &&
         (unsigned long long)pl.total * pl.Wc < 0x100000000ull;
}

hipError_t launch_input_f32_staged(const Geom& g, const MatBT& bt, const void* x, void* V,
                                   hipStream_t s) {
  if (!input_f32_staged_supported(g)) return hipErrorInvalidValue;
  switch (g.m) {
    case 2: return launch_input_staged_m<2>(g, bt, (const float*)x, (float*)V, s);
    case 4: return launch_input_staged_m<4>(g, bt, (const float*)x, (float*)V, s);
    default: return launch_input_staged_m<6>(g, bt, (const float*)x, (float*)V, s);
  }
}

hipError_t launch_fused_fwd_f32(const Geom& g, const MatBT& bt, const MatAT& at, const void* x,
                                const void* U, void* y, hipStream_t s) {
  if (!fused_fwd_f32_supported(g)) return hipErrorInvalidValue;
  if (g.m == 2) return launch_m<2>(g, bt, at, (const float*)x, (const float*)U, (float*)y, s);
  return launch_m<4>(g, bt, at, (const float*)x, (const float*)U, (float*)y, s);
}

}  // namespace wino
