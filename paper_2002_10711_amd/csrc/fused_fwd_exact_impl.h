// Single-kernel int8 forward for F(2x2,3x3) and F(4x4,3x3) when the input transform is
// EXACT, with the input transform itself on the matrix cores.
//
// If 2^s B^T is an integer matrix (s <= 3; true for Cook-Toom points 0, +-1, +-1/2:
// 4 B^T has entries 0, +-1, +-2, +-4, +-5) and the input holds int8 codes, then every
// partial sum of B^T d B is a small dyadic rational that fp32 represents exactly, so
// the order of evaluation cannot change a bit of it.  The transform of a whole patch
// is then one integer matrix-vector product
//
//     4^s V[(i,k)] = sum_{(j,l)} (2^s B^T[i][j] * 2^s B^T[k][l]) * d[(j,l)]
//
// with int8 factors: a 36 x 64 int8 matrix W (the Kronecker square of 2^s B^T, patch
// index (j,l) padded to 8 x 8) times the 8 x 8 byte window of the image that starts
// at the tile's top-left corner.  v_mfma_i32_16x16x64_i8 does 16 such windows
// (16 channels of one tile) per instruction, three instructions for the 36 positions.
// Window bytes outside the 6 x 6 patch meet zero columns of W, so they need not be
// cleared; only pixels outside the image must be zero.
// The quantizer keeps its definition: V * r_v = (4^s V) * (r_v / 4^s), both exact
// scalings, then round-half-even and saturate (Sec. 3.2, Sec. 5.1).
//
// The rest is the fused forward of fused_fwd.hip: quantized V goes to LDS as the
// channel-contiguous operand of the per-position GEMMs, whose accumulators stay in
// registers for the lane-local output transform.  Per 64 input channels:
//   1. stage n rows x (4 TWB + 4) bytes per channel and tile row into LDS, plain
//      copy in image order (coalesced loads, conflict-free LDS stores);
//   2. every lane gathers its window operands (two 8-byte row pieces per window)
//      into registers; barrier; the staging area is now free and is reused as Vl;
//   3. per window group: 3 MFMAs against W (held in registers, built by the host),
//      windows as the "A" operand so that a lane receives four consecutive channels
//      of one position: quantize, pack into a dword, store into Vl[p][tile][channel];
//   4. barrier; wave w: one MFMA per position against U[p][16 k of w][64 c].
#pragma once
#include <string.h>

#ifndef WINO_EXACT_M
#error "define WINO_EXACT_M (2, 4 or 6): the tile size this translation unit instantiates"
#endif

#include "fastdiv.h"
#include "input_stage.h"
#include "output_stage.h"

// Development aid, compiled only with -DWINO_PROFILE_PHASES (F4 kernels): every wavefront
// records the shader clock at its phase boundaries; wino_debug_read_phases() copies them out.
#if defined(WINO_PROFILE_PHASES) && WINO_EXACT_M == 4
__device__ unsigned long long wino_phase_ts[4096 * 16];
#define WINO_TS(slot)                                                                     \
  if ((threadIdx.x & 63) == 0 && blockIdx.y == 0 && blockIdx.x < 1024)                      \
    wino_phase_ts[(blockIdx.x * 4 + (threadIdx.x >> 6)) * 16 + (slot)] = __builtin_amdgcn_s_memtime()
extern "C" int wino_debug_read_phases(unsigned long long* host, size_t count) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(wino_phase_ts), count * sizeof(unsigned long long));
}
#else
#define WINO_TS(slot)
#endif

namespace wino {
namespace {

// F(2x2,3x3) and F(4x4,3x3): the n x n patch fits the 8 x 8 window and the products of
// the usual matrices fit int8.  F(6x6,3x3) fills the window (n = 8) and its products do not
// fit (4 B^T reaches 21, products 441): there W is split into two int8 digits,
// W = 16 Wh + Wl with Wl in [-8, 7], two MFMAs per block of 16 positions whose results are
// recombined in integers (exact), and the digits are built inside the kernel (two 64 x 64
// byte matrices exceed what kernel arguments can carry): the wavefronts compute one block
// of 16 positions each and hand it to the others through LDS.  Only the stand-alone input
// stage exists for F(6x6,3x3): 64 accumulator sets do not fit a one-kernel forward.

// LDS geometry of the staged input: a row holds the image columns from tw0*m - pad on,
// up to the second dword of the last tile's window (which starts at byte (TWB-1)*m); a
// channel plane is n rows, made odd so that the 16 channels of a window group fall into
// 16 different banks.
// (m = 6: all eight window columns are used and a window may start in mid-dword, so it can
// reach into a third dword)
__host__ __device__ inline int xs_row_dw(int M, int TWB) {
  return (((TWB - 1) * M) >> 2) + (M == 6 ? 3 : 2);
}
__host__ __device__ inline int xs_plane_dw(int M, int TWB) {
  return ((M + 2) * xs_row_dw(M, TWB)) | 1;
}

// Vl: quantized transformed input, [position][tile][64 channels]; the position pitch is
// padded by 4 dwords so that the 16 positions a wavefront stores at once fall into
// different banks.
constexpr int kVlPitch = 16 * 16 + 4;

// The Kronecker matrix W[p][(j,l)] = (2^s B^T)[i][j] * (2^s B^T)[k][l], p = i*6 + k, laid out
// by the host as MFMA operand registers: w[(blk*64 + lane)*4 .. +3] are the 16 bytes
// (j, l) = (2*(lane/16) + b/8, b%8), b = 0..15, of row p = blk*16 + lane%16 (zero for
// p >= 36 and for j, l >= 6).
struct KronW { uint32_t v[3 * 64 * 4]; };
// F(6x6,3x3): the integer matrix 2^s B^T itself; the kernel builds W's digits from it.
struct KronB { int bi[64]; };
template <int M> struct KronArg { typedef KronW type; };
template <> struct KronArg<6> { typedef KronB type; };

// Per-position factors of the two quantizer sites of the fused kernels (n*n <= 36
// positions): rv[p] multiplies the transformed input before rounding (every entry the
// per-tensor factor when there is one scale), w[p] brings accumulator p to real units
// (used only with per-position scales).
struct PosPair { float rv[36]; float w[36]; };

struct __attribute__((packed, aligned(4))) U64A4 { uint32_t lo, hi; };   // 8 bytes, dword aligned

// Launch plan computed by the host.  The reciprocals (fastdiv.h) turn the kernel's few
// integer divisions into one multiply-high each.
struct XPlan {
  int RB, TWB;               // tile rows and tiles per row of a workgroup (RB * TWB <= 16)
  uint32_t inv_twb;          // numerators < 16
  uint32_t inv_strip, inv_wq;   // numerators < 256
  uint32_t inv_th;           // numerators < N * TH
  int w_off;                 // F(6x6,3x3): dword offset in LDS of the digits of W
};

// kLoad: 0 = byte loads (W < 4), 1 = one dword per lane at any byte address,
// 2 = 8 bytes per lane from a dword-aligned address (W % 4 == 0, W >= 8, x aligned),
// 3 = whole image rows: the workgroup spans the full width (TW == kTWB, W == kTWB * m,
// pad == 1, x aligned to min(W, 16) bytes), a lane loads one row of one channel (W bytes,
// consecutive lanes consecutive rows) and shifts it by one byte into its staged form --
// one funnel shift per staged dword instead of a dozen operations.
// kTWB > 0: the workgroup shape (TWB, RB) = (kTWB, 16 / kTWB) is a compile-time constant,
// which folds the index arithmetic; 0 = taken from the plan at run time.
// kThreads: threads of the workgroup (256, or 512 for the 128-output-channel kernel).
template <int M, int kLoad, int kTWB, int kThreads = 256>
__device__ __forceinline__ void stage_planes(const Geom& g, const XPlan& pl,
                                             const int8_t* __restrict__ x, uint32_t* Xs, int c0,
                                             int r0, int tw0) {
  // Same lane mapping and branch-free batched loads as stage_strips (input_stage.h);
  // the dwords are stored as they are: Xs[(rs*64 + c)*plane + j*row + lq].
  constexpr int n = M + 2;
  const int RB = kTWB ? 16 / (kTWB ? kTWB : 1) : pl.RB, TWB = kTWB ? kTWB : pl.TWB;
  const int WQ = xs_row_dw(M, TWB), plane = xs_plane_dw(M, TWB);
  const int R = g.N * g.TH;
  if constexpr (kLoad == 3) {
    static_assert(kLoad != 3 || kTWB > 0, "whole-row staging needs a compile-time shape");
    // bytes per image row: the tiles of a row cover it exactly (m = 2, 4), or, for m = 6,
    // rows of 16, 32, 64 bytes under 4, 8, 16 tile slots (3, 6, 11 tiles and idle slots)
    constexpr int RW = (kTWB ? kTWB : 1) * (M == 6 ? 4 : M);
    constexpr int ND = RW / 4;                         // dwords per image row; WQ >= ND + 1
    constexpr int WQc = (((kTWB ? kTWB : 1) - 1) * M >> 2) + (M == 6 ? 3 : 2);   // = WQ
    constexpr int RBc = 16 / (kTWB ? kTWB : 1);
    constexpr int nrows = RBc * n * 64;                // rows to stage: (rs, channel, j), j fastest
    constexpr int per = (nrows + kThreads - 1) / kThreads;
    uint32_t rw[per][ND];
    uint32_t* dst[per];
    uint32_t* dump = Xs + RB * 64 * plane;             // WQ dwords nobody reads (see make_xlaunch)
#pragma unroll
    for (int i = 0; i < per; ++i) {
      const int id = (int)threadIdx.x + i * kThreads;
      const int idc = (nrows % kThreads == 0 || id < nrows) ? id : nrows - 1;
      const int cj = idc % (n * 64), rs = idc / (n * 64);
      const int c = cj / n, j = cj - c * n;
      const int r = r0 + rs;
      const int rc = r < R ? r : R - 1;
      const int img = (int)fast_div(rc, pl.inv_th), th = rc - img * g.TH;
      const int h = th * M - 1 + j;
      const int hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h);
      const bool ok = r < R && h == hc && c0 + c < g.C;
      const int cc = c0 + c < g.C ? c0 + c : c0;       // a channel that exists
      const int8_t* src = x + (((size_t)img * g.C + cc) * g.H + hc) * RW;
      if constexpr (RW % 16 == 0) {
#pragma unroll
        for (int q = 0; q < RW / 16; ++q) {
          const v4i t = *(const v4i*)(src + 16 * q);
          rw[i][4 * q + 0] = ok ? (uint32_t)t.x : 0u;
          rw[i][4 * q + 1] = ok ? (uint32_t)t.y : 0u;
          rw[i][4 * q + 2] = ok ? (uint32_t)t.z : 0u;
          rw[i][4 * q + 3] = ok ? (uint32_t)t.w : 0u;
        }
      } else if constexpr (RW == 8) {
        typedef uint32_t v2u __attribute__((ext_vector_type(2)));
        const v2u t = *(const v2u*)src;
        rw[i][0] = ok ? t.x : 0u;
        rw[i][1] = ok ? t.y : 0u;
      } else {
        static_assert(RW % 16 == 0 || RW == 8 || RW == 4, "row widths: 4, 8, 16, 32, 64 bytes");
        const uint32_t t = *(const uint32_t*)src;
        rw[i][0] = ok ? t : 0u;
      }
      dst[i] = (nrows % kThreads == 0 || id < nrows) ? Xs + (rs * 64 + c) * plane + j * WQ : dump;
    }
#pragma unroll
    for (int i = 0; i < per; ++i) {
      // staged dword k = image bytes 4k-1 .. 4k+2 (zero outside the row)
#pragma unroll
      for (int k = 0; k < WQc; ++k) {
        const uint32_t hi = k < ND ? rw[i][k] : 0u, lo = (k > 0 && k <= ND) ? rw[i][k - 1] : 0u;
        dst[i][k] = k <= ND ? __builtin_amdgcn_alignbyte(hi, lo, 3) : 0u;
      }
    }
    return;
  }
  const int wbase = tw0 * M - g.pad;
  const int nthr = kThreads, tid = threadIdx.x;
  const int strip = WQ * n;
  const int slots = kTWB ? nthr / strip : (int)fast_div(nthr, pl.inv_strip);
  const int sidx = kTWB ? tid / strip : (int)fast_div(tid, pl.inv_strip), rem = tid - sidx * strip;
  const int j = kTWB ? rem / WQ : (int)fast_div(rem, pl.inv_wq), lq = rem - j * WQ;
  const bool lane_on = sidx < slots;
  const int w = wbase + lq * 4;                    // first of the lane's four image columns
  // wl: column the lane really loads from; the wanted bytes are the loaded ones shifted
  // by (w - wl) bytes (right if positive, left if negative, zero fill).
  int wl = 0, lsh = 0, rsh = 0;
  bool overlap = true;
  if (kLoad == 1) {
    wl = w < 0 ? 0 : (w > g.W - 4 ? g.W - 4 : w);
    overlap = w - wl > -4 && w - wl < 4;
  } else if (kLoad == 2) {
    const int wa = w & ~3;
    wl = wa < 0 ? 0 : (wa > g.W - 8 ? g.W - 8 : wa);
    overlap = w - wl > -4 && w - wl < 8;
  }
  if (kLoad != 0 && overlap) {
    lsh = w < wl ? 8 * (wl - w) : 0;
    rsh = w > wl ? 8 * (w - wl) : 0;
  }
  const int chs = g.H * g.W;
  const int npass = (16 + slots - 1) / slots;      // slots is uniform: scalar division
  const int lane_c = sidx * 4 * chs;               // byte offset of the lane's first channel
  const int pass_c = slots * 4 * chs;              // ... added per pass (uniform)
  constexpr int kBatch = 8;
  uint32_t* dump = Xs + RB * 64 * plane;           // 4 dwords nobody reads
  for (int rs = 0; rs < RB; ++rs) {
    const int r = r0 + rs;
    const int rc = r < R ? r : R - 1;
    const int img = (int)fast_div(rc, pl.inv_th), th = rc - img * g.TH;
    const int h = th * M - g.pad + j;
    const int hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h);
    const bool rowok = lane_on && r < R && h == hc && overlap;
    // uniform base of (image, channel block) + the lane's 32-bit offset inside it
    const int8_t* ibase = x + ((size_t)img * g.C + c0) * chs;
    const int loff = hc * g.W + wl;
    uint32_t* xrow = Xs + (rs * 64) * plane + j * WQ + lq;
    for (int ps0 = 0; ps0 < npass; ps0 += kBatch) {
      uint64_t q[kBatch][4];
      uint32_t msk[kBatch][4];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int cq = (ps0 + u) * slots + sidx;
        const bool ok = rowok && cq < 16;
        const int coff = lane_c + (ps0 + u) * pass_c;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bool cok = ok && c0 + cq * 4 + e < g.C;
          msk[u][e] = 0u - (uint32_t)cok;
          const int off = loff + ((coff + e * chs) & (int)msk[u][e]);
          if constexpr (kLoad == 2) {
            const U64A4 t = *(const U64A4*)(ibase + off);
            q[u][e] = ((uint64_t)t.hi << 32) | t.lo;
          } else if constexpr (kLoad == 1) {
            q[u][e] = ((const UnalignedU32*)(ibase + off))->v;
          } else {
            q[u][e] = load_quad_guarded(ibase + off, w, g.W);
          }
        }
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int cq = (ps0 + u) * slots + sidx;
        const bool live = lane_on && cq < 16;
        uint32_t* dst = live ? xrow + cq * 4 * plane : dump;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          dst[live ? e * plane : 0] = (uint32_t)((q[u][e] << lsh) >> rsh) & msk[u][e];
      }
    }
  }
}

// F(4x4,3x3): P = 36 positions are two full blocks of 16 and a block with 4.  The third
// block's MFMA results occupy columns 0 .. 3 only (lanes with r < 4); quantizing them one
// window group at a time would spend a full set of vector instructions on a quarter of the
// lanes.  The four window groups of one tile (its four blocks of 16 channels) are therefore
// merged first: group c's columns 0 .. 3 move to columns 4c .. 4c + 3 with row-shift moves
// (three per register), and one quantize-and-pack serves all four.  Lane r then holds
// position 32 + r % 4 of channel group r / 4.
__device__ __forceinline__ v4i merge_tail_groups(const v4i& t0, const v4i& t1, const v4i& t2,
                                                 const v4i& t3) {
  v4i m;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    int v = t0[e];
    // update_dpp(old, src, ctrl, row_mask, bank_mask, bound_ctrl): row_shr:n = 0x110 + n;
    // bank b = lanes 4b .. 4b + 3 of every row of 16
    v = __builtin_amdgcn_update_dpp(v, t1[e], 0x114, 0xf, 0x2, false);
    v = __builtin_amdgcn_update_dpp(v, t2[e], 0x118, 0xf, 0x4, false);
    v = __builtin_amdgcn_update_dpp(v, t3[e], 0x11c, 0xf, 0x8, false);
    m[e] = v;
  }
  return m;
}

// Grid: x = blocks of RB tile rows, y = blocks of TWB tiles along a row, z = blocks of 64
// output channels.
// kOneBlock: C <= 64, a single channel block; the accumulators then start life at the
// first per-position MFMA (zero "C" operand) instead of occupying 144 registers during
// staging and transform.
// kFast: whole tiles, K % 4 == 0 (see output_stage.h).
template <int M, bool kSparseA, int kLoad, bool kOneBlock, int kTWB, bool kFast>
__global__ __launch_bounds__(256) void fused_fwd_exact_kernel(
    const int8_t* __restrict__ x, const int8_t* __restrict__ U, void* __restrict__ y, int pos,
    float r_vs, float r_m, float r_y, float qmax, Geom g, XPlan pl, MatAT at, KronW kw,
    PosPair pp) {
  // (pointers and scalars first: they sit next to the geometry in the argument block,
  // so one batch of scalar loads at kernel start brings in everything staging needs)
  constexpr int n = M + 2, P = n * n;
  constexpr int NBLK = (P + 15) / 16;                  // 16-position blocks of the transform
  constexpr int NSTEP = 16 * NBLK;                     // (window group, block) steps per wave
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  uint32_t* Xs = lds;
  uint32_t* Vl = lds;                                  // aliases Xs
  const int RB = kTWB ? 16 / (kTWB ? kTWB : 1) : pl.RB, TWB = kTWB ? kTWB : pl.TWB;
  const int WQ = xs_row_dw(M, TWB), plane = xs_plane_dw(M, TWB);
  const int r0 = blockIdx.x * RB, tw0 = blockIdx.y * TWB, kb = blockIdx.z * 64;
  const int R = g.N * g.TH;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, grp = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps tile math scalar
  const float lo = kMagic - qmax, hi = kMagic + qmax;

  WINO_TS(0);
  // U rows of this wave: output channels kb + wave*16 + r, 16 bytes at channel grp*16 -- in
  // the blocked layout of the weights (u_byte_index) 1 KB of consecutive bytes per
  // wavefront and channel block; 32-bit offsets from the (uniform) base pointer
  const uint32_t uoff = (uint32_t)((kb + wave * 16) >> 4) * (uint32_t)(g.Cp >> 6) * 1024u +
                        (uint32_t)(grp * 16 + r) * 16u;
  const uint32_t up = (uint32_t)g.Kp * (uint32_t)g.Cp;
  v4i acc[P];
  if constexpr (!kOneBlock) {
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p] = v4i{0, 0, 0, 0};
  }

  // quantizer factor of the positions this lane produces in the transform (p = blk*16 + r)
  float rq[NBLK];
#pragma unroll
  for (int blk = 0; blk < NBLK; ++blk) rq[blk] = r_vs;
  if (pos) {
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) rq[blk] = pp.rv[blk * 16 + r < P ? blk * 16 + r : P - 1];
  }

  const int nblk = kOneBlock ? 1 : (g.Cp >> 6);
  for (int cb = 0; cb < nblk; ++cb) {
    if (cb) __syncthreads();                           // previous block's Vl fully consumed
    WINO_TS(1);
    stage_planes<M, kLoad, kTWB>(g, pl, x, Xs, cb * 64, r0, tw0);
    // the lane's slice of W, as MFMA operand registers (one per 16-position block)
    v4i Wb[NBLK];
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) Wb[blk] = *(const v4i*)&kw.v[(blk * 64 + lane) * 4];
    __syncthreads();
    WINO_TS(2);

    // Window group gi of this wave: tile tl = wave*4 + gi/4, channels (gi%4)*16 .. +15.
    // "A" operand row = channel (gi%4)*16 + r: rows 2 grp and 2 grp + 1 of its window,
    // 8 bytes each (rows and columns beyond the n x n patch meet zero entries of W: any
    // staged bytes will do).  The window starts at byte twl*m of the staged row: dword
    // aligned for m = 4, possibly in mid-dword for m = 2 (funnel shift).
    v4i Aw[16];
    {
      const int j0 = 2 * grp < n ? 2 * grp : 0, j1 = 2 * grp + 1 < n ? 2 * grp + 1 : 0;
      const uint32_t* lane_x = Xs + r * plane + j0 * WQ;       // per lane; the rest is uniform
      const int dj = (j1 - j0) * WQ;
#pragma unroll
      for (int t4 = 0; t4 < 4; ++t4) {
        const int tl = wave * 4 + t4;
        int rs = kTWB ? tl / (kTWB ? kTWB : 1) : (int)fast_div(tl, pl.inv_twb);
        const int twl = tl - rs * TWB;
        rs = rs < RB ? rs : 0;                         // tiles beyond RB*TWB: results unused
        const uint32_t* p0 = lane_x + rs * 64 * plane + ((twl * M) >> 2);
        const int sh = (twl * M) & 3;                  // uniform
#pragma unroll
        for (int cg = 0; cg < 4; ++cg) {
          const uint32_t* p1 = p0 + cg * 16 * plane;
          if constexpr (M == 4) {
            Aw[t4 * 4 + cg] = v4i{(int)p1[0], (int)p1[1], (int)p1[dj], (int)p1[dj + 1]};
          } else {
            const uint32_t a0 = __builtin_amdgcn_alignbyte(p1[1], p1[0], sh);
            const uint32_t a1 = __builtin_amdgcn_alignbyte(p1[dj + 1], p1[dj], sh);
            Aw[t4 * 4 + cg] = v4i{(int)a0, (int)p1[1], (int)a1, (int)p1[dj + 1]};
          }
        }
      }
    }
    // All P "A" operands of the per-position GEMMs are fetched during the transform
    // below, one load per pipeline step: that phase is bound by the vector ALU and leaves
    // the memory pipe idle, while the loads (36 KB per wavefront through the L1) would
    // otherwise stall the MFMA loop.
    constexpr int kDepth = P;
    const uint32_t ub = uoff + (uint32_t)cb * 1024u;
    v4i bufU[kDepth];
    __syncthreads();                                   // Xs is free: Vl may overwrite it
    WINO_TS(3);

    // D[channel][position]: a lane gets positions p = blk*16 + r of channels
    // (gi%4)*16 + 4 grp .. + 3, i.e. one dword of Vl per MFMA.
    // Software pipeline over the (group, block) steps: the MFMA of step s + 1 is issued
    // before the results of step s are quantized, so the matrix pipe works while the
    // vector ALU rounds and packs.
    uint32_t* lane_v = Vl + r * kVlPitch + grp;
    v4i cur = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[0], Wb[0], v4i{0, 0, 0, 0}, 0, 0, 0);
    static_assert(NSTEP >= P, "one U load per step must cover all positions");
    if constexpr (M == 4) {
      // two full blocks per window group, the third block once per tile
      // (merge_tail_groups): 32 + 4 steps, one U load each = the 36 positions
      uint32_t* lane_v2 = Vl + (32 + (r & 3)) * kVlPitch + (r >> 2) * 4 + grp;
      const float rq2 = pos ? pp.rv[32 + (r & 3)] : r_vs;
      const v4i zero4 = v4i{0, 0, 0, 0};
      v4i tail[4];
#pragma unroll
      for (int st = 0; st < 32; ++st) {
        const int gi = st >> 1, blk = st & 1, q = gi >> 2;
        bufU[st] = *(const v4i*)(U + (ub + (uint32_t)st * up));
        v4i nxt = cur;
        if (st + 1 < 32)
          nxt = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[(st + 1) >> 1], Wb[(st + 1) & 1], zero4, 0, 0, 0);
        if ((st & 7) >= 2 && (st & 7) < 6)
          tail[(st & 7) - 2] =
              __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[q * 4 + (st & 7) - 2], Wb[2], zero4, 0, 0, 0);
        const uint32_t packed = pack_codes(quantize_bits((float)cur[0], rq[blk], lo, hi),
                                           quantize_bits((float)cur[1], rq[blk], lo, hi),
                                           quantize_bits((float)cur[2], rq[blk], lo, hi),
                                           quantize_bits((float)cur[3], rq[blk], lo, hi));
        const int tl = wave * 4 + q;
        lane_v[blk * 16 * kVlPitch + tl * 16 + (gi & 3) * 4] = packed;
        cur = nxt;
        if ((st & 7) == 7) {
          bufU[32 + q] = *(const v4i*)(U + (ub + (uint32_t)(32 + q) * up));
          const v4i m4 = merge_tail_groups(tail[0], tail[1], tail[2], tail[3]);
          lane_v2[tl * 16] = pack_codes(quantize_bits((float)m4[0], rq2, lo, hi),
                                        quantize_bits((float)m4[1], rq2, lo, hi),
                                        quantize_bits((float)m4[2], rq2, lo, hi),
                                        quantize_bits((float)m4[3], rq2, lo, hi));
        }
      }
    } else {
#pragma unroll
    for (int st = 0; st < NSTEP; ++st) {
      const int gi = st / NBLK, blk = st % NBLK;
      if (st < kDepth) bufU[st] = *(const v4i*)(U + (ub + (uint32_t)st * up));
      v4i nxt = cur;
      if (st + 1 < NSTEP)   // every lane takes part in the MFMA; only the stores are predicated
        nxt = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[(st + 1) / NBLK], Wb[(st + 1) % NBLK],
                                                    v4i{0, 0, 0, 0}, 0, 0, 0);
      // four codes into one dword with three byte permutes
      const uint32_t packed = pack_codes(quantize_bits((float)cur[0], rq[blk], lo, hi),
                                         quantize_bits((float)cur[1], rq[blk], lo, hi),
                                         quantize_bits((float)cur[2], rq[blk], lo, hi),
                                         quantize_bits((float)cur[3], rq[blk], lo, hi));
      const int tl = wave * 4 + (gi >> 2);
      if (blk * 16 + r < P) lane_v[blk * 16 * kVlPitch + tl * 16 + (gi & 3) * 4] = packed;
      cur = nxt;
    }
    }
    __syncthreads();
    WINO_TS(4);

    // The operands of V are read from LDS kAheadV positions ahead of their MFMAs and the
    // order is pinned (left to itself the compiler reads two, waits for them and multiplies:
    // 18 LDS round trips that a lone wavefront per SIMD sits out).
    // (Not for F(2x2,3x3): with its 16 positions the pinned order measured 4 % slower than
    // the compiler's own, 64 -> 64 at 32 x 32, batch 256: 24.3 -> 25.2 us; F(4x4,3x3) on the
    // same layer: 23.0 -> 21.4.)
    const uint32_t* lane_b = Vl + r * 16 + grp * 4;
    constexpr int kAheadV = M == 2 ? 0 : 4;
    v4i bvr[kAheadV ? kAheadV : 1];
#pragma unroll
    for (int p = 0; p < kAheadV && p < P; ++p) bvr[p] = *(const v4i*)(lane_b + p * kVlPitch);
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const v4i au = bufU[p];
      v4i bv;
      if constexpr (kAheadV > 0) {
        bv = bvr[p % (kAheadV ? kAheadV : 1)];
        if (p + kAheadV < P)
          bvr[p % (kAheadV ? kAheadV : 1)] = *(const v4i*)(lane_b + (p + kAheadV) * kVlPitch);
        __builtin_amdgcn_sched_barrier(0);
      } else {
        bv = *(const v4i*)(lane_b + p * kVlPitch);
      }
      if constexpr (kOneBlock)
        acc[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(au, bv, v4i{0, 0, 0, 0}, 0, 0, 0);
      else
        acc[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(au, bv, acc[p], 0, 0, 0);
      if constexpr (kAheadV > 0) __builtin_amdgcn_sched_barrier(0);
    }
  }

  WINO_TS(5);
  const int rs = kTWB ? r / (kTWB ? kTWB : 1) : (int)fast_div(r, pl.inv_twb), twl = r - rs * TWB;
  const int rr_ = r0 + rs, tw = tw0 + twl, k0 = kb + wave * 16 + grp * 4;
  // k0 < K: the channel block is padded to 64, so whole lanes may lie beyond K (the
  // per-channel guard inside finish_lane is compiled out when kFast)
  if (rs < RB && rr_ < R && tw < g.TW && k0 < g.K) {
    const int img = (int)fast_div(rr_, pl.inv_th), th = rr_ - img * g.TH;
    finish_lane_any<M, kSparseA, kFast>(g, at, acc, y, img, th, tw, k0, r_m, r_y, qmax, pos != 0,
                                        pp.w);
  }
  WINO_TS(6);
}


// The same forward for 128 output channels in one workgroup of EIGHT wavefronts (two per
// SIMD): wavefronts 0-3 own output channels 0..63 of the block, 4-7 channels 64..127, and
// all eight share the staging and the transform (two tiles per wavefront), which the
// 64-channel kernel would repeat per block of output channels.  One or two blocks of 64
// input channels (kRegions), each transformed into an LDS region of its own, so that the
// accumulators start life at the per-position MFMAs and the kernel stays within 256
// registers per lane.  Cook-Toom A^T pattern, no quantizer on M, compile-time shape.
// Grid: x = blocks of RB tile rows, y = blocks of TWB tiles along a row, z = blocks of 128
// output channels.
template <int M, int kLoad, int kTWB, int kRegions, bool kFast>
__global__ __launch_bounds__(512) void fused_fwd_exact_wide_kernel(
    const int8_t* __restrict__ x, const int8_t* __restrict__ U, void* __restrict__ y, int pos,
    float r_vs, float r_m, float r_y, float qmax, Geom g, XPlan pl, MatAT at, KronW kw,
    PosPair pp) {
  static_assert(kTWB > 0, "compile-time workgroup shape");
  constexpr int n = M + 2, P = n * n;
  constexpr int NBLK = (P + 15) / 16;
  constexpr int NG = 8;                                // window groups per wavefront: 2 tiles x 4
  constexpr int NSTEP = NG * NBLK;
  constexpr int RB = 16 / kTWB, TWB = kTWB;
  constexpr int WQ = (((kTWB - 1) * M) >> 2) + 2, plane = ((M + 2) * WQ) | 1;
  constexpr int kXsDw = RB * 64 * plane + 20, kVlDw = P * kVlPitch;
  constexpr int kRegionDw = kXsDw > kVlDw ? kXsDw : kVlDw;
  static_assert(kRegionDw % 4 == 0, "regions keep the 16-byte alignment of the operand reads");
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  const int r0 = blockIdx.x * RB, tw0 = blockIdx.y * TWB, kb = blockIdx.z * 128;
  const int R = g.N * g.TH;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, grp = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // 0..7
  const int kw16 = kb + (wave >> 2) * 64 + (wave & 3) * 16;    // first output channel of the wave
  const float lo = kMagic - qmax, hi = kMagic + qmax;
  const uint32_t uoff = (uint32_t)(kw16 >> 4) * (uint32_t)(g.Cp >> 6) * 1024u +
                        (uint32_t)(grp * 16 + r) * 16u;
  const uint32_t up = (uint32_t)g.Kp * (uint32_t)g.Cp;

  v4i Wb[NBLK];
  float rq[NBLK];                                      // see fused_fwd_exact_kernel
#pragma unroll
  for (int blk = 0; blk < NBLK; ++blk) {
    Wb[blk] = *(const v4i*)&kw.v[(blk * 64 + lane) * 4];
    rq[blk] = r_vs;
  }
  if (pos) {
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) rq[blk] = pp.rv[blk * 16 + r < P ? blk * 16 + r : P - 1];
  }

  // U operands of the per-position MFMAs, in the order (position, channel block), through
  // a register ring; the first ring-full is fetched during the last transform phase
  constexpr int Q = P * kRegions;
  constexpr int kDepth = M == 4 ? 12 : 8;
  static_assert(Q % kDepth == 0, "ring depth must divide the operand sequence");
  v4i bufU[kDepth];

#pragma unroll
  for (int cb = 0; cb < kRegions; ++cb) {
    uint32_t* Xs = lds + cb * kRegionDw;
    uint32_t* Vl = Xs;                                 // the region's V overwrites its staging
    stage_planes<M, kLoad, kTWB, 512>(g, pl, x, Xs, cb * 64, r0, tw0);
    __syncthreads();
    v4i Aw[NG];
    {
      const int j0 = 2 * grp < n ? 2 * grp : 0, j1 = 2 * grp + 1 < n ? 2 * grp + 1 : 0;
      const uint32_t* lane_x = Xs + r * plane + j0 * WQ;
      const int dj = (j1 - j0) * WQ;
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        const int tl = wave * 2 + t2;
        const int rs = tl / kTWB, twl = tl - rs * kTWB;
        const uint32_t* p0 = lane_x + rs * 64 * plane + ((twl * M) >> 2);
        const int sh = (twl * M) & 3;
#pragma unroll
        for (int cg = 0; cg < 4; ++cg) {
          const uint32_t* p1 = p0 + cg * 16 * plane;
          if constexpr (M == 4) {
            Aw[t2 * 4 + cg] = v4i{(int)p1[0], (int)p1[1], (int)p1[dj], (int)p1[dj + 1]};
          } else {
            const uint32_t a0 = __builtin_amdgcn_alignbyte(p1[1], p1[0], sh);
            const uint32_t a1 = __builtin_amdgcn_alignbyte(p1[dj + 1], p1[dj], sh);
            Aw[t2 * 4 + cg] = v4i{(int)a0, (int)p1[1], (int)a1, (int)p1[dj + 1]};
          }
        }
      }
    }
    __syncthreads();                                   // the region's staging is free
    if (cb == kRegions - 1) {
#pragma unroll
      for (int q = 0; q < kDepth; ++q)
        bufU[q] = *(const v4i*)(U + (uoff + (uint32_t)(q % kRegions) * 1024u +
                                     (uint32_t)(q / kRegions) * up));
    }
    uint32_t* lane_v = Vl + r * kVlPitch + grp;
    v4i cur = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[0], Wb[0], v4i{0, 0, 0, 0}, 0, 0, 0);
    if constexpr (M == 4) {
      // two full blocks per window group, the third block once per tile (merge_tail_groups)
      uint32_t* lane_v2 = Vl + (32 + (r & 3)) * kVlPitch + (r >> 2) * 4 + grp;
      const float rq2 = pos ? pp.rv[32 + (r & 3)] : r_vs;
      const v4i zero4 = v4i{0, 0, 0, 0};
      v4i tail[4];
#pragma unroll
      for (int st = 0; st < 2 * NG; ++st) {
        const int gi = st >> 1, blk = st & 1, q = gi >> 2;
        v4i nxt = cur;
        if (st + 1 < 2 * NG)
          nxt = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[(st + 1) >> 1], Wb[(st + 1) & 1], zero4, 0, 0, 0);
        if ((st & 7) >= 2 && (st & 7) < 6)
          tail[(st & 7) - 2] =
              __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[q * 4 + (st & 7) - 2], Wb[2], zero4, 0, 0, 0);
        const uint32_t packed = pack_codes(quantize_bits((float)cur[0], rq[blk], lo, hi),
                                           quantize_bits((float)cur[1], rq[blk], lo, hi),
                                           quantize_bits((float)cur[2], rq[blk], lo, hi),
                                           quantize_bits((float)cur[3], rq[blk], lo, hi));
        const int tl = wave * 2 + q;
        lane_v[blk * 16 * kVlPitch + tl * 16 + (gi & 3) * 4] = packed;
        cur = nxt;
        if ((st & 7) == 7) {
          const v4i m4 = merge_tail_groups(tail[0], tail[1], tail[2], tail[3]);
          lane_v2[tl * 16] = pack_codes(quantize_bits((float)m4[0], rq2, lo, hi),
                                        quantize_bits((float)m4[1], rq2, lo, hi),
                                        quantize_bits((float)m4[2], rq2, lo, hi),
                                        quantize_bits((float)m4[3], rq2, lo, hi));
        }
      }
    } else {
#pragma unroll
    for (int st = 0; st < NSTEP; ++st) {
      const int gi = st / NBLK, blk = st % NBLK;
      v4i nxt = cur;
      if (st + 1 < NSTEP)
        nxt = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[(st + 1) / NBLK], Wb[(st + 1) % NBLK],
                                                    v4i{0, 0, 0, 0}, 0, 0, 0);
      // four codes into one dword with three byte permutes
      const uint32_t packed = pack_codes(quantize_bits((float)cur[0], rq[blk], lo, hi),
                                         quantize_bits((float)cur[1], rq[blk], lo, hi),
                                         quantize_bits((float)cur[2], rq[blk], lo, hi),
                                         quantize_bits((float)cur[3], rq[blk], lo, hi));
      const int tl = wave * 2 + (gi >> 2);
      if (blk * 16 + r < P) lane_v[blk * 16 * kVlPitch + tl * 16 + (gi & 3) * 4] = packed;
      cur = nxt;
    }
    }
  }
  __syncthreads();

  v4i acc[P];
  // (the operands of V are read from LDS kAheadV steps ahead of their MFMAs, as in the
  // four-wavefront kernel, and like there not for F(2x2,3x3))
  const uint32_t* lane_b = lds + r * 16 + grp * 4;
  constexpr int kAheadV = M == 2 ? 0 : 4;
  v4i bvr[kAheadV ? kAheadV : 1];
#pragma unroll
  for (int q = 0; q < kAheadV && q < Q; ++q)
    bvr[q] = *(const v4i*)(lane_b + (q % kRegions) * kRegionDw + (q / kRegions) * kVlPitch);
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int p = q / kRegions, cb = q % kRegions;
    const v4i au = bufU[q % kDepth];
    if (q + kDepth < Q)
      bufU[q % kDepth] = *(const v4i*)(U + (uoff + (uint32_t)((q + kDepth) % kRegions) * 1024u +
                                            (uint32_t)((q + kDepth) / kRegions) * up));
    v4i bv;
    if constexpr (kAheadV > 0) {
      bv = bvr[q % (kAheadV ? kAheadV : 1)];
      if (q + kAheadV < Q)
        bvr[q % (kAheadV ? kAheadV : 1)] =
            *(const v4i*)(lane_b + ((q + kAheadV) % kRegions) * kRegionDw +
                          ((q + kAheadV) / kRegions) * kVlPitch);
      __builtin_amdgcn_sched_barrier(0);
    } else {
      bv = *(const v4i*)(lane_b + cb * kRegionDw + p * kVlPitch);
    }
    if (cb == 0)
      acc[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(au, bv, v4i{0, 0, 0, 0}, 0, 0, 0);
    else
      acc[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(au, bv, acc[p], 0, 0, 0);
    if constexpr (kAheadV > 0) __builtin_amdgcn_sched_barrier(0);
  }

  const int rs = r / kTWB, twl = r - rs * kTWB;
  const int rr_ = r0 + rs, tw = tw0 + twl, k0 = kw16 + grp * 4;
  if (rr_ < R && tw < g.TW && k0 < g.K) {
    const int img = (int)fast_div(rr_, pl.inv_th), th = rr_ - img * g.TH;
    finish_lane_any<M, true, kFast>(g, at, acc, y, img, th, tw, k0, r_m, r_y, qmax, pos != 0, pp.w);
  }
}

// The input stage alone, for the layers whose accumulators do not fit the fused kernel
// and for the per-stage calls: same staging, window gather and MFMA transform, then the
// block's V tile goes from LDS to memory in the GEMM's operand order V[p][t][c].
// Grid: x = blocks of RB tile rows, y = blocks of TWB tiles along a row, z = blocks of 64
// input channels.  Tiles of a workgroup that lie beyond the image are not written; the
// rows of V between T and Tp are never read by anything that reaches the output.
// kTPW: tiles per wavefront, 4 or 3.  The workgroup shapes are powers of two, so a row of 3
// or 6 tiles (F(6x6,3x3) on 16 or 32 pixels) leaves 4 of the 16 tile slots empty, and with
// four slots per wavefront the empty ones cost as much as the others.  With kTPW = 3 the at
// most 12 real tiles of the workgroup are dealt out three to a wavefront (the host checks
// that one workgroup spans the tile row and that RB * TW <= 12); V in LDS keeps the slot
// order, so the stores do not change.
template <int M, int kLoad, int kTWB, int kTPW = 4>
__global__ __launch_bounds__(256) void input_transform_exact_kernel(
    const int8_t* __restrict__ x, int8_t* __restrict__ V, PosScale rvs, float qmax, Geom g,
    XPlan pl, typename KronArg<M>::type kw) {
  constexpr int n = M + 2, P = n * n;
  constexpr int NBLK = (P + 15) / 16, NSTEP = 4 * kTPW * NBLK;
  static_assert(kTPW == 4 || (kTPW == 3 && M == 6), "three tiles per wavefront: F(6x6,3x3) only");
  constexpr int ND = M == 6 ? 2 : 1;                   // int8 digits of W
  static_assert(M != 6 || NBLK == 4, "one block of positions per wavefront builds W");
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  uint32_t* Xs = lds;
  uint32_t* Vl = lds;                                  // aliases Xs
  const int RB = kTWB ? 16 / (kTWB ? kTWB : 1) : pl.RB, TWB = kTWB ? kTWB : pl.TWB;
  const int WQ = xs_row_dw(M, TWB), plane = xs_plane_dw(M, TWB);
  const int r0 = blockIdx.x * RB, tw0 = blockIdx.y * TWB, cb = blockIdx.z;
  const int R = g.N * g.TH;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, grp = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const float lo = kMagic - qmax, hi = kMagic + qmax;

  stage_planes<M, kLoad, kTWB>(g, pl, x, Xs, cb * 64, r0, tw0);
  // quantizer factor of the positions this lane produces (p = blk*16 + r): one per
  // position, all equal for a per-tensor scale
  float rq[NBLK];
#pragma unroll
  for (int blk = 0; blk < NBLK; ++blk) rq[blk] = rvs.r[blk * 16 + r < P ? blk * 16 + r : P - 1];
  v4i Wb[NBLK * ND];
  if constexpr (M != 6) {
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) Wb[blk] = *(const v4i*)&kw.v[(blk * 64 + lane) * 4];
  }
  __syncthreads();

  if constexpr (M == 6) {
    // Digits of W, block `wave` (positions p = wave*16 + r: i = p / 8, k = p % 8): the lane's
    // 16 bytes are the patch entries (j, l) = (2 grp + b / 8, b % 8), W = bi[i][j] * bi[k][l],
    // Wh = floor((W + 8) / 16), Wl = W - 16 Wh.  Stored as [block][digit][lane] x 16 bytes.
    const int i = 2 * wave + (r >> 3), k = r & 7;
    int bk[8];
#pragma unroll
    for (int l = 0; l < 8; ++l) bk[l] = kw.bi[k * 8 + l];
    uint32_t wl[4], wh[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const int bij = kw.bi[i * 8 + 2 * grp + (d >> 1)];
      uint32_t ql = 0, qh = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int w = bij * bk[(d & 1) * 4 + e];
        const int h = (w + 8) >> 4;
        qh |= ((uint32_t)h & 0xffu) << (8 * e);
        ql |= ((uint32_t)(w - 16 * h) & 0xffu) << (8 * e);
      }
      wl[d] = ql;
      wh[d] = qh;
    }
    v4i* Wl = (v4i*)(lds + pl.w_off);
    Wl[(wave * 2 + 0) * 64 + lane] = v4i{(int)wl[0], (int)wl[1], (int)wl[2], (int)wl[3]};
    Wl[(wave * 2 + 1) * 64 + lane] = v4i{(int)wh[0], (int)wh[1], (int)wh[2], (int)wh[3]};
  }

  // window operands: see fused_fwd_exact_kernel
  v4i Aw[4 * kTPW];
  int slot[kTPW];                                      // tile slot (rs * TWB + twl) of the wave's tiles
  {
    const int j0 = 2 * grp < n ? 2 * grp : 0, j1 = 2 * grp + 1 < n ? 2 * grp + 1 : 0;
    const uint32_t* lane_x = Xs + r * plane + j0 * WQ;
    const int dj = (j1 - j0) * WQ;
#pragma unroll
    for (int t4 = 0; t4 < kTPW; ++t4) {
      int tl = wave * kTPW + t4;
      if constexpr (kTPW != 4) {
        // real tile number v -> slot; v / TW by comparison (at most four tile rows)
        const int v = tl;
        const int vr = (v >= g.TW) + (v >= 2 * g.TW) + (v >= 3 * g.TW);
        tl = vr < RB ? vr * TWB + (v - vr * g.TW) : RB * TWB - 1;   // (past the last: an empty slot)
      }
      slot[t4] = tl;
      int rs = kTWB ? tl / (kTWB ? kTWB : 1) : (int)fast_div(tl, pl.inv_twb);
      const int twl = tl - rs * TWB;
      rs = rs < RB ? rs : 0;
      const uint32_t* p0 = lane_x + rs * 64 * plane + ((twl * M) >> 2);
      const int sh = (twl * M) & 3;
#pragma unroll
      for (int cg = 0; cg < 4; ++cg) {
        const uint32_t* p1 = p0 + cg * 16 * plane;
        if constexpr (M == 4) {
          Aw[t4 * 4 + cg] = v4i{(int)p1[0], (int)p1[1], (int)p1[dj], (int)p1[dj + 1]};
        } else if constexpr (M == 6) {
          // all eight columns count: both dwords of a row are shifted into place
          const uint32_t a0 = __builtin_amdgcn_alignbyte(p1[1], p1[0], sh);
          const uint32_t a1 = __builtin_amdgcn_alignbyte(p1[2], p1[1], sh);
          const uint32_t b0 = __builtin_amdgcn_alignbyte(p1[dj + 1], p1[dj], sh);
          const uint32_t b1 = __builtin_amdgcn_alignbyte(p1[dj + 2], p1[dj + 1], sh);
          Aw[t4 * 4 + cg] = v4i{(int)a0, (int)a1, (int)b0, (int)b1};
        } else {
          const uint32_t a0 = __builtin_amdgcn_alignbyte(p1[1], p1[0], sh);
          const uint32_t a1 = __builtin_amdgcn_alignbyte(p1[dj + 1], p1[dj], sh);
          Aw[t4 * 4 + cg] = v4i{(int)a0, (int)p1[1], (int)a1, (int)p1[dj + 1]};
        }
      }
    }
  }
  __syncthreads();                                     // Xs is free: Vl may overwrite it
  if constexpr (M == 6) {
    const v4i* Wl = (const v4i*)(lds + pl.w_off);
#pragma unroll
    for (int q = 0; q < NBLK * ND; ++q) Wb[q] = Wl[q * 64 + lane];
  }

  uint32_t* lane_v = Vl + r * kVlPitch + grp;
  const v4i zero4 = v4i{0, 0, 0, 0};
  if constexpr (M == 4) {
    // two full blocks per window group, the third block once per tile (merge_tail_groups)
    uint32_t* lane_v2 = Vl + (32 + (r & 3)) * kVlPitch + (r >> 2) * 4 + grp;
    const float rq2 = rvs.r[32 + (r & 3)];
    v4i cur = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[0], Wb[0], zero4, 0, 0, 0);
    v4i tail[4];
#pragma unroll
    for (int st = 0; st < 32; ++st) {
      const int gi = st >> 1, blk = st & 1, q = gi >> 2;
      v4i nxt = cur;
      if (st + 1 < 32)
        nxt = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[(st + 1) >> 1], Wb[(st + 1) & 1], zero4, 0, 0, 0);
      // the tile's third-block MFMAs, one per step in mid-tile, consumed at its end
      if ((st & 7) >= 2 && (st & 7) < 6)
        tail[(st & 7) - 2] =
            __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[q * 4 + (st & 7) - 2], Wb[2], zero4, 0, 0, 0);
      const uint32_t packed = pack_codes(quantize_bits((float)cur[0], rq[blk], lo, hi),
                                         quantize_bits((float)cur[1], rq[blk], lo, hi),
                                         quantize_bits((float)cur[2], rq[blk], lo, hi),
                                         quantize_bits((float)cur[3], rq[blk], lo, hi));
      const int tl = wave * 4 + q;
      lane_v[blk * 16 * kVlPitch + tl * 16 + (gi & 3) * 4] = packed;
      cur = nxt;
      if ((st & 7) == 7) {
        const v4i m4 = merge_tail_groups(tail[0], tail[1], tail[2], tail[3]);
        lane_v2[tl * 16] = pack_codes(quantize_bits((float)m4[0], rq2, lo, hi),
                                      quantize_bits((float)m4[1], rq2, lo, hi),
                                      quantize_bits((float)m4[2], rq2, lo, hi),
                                      quantize_bits((float)m4[3], rq2, lo, hi));
      }
    }
  } else {
  // (two digits: cur / curh hold 4^s V's low and high parts, recombined when consumed)
  v4i cur = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[0], Wb[0], zero4, 0, 0, 0);
  v4i curh = zero4;
  if constexpr (ND == 2) curh = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[0], Wb[1], zero4, 0, 0, 0);
#pragma unroll
  for (int st = 0; st < NSTEP; ++st) {
    const int gi = st / NBLK, blk = st % NBLK;
    v4i nxt = cur, nxth = curh;
    if (st + 1 < NSTEP) {
      nxt = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[(st + 1) / NBLK], Wb[((st + 1) % NBLK) * ND],
                                                  zero4, 0, 0, 0);
      if constexpr (ND == 2)
        nxth = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aw[(st + 1) / NBLK],
                                                     Wb[((st + 1) % NBLK) * ND + 1], zero4, 0, 0, 0);
    }
    if constexpr (ND == 2) cur = (curh << 4) + cur;
    const uint32_t packed = pack_codes(quantize_bits((float)cur[0], rq[blk], lo, hi),
                                       quantize_bits((float)cur[1], rq[blk], lo, hi),
                                       quantize_bits((float)cur[2], rq[blk], lo, hi),
                                       quantize_bits((float)cur[3], rq[blk], lo, hi));
    const int tl = slot[gi >> 2];
    if (blk * 16 + r < P) lane_v[blk * 16 * kVlPitch + tl * 16 + (gi & 3) * 4] = packed;
    cur = nxt;
    curh = nxth;
  }
  }
  __syncthreads();

  // Vl[p][tile][16 dwords] -> V[p][t][cb*64 ..]: a lane moves 16 bytes, a wavefront the 16
  // tiles of one position (1 KB, contiguous in V when the tiles are consecutive and
  // Cp == 64); wave w takes the positions p = w, w + 4, ...
  const int tl = lane >> 2, q4 = lane & 3;
  const int rs = kTWB ? tl / (kTWB ? kTWB : 1) : (int)fast_div(tl, pl.inv_twb), twl = tl - rs * TWB;
  const int rr_ = r0 + rs, tw = tw0 + twl;
  if (rs < RB && rr_ < R && tw < g.TW) {
    const uint32_t t = (uint32_t)rr_ * (uint32_t)g.TW + (uint32_t)tw;
    const uint32_t voff = t * (uint32_t)g.Cp + (uint32_t)cb * 64u + (uint32_t)q4 * 16u;
    const size_t vp = (size_t)g.Tp * g.Cp;
    const uint32_t* src = Vl + tl * 16 + q4 * 4;
    static_assert(P % 4 == 0, "positions are dealt out to four wavefronts");
#pragma unroll
    for (int i = 0; i < P / 4; ++i) {
      const int p = i * 4 + wave;
      *(v4i*)(V + (size_t)p * vp + voff) = *(const v4i*)(src + p * kVlPitch);
    }
  }
}

}  // namespace

#if WINO_EXACT_M == 2   // the shape predicates are defined once
// Images narrower than a dword (W < 4) are staged byte by byte, which exists for the
// two-tile workgroup shape only (W < 4 and pad <= 1 give at most two tiles per row).
static bool narrow_ok(const Geom& g) { return g.W >= 4 || g.TW <= 2; }

// Host: smallest s <= 3 with 2^s B^T integral, all pairwise products within int8, and
// every intermediate of the fp32 evaluation exactly representable (so that integer and
// float evaluation agree bit for bit); -1 if there is none.
int exact_input_shift(const Geom& g, const MatBT& bt) {
  if (!g.i8 || (g.m != 2 && g.m != 4 && g.m != 6)) return -1;
  // products of two entries: one int8 digit for m = 2, 4; two digits (base 16) for m = 6
  const float prodmax = g.m == 6 ? 2031.0f : 127.0f;
  for (int s = 0; s <= 3; ++s) {
    const float sc = (float)(1 << s);
    bool ok = true;
    float amax = 0.0f, rowmax = 0.0f;
    for (int i = 0; i < g.n && ok; ++i) {
      float rowsum = 0.0f;
      for (int j = 0; j < g.n; ++j) {
        const float v = bt.v[i * g.n + j] * sc;
        if (!(v <= 127.0f && v >= -127.0f) || v != (float)(int)v) { ok = false; break; }
        const float a = v < 0 ? -v : v;
        amax = a > amax ? a : amax;
        rowsum += a;
      }
      rowmax = rowsum > rowmax ? rowsum : rowmax;
    }
    if (!ok) continue;
    if (amax * amax > prodmax) return -1;
    // |4^s V| <= 128 * rowmax^2 must stay below 2^24 (fp32 exact integers)
    if (128.0f * rowmax * rowmax >= 16777216.0f) return -1;
    return s;
  }
  return -1;
}

bool input_exact_supported(const Geom& g, const MatBT& bt) {
  // the reciprocal of TH must be exact for every tile row index (see XPlan), and the
  // per-lane offsets into V are 32-bit
  const unsigned long long R = (unsigned long long)g.N * g.TH;
  return R * (unsigned long long)g.TH < 0x100000000ull &&
         (unsigned long long)g.Tp * g.Cp < 0x100000000ull && exact_input_shift(g, bt) >= 0;
}

bool fused_fwd_exact_supported(const Geom& g, const MatBT& bt) {
  // What the one-kernel forward can run (whether it is the fastest sequence for a shape is
  // measured, not decided here: with long reductions it mostly is not -- F4 keeps 144
  // accumulator registers alive through every block's staging and transform, and fewer
  // than 128 workgroups leave most of the chip idle for a whole long reduction).
  // (byte-wise staging is built for a single channel block only)
  return (g.m == 2 || g.m == 4) && g.Kp <= 128 && narrow_ok(g) && (g.W >= 4 || g.Cp == 64) &&
         input_exact_supported(g, bt);
}

// As a stand-alone input stage: wherever the matrix B^T allows it.
bool input_exact_preferred(const Geom& g, const MatBT& bt, const void* x) {
  (void)x;
  return narrow_ok(g) && input_exact_supported(g, bt);
}
#endif

namespace {

// What the host prepares for either kernel: W, the plan, the scaled quantizer factor,
// the LDS size and the grid extents along tile rows and row pieces.
struct XLaunch {
  KronW kw;
  KronB kb;
  XPlan pl;
  float r_vs;
  size_t lds_bytes;
  int nrb, ntwb, load;
};

template <int M>
bool make_xlaunch(const Geom& g, const MatBT& bt, const void* x, float r_v, XLaunch* xl,
                  bool allow_one_tile_rows = false) {
  constexpr int n = M + 2, P = n * n, NBLK = (P + 15) / 16;
  const int sft = exact_input_shift(g, bt);
  if (sft < 0 || !input_exact_supported(g, bt)) return false;
  const float bt_scale = (float)(1 << sft);
  xl->r_vs = r_v / (float)(1 << (2 * sft));              // exact power-of-two scaling
  if (!(xl->r_vs * (float)(1 << (2 * sft)) == r_v)) return false;   // underflow
  // W in MFMA register order (see KronW)
  KronW& kw = xl->kw;
  memset(&kw, 0, sizeof kw);
  int bi[8][8] = {};
  for (int i = 0; i < n; ++i)
    for (int j = 0; j < n; ++j) bi[i][j] = (int)(bt.v[i * n + j] * bt_scale);
  for (int i = 0; i < 8; ++i)
    for (int j = 0; j < 8; ++j) xl->kb.bi[i * 8 + j] = bi[i][j];
  for (int blk = 0; M != 6 && blk < NBLK; ++blk)
    for (int lane = 0; lane < 64; ++lane) {
      const int p = blk * 16 + (lane & 15), kgrp = lane >> 4;
      const int i = p < P ? p / n : 7, k = p < P ? p % n : 7;     // row 7 of bi is zero
      for (int d = 0; d < 4; ++d) {
        uint32_t word = 0;
        for (int e = 0; e < 4; ++e) {
          const int b = d * 4 + e, j = 2 * kgrp + b / 8, l = b % 8;
          word |= (uint32_t)((bi[i][j] * bi[k][l]) & 0xff) << (8 * e);
        }
        kw.v[(blk * 64 + lane) * 4 + d] = word;
      }
    }
  const int R = g.N * g.TH;
  // Workgroup shape: 16 tiles as RB tile rows x TWB tiles per row, TWB the power of two
  // that covers the tile row (16 at most).  Tile slots beyond the image (TWB > TW, tile
  // rows beyond N * TH) are masked everywhere, so every shape is one of four, all known
  // at compile time.
  // (the stand-alone input stage of F2 and F4 also has a 16 x 1 shape for images of one tile
  // per row -- 4 x 4 pixels with F4 -- where the 8 x 2 shape would waste every other slot;
  // for F6 sixteen staged tile rows would not fit the LDS)
  const int TWB = g.TW > 8 ? 16 : g.TW > 4 ? 8 : g.TW > 2 ? 4
                  : (M != 6 && g.TW == 1 && g.W >= 4 && allow_one_tile_rows) ? 1 : 2;
  const int RB = 16 / TWB;
  // (+ 20 dwords: the dump area of surplus staging lanes, up to one staged row)
  const size_t xs_b = ((size_t)RB * 64 * xs_plane_dw(M, TWB) + 20) * 4, vl_b = (size_t)P * kVlPitch * 4;
  xl->lds_bytes = xs_b > vl_b ? xs_b : vl_b;
  XPlan& pl = xl->pl;
  pl.w_off = 0;
  if (M == 6) {
    // the digits of W behind the staging / V region: [4 blocks][2 digits][64 lanes] x 16 bytes
    xl->lds_bytes = (xl->lds_bytes + 15) / 16 * 16;
    pl.w_off = (int)(xl->lds_bytes / 4);
    xl->lds_bytes += 8192;
  }
  xl->ntwb = (g.TW + TWB - 1) / TWB;
  xl->nrb = (R + RB - 1) / RB;
  const int strip = n * xs_row_dw(M, TWB);
  if (xl->lds_bytes > (M == 6 ? 81920u : 65536u) || xl->ntwb > 65535 || strip > 256) return false;
  pl.RB = RB;
  pl.TWB = TWB;
  pl.inv_twb = make_inv(TWB);
  pl.inv_strip = make_inv(strip);
  pl.inv_wq = make_inv(xs_row_dw(M, TWB));
  pl.inv_th = make_inv(g.TH);
  xl->load = g.W < 4 ? 0 : (g.W % 4 == 0 && g.W >= 8 && ((uintptr_t)x & 3) == 0) ? 2 : 1;
  // whole-row staging: the workgroup spans the image width, rows are 8, 16, 32 or 64 bytes
  if (M != 6 && xl->load == 2 && g.pad == 1 && g.TW == TWB && g.W == TWB * M && g.W >= 8 &&
      ((uintptr_t)x & (g.W >= 16 ? 15 : 7)) == 0)
    xl->load = 3;
  // ... F(6x6,3x3): rows of 16, 32 or 64 bytes under 4, 8 or 16 tile slots
  if (M == 6 && xl->load == 2 && g.pad == 1 && g.W == 4 * TWB && g.TW <= TWB && g.W >= 16 &&
      ((uintptr_t)x & 15) == 0)
    xl->load = 3;
  // ... or 4 bytes: images four pixels wide (two tiles of F2 or one of F4 per row)
  if (M != 6 && g.W == 4 && g.pad == 1 && g.TW == TWB && TWB * M == 4 && ((uintptr_t)x & 3) == 0)
    xl->load = 3;
  return true;
}

template <int M>
hipError_t launch_input_m(const Geom& g, const MatBT& bt, const void* x, void* V, float r_v,
                          float qmax, hipStream_t s, const PosScale* rv_pos) {
  XLaunch xl;
  if (!make_xlaunch<M>(g, bt, x, r_v, &xl, true) || g.Cp / 64 > 65535) return hipErrorInvalidValue;
  // per-position factors, each scaled by 4^-s like the per-tensor one (exact, or refuse)
  PosScale rvs;
  const float sc = r_v / xl.r_vs;                        // 4^s, exactly
  for (int p = 0; p < 64; ++p) {
    rvs.r[p] = rv_pos ? rv_pos->r[p] / sc : xl.r_vs;
    if (rv_pos && p < (M + 2) * (M + 2) && !(rvs.r[p] * sc == rv_pos->r[p])) return hipErrorInvalidValue;
  }
  dim3 grid((unsigned)xl.nrb, (unsigned)xl.ntwb, (unsigned)(g.Cp / 64));
  const int8_t* xi = (const int8_t*)x;
  int8_t* Vi = (int8_t*)V;
  const int TWB = xl.pl.TWB;
  typename KronArg<M>::type karg;
  if constexpr (M == 6) karg = xl.kb;
  else karg = xl.kw;
  // (F(6x6,3x3): at most 12 real tiles in a workgroup that spans the tile row: three tiles
  // per wavefront instead of four slots)
  const bool three = M == 6 && xl.ntwb == 1 && xl.pl.RB * g.TW <= 12 && g.TW < TWB;
#define WINO_LAUNCH_IN(LOAD, TWBC)                                                         \
  do {                                                                                     \
    auto kern = input_transform_exact_kernel<M, LOAD, TWBC>;                               \
    if constexpr (M == 6 && TWBC >= 4) {                                                   \
      if (three) kern = input_transform_exact_kernel<M, LOAD, TWBC, 3>;                    \
    }                                                                                      \
    if (xl.lds_bytes > 65536) {                                                            \
      const hipError_t e = hipFuncSetAttribute(                                            \
          (const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)xl.lds_bytes); \
      if (e != hipSuccess) return e;                                                       \
    }                                                                                      \
    kern<<<grid, 256, xl.lds_bytes, s>>>(xi, Vi, rvs, qmax, g, xl.pl, karg);               \
  } while (0)
  // (whole-row staging is built for rows of 4, 8, 16, 32 or 64 bytes; for m = 6: 16, 32, 64)
#define WINO_LAUNCH_IN2(TWBC)                                                              \
  do {                                                                                     \
    if (xl.load == 3) {                                                                    \
      if constexpr (M == 6 ? TWBC >= 4 : (TWBC * M) % 4 == 0) WINO_LAUNCH_IN(3, TWBC);     \
      else return hipErrorInvalidValue;                                                    \
    } else if (xl.load == 2) WINO_LAUNCH_IN(2, TWBC);                                      \
    else WINO_LAUNCH_IN(1, TWBC);                                                          \
  } while (0)
  if (xl.load == 0) {                                    // byte-wise staging: see narrow_ok
    if (TWB != 2) return hipErrorInvalidValue;
    WINO_LAUNCH_IN(0, 2);
  } else if (TWB == 16) WINO_LAUNCH_IN2(16);
  else if (TWB == 8) WINO_LAUNCH_IN2(8);
  else if (TWB == 4) WINO_LAUNCH_IN2(4);
  else if (TWB == 2) WINO_LAUNCH_IN2(2);
  else WINO_LAUNCH_IN2(1);
#undef WINO_LAUNCH_IN2
#undef WINO_LAUNCH_IN
  return hipGetLastError();
}

template <int M>
hipError_t launch_exact_m(const Geom& g, const MatBT& bt, const MatAT& at, const void* x,
                          const void* U, void* y, float r_v, float r_m, float r_y, float qmax,
                          const PosScale* rv_pos, const PosScale* w_pos, hipStream_t s) {
  constexpr int P = (M + 2) * (M + 2);
  XLaunch xl;
  if (!fused_fwd_exact_supported(g, bt) || !make_xlaunch<M>(g, bt, x, r_v, &xl))
    return hipErrorInvalidValue;
  if ((rv_pos == nullptr) != (w_pos == nullptr)) return hipErrorInvalidValue;
  // quantizer factors per position, each scaled by 4^-s like the per-tensor one (exact, or
  // refuse), and the accumulators' factors
  PosPair pp;
  memset(&pp, 0, sizeof pp);
  const float sc = r_v / xl.r_vs;                        // 4^s, exactly
  for (int p = 0; p < P; ++p) {
    pp.rv[p] = rv_pos ? rv_pos->r[p] / sc : xl.r_vs;
    if (rv_pos && !(pp.rv[p] * sc == rv_pos->r[p])) return hipErrorInvalidValue;
    pp.w[p] = w_pos ? w_pos->r[p] : 1.0f;
  }
  const int pos = w_pos != nullptr;
  dim3 grid((unsigned)xl.nrb, (unsigned)xl.ntwb, (unsigned)(g.Kp / 64));
  const XPlan& pl = xl.pl;
  const KronW& kw = xl.kw;
  const size_t lb = xl.lds_bytes;
  const int TWB = pl.TWB, load = xl.load;
  const bool sa = sparse_at<M>(at.v);
  const int8_t* xi = (const int8_t*)x;
  const int8_t* Ui = (const int8_t*)U;
  const bool one = g.Cp == 64;
#define WINO_LAUNCH_XK(SA, LOAD, ONE, TWBC, FAST)                                          \
  fused_fwd_exact_kernel<M, SA, LOAD, ONE, TWBC, FAST><<<grid, 256, lb, s>>>(                \
      xi, Ui, y, pos, xl.r_vs, r_m, r_y, qmax, g, pl, at, kw, pp)
  // The common case -- Cook-Toom A^T pattern, dword staging loads -- gets the compile-time
  // workgroup shapes and, with whole tiles and K % 4 == 0, a branch-free output side.  The
  // quantizer after the Hadamard stage and per-position scales are run-time options of
  // every kernel.
  // (the branch-free output side stores 2 or 4 codes at a time: y must be aligned for that)
  const bool fast = g.Ho % M == 0 && g.Wo % M == 0 && g.K % 4 == 0 && ((uintptr_t)y & 3) == 0;
  // 128 output channels and at most 128 input channels: eight wavefronts share one
  // transform (fused_fwd_exact_wide_kernel)
  if (sa && load >= 2 && g.Kp == 128 && g.Cp <= 128) {
    constexpr int n_ = M + 2, P_ = n_ * n_;
    const int plane_ = xs_plane_dw(M, TWB);
    const size_t xs_dw = (size_t)(16 / TWB) * 64 * plane_ + 20, vl_dw = (size_t)P_ * kVlPitch;
    const int regions = g.Cp / 64;
    const size_t lbw = regions * (xs_dw > vl_dw ? xs_dw : vl_dw) * 4;
    dim3 gridw((unsigned)xl.nrb, (unsigned)xl.ntwb, 1u);
#define WINO_LAUNCH_W(LOAD, TWBC, REG, FAST)                                               \
  do {                                                                                     \
    auto kern = fused_fwd_exact_wide_kernel<M, LOAD, TWBC, REG, FAST>;                      \
    if (lbw > 65536) {                                                                     \
      const hipError_t e = hipFuncSetAttribute(                                            \
          (const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lbw);        \
      if (e != hipSuccess) return e;                                                       \
    }                                                                                      \
    kern<<<gridw, 512, lbw, s>>>(xi, Ui, y, pos, xl.r_vs, r_m, r_y, qmax, g, pl, at, kw, pp);        \
  } while (0)
#define WINO_LAUNCH_W1(LOAD, TWBC, REG) \
  do { if (fast) WINO_LAUNCH_W(LOAD, TWBC, REG, true); else WINO_LAUNCH_W(LOAD, TWBC, REG, false); } while (0)
#define WINO_LAUNCH_W2(LOAD, TWBC) \
  do { if (regions == 2) WINO_LAUNCH_W1(LOAD, TWBC, 2); else WINO_LAUNCH_W1(LOAD, TWBC, 1); } while (0)
#define WINO_LAUNCH_W3(TWBC) \
  do { if (load == 3) WINO_LAUNCH_W2(3, TWBC); else WINO_LAUNCH_W2(2, TWBC); } while (0)
    if (TWB == 16) WINO_LAUNCH_W3(16);
    else if (TWB == 8) WINO_LAUNCH_W3(8);
    else if (TWB == 4) WINO_LAUNCH_W3(4);
    else WINO_LAUNCH_W3(2);
#undef WINO_LAUNCH_W3
#undef WINO_LAUNCH_W2
#undef WINO_LAUNCH_W1
#undef WINO_LAUNCH_W
    return hipGetLastError();
  }
  if (sa && load >= 1) {
#define WINO_LAUNCH_C1(LOAD, TWBC, FAST) \
  do { if (one) WINO_LAUNCH_XK(true, LOAD, true, TWBC, FAST);  \
       else WINO_LAUNCH_XK(true, LOAD, false, TWBC, FAST); } while (0)
#define WINO_LAUNCH_C2(LOAD, TWBC) \
  do { if (fast) WINO_LAUNCH_C1(LOAD, TWBC, true); else WINO_LAUNCH_C1(LOAD, TWBC, false); } while (0)
#define WINO_LAUNCH_C3(TWBC) \
  do { if (load == 3) WINO_LAUNCH_C2(3, TWBC); else if (load == 2) WINO_LAUNCH_C2(2, TWBC); \
       else WINO_LAUNCH_C2(1, TWBC); } while (0)
    if (TWB == 16) WINO_LAUNCH_C3(16);
    else if (TWB == 8) WINO_LAUNCH_C3(8);
    else if (TWB == 4) WINO_LAUNCH_C3(4);
    else WINO_LAUNCH_C3(2);
#undef WINO_LAUNCH_C3
#undef WINO_LAUNCH_C2
#undef WINO_LAUNCH_C1
    return hipGetLastError();
  }
  // everything else (a dense A^T; byte-wise staging): the dense-A^T kernel, its shape read
  // from the plan -- except for byte-wise staging (W < 4), which takes the two-tile shape
  // at compile time, so that it issues no loads for channel quads beyond 16
  if (load == 0) {
    if (TWB != 2) return hipErrorInvalidValue;
    if (one) WINO_LAUNCH_XK(false, 0, true, 2, false);
    else WINO_LAUNCH_XK(false, 0, false, 2, false);
  } else if (load >= 2) {
    if (one) WINO_LAUNCH_XK(false, 2, true, 0, false);
    else WINO_LAUNCH_XK(false, 2, false, 0, false);
  } else {
    if (one) WINO_LAUNCH_XK(false, 1, true, 0, false);
    else WINO_LAUNCH_XK(false, 1, false, 0, false);
  }
#undef WINO_LAUNCH_XK
  return hipGetLastError();
}

}  // namespace

#if WINO_EXACT_M == 6
hipError_t launch_input_exact_m6(const Geom& g, const MatBT& bt, const void* x, void* V, float r_v,
                                 float qmax, hipStream_t s, const PosScale* rv_pos) {
  return launch_input_m<6>(g, bt, x, V, r_v, qmax, s, rv_pos);
}
#elif WINO_EXACT_M == 2
hipError_t launch_input_exact_m2(const Geom& g, const MatBT& bt, const void* x, void* V, float r_v,
                                 float qmax, hipStream_t s, const PosScale* rv_pos) {
  return launch_input_m<2>(g, bt, x, V, r_v, qmax, s, rv_pos);
}
hipError_t launch_fused_fwd_exact_m2(const Geom& g, const MatBT& bt, const MatAT& at, const void* x,
                                     const void* U, void* y, float r_v, float r_m, float r_y,
                                     float qmax, const PosScale* rv_pos, const PosScale* w_pos,
                                     hipStream_t s) {
  return launch_exact_m<2>(g, bt, at, x, U, y, r_v, r_m, r_y, qmax, rv_pos, w_pos, s);
}
#else
hipError_t launch_input_exact_m2(const Geom& g, const MatBT& bt, const void* x, void* V, float r_v,
                                 float qmax, hipStream_t s, const PosScale* rv_pos);
hipError_t launch_input_exact_m6(const Geom& g, const MatBT& bt, const void* x, void* V, float r_v,
                                 float qmax, hipStream_t s, const PosScale* rv_pos);
hipError_t launch_fused_fwd_exact_m2(const Geom& g, const MatBT& bt, const MatAT& at, const void* x,
                                     const void* U, void* y, float r_v, float r_m, float r_y,
                                     float qmax, const PosScale* rv_pos, const PosScale* w_pos,
                                     hipStream_t s);

hipError_t launch_input_exact(const Geom& g, const MatBT& bt, const void* x, void* V, float r_v,
                              float qmax, hipStream_t s, const PosScale* rv_pos) {
  if (g.m == 2) return launch_input_exact_m2(g, bt, x, V, r_v, qmax, s, rv_pos);
  if (g.m == 4) return launch_input_m<4>(g, bt, x, V, r_v, qmax, s, rv_pos);
  if (g.m == 6) return launch_input_exact_m6(g, bt, x, V, r_v, qmax, s, rv_pos);
  return hipErrorInvalidValue;
}

hipError_t launch_fused_fwd_exact(const Geom& g, const MatBT& bt, const MatAT& at, const void* x,
                                  const void* U, void* y, float r_v, float r_m, float r_y,
                                  float qmax, const PosScale* rv_pos, const PosScale* w_pos,
                                  hipStream_t s) {
  if (g.m == 2)
    return launch_fused_fwd_exact_m2(g, bt, at, x, U, y, r_v, r_m, r_y, qmax, rv_pos, w_pos, s);
  if (g.m == 4) return launch_exact_m<4>(g, bt, at, x, U, y, r_v, r_m, r_y, qmax, rv_pos, w_pos, s);
  return hipErrorInvalidValue;
}
#endif

}  // namespace wino
