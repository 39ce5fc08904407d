// int8 input transform, shared by the stand-alone kernel and the fully fused forward.
//
// A workgroup owns RB consecutive tile rows (a tile row is one (image, th) pair), TWB
// tiles of each and a block of 64 channels.
//
// Phase 1 (stage_strips) copies the n input rows of every tile row into LDS, transposed
// from the image's NCHW order to pixel-major / channel-minor: LDS dword
// (row, column, cq) holds channels 4cq..4cq+3 of one pixel.  Lanes run along the image
// row, so the global reads are contiguous (for a 32-wide int8 image, whole rows back
// to back); a lane loads the same four pixels of four consecutive channels and
// transposes the 4x4 bytes in registers.  Columns are stored shifted by `pad`, so
// that tile tw starts at LDS column tw*m.
//
// Phase 2 (transform_quad): one thread per (tile, channel quad).  Its n*n LDS reads
// are conflict-free (lanes along cq read consecutive dwords; the pixel pitch kCBQ makes
// the four tiles of a wavefront fall into different banks).  The four channels are
// transformed one after the other and their int8 results packed into one dword per
// Winograd position.
#pragma once
#include <type_traits>

#include "transform_math.h"

namespace wino {

template <int M>
struct InCfg {
  static constexpr int kCBQ = M == 4 ? 18 : 20;   // LDS dwords per pixel (16 used)
};

// LDS columns per staged row (a multiple of 4) and LDS dwords of the staging area,
// including a 4-pixel dump area behind the rows.
__host__ __device__ inline int stage_cols(int M, int TWB) { return (TWB * M + 2 + 3) / 4 * 4; }
template <int M>
__host__ __device__ inline int stage_dwords(int RB, int TWB) {
  return (RB * (M + 2) * stage_cols(M, TWB) + 4) * InCfg<M>::kCBQ;
}

#if defined(__HIPCC__)

struct __attribute__((packed)) UnalignedU32 { uint32_t v; };   // dword at any byte address

__device__ __forceinline__ uint32_t load_quad_guarded(const int8_t* row, int w, int W) {
  // four pixels of one channel row starting at column w; zero outside [0, W).  Branch-free:
  // every byte is loaded from a column clamped into the row and masked afterwards, so all
  // loads of a batch are in flight together.  `row` must point at a row that exists.
  uint32_t v = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int ww = w + e;
    const int wc = ww < 0 ? 0 : (ww >= W ? W - 1 : ww);
    const uint32_t b = (uint32_t)(uint8_t)row[wc];
    v |= (b & (0u - (uint32_t)(ww == wc))) << (8 * e);
  }
  return v;
}

// Phase 1.  A "strip" is the n rows x WQ column quads one channel quad needs for one
// tile row.  Lane -> (slot, row j, column quad lq), fixed for the whole call (one
// division per thread); a pass stages `slots` channel quads.  All loads of a batch of
// passes (8, 4, 2 or 1, as many as remain) are issued before the first is used (a
// workgroup has few wavefronts and nothing else hides the memory latency), and they are
// branch-free: every lane loads a
// dword from an address clamped into its image row, shifts out the bytes that fell
// outside the row and masks rows / channels / tile rows that do not exist.  (Branches
// around the loads or the LDS stores make the compiler sink the loads into them and
// wait for each one separately.)  The caller synchronises afterwards.
// Requires blockDim.x >= n * WQ (the launcher guarantees it).
template <int M, bool kWide>
__device__ __forceinline__ void stage_strips(const Geom& g, const int8_t* __restrict__ x,
                                             uint32_t* lds, int c0, int r0, int tw0, int RB,
                                             int TWB) {
  constexpr int n = M + 2, CBQ = InCfg<M>::kCBQ;
  const int Wc = stage_cols(M, TWB), WQ = Wc >> 2;
  const int R = g.N * g.TH;
  const int wbase = tw0 * M - g.pad;
  const int nthr = blockDim.x, tid = threadIdx.x;
  const int strip = WQ * n;
  const int slots = nthr / strip;
  const int sidx = tid / strip, rem = tid - sidx * strip;
  const int j = rem / WQ, lq = rem - j * WQ;
  const bool lane_on = sidx < slots;
  const int w = wbase + lq * 4;
  const int wl = kWide ? (w < 0 ? 0 : (w > g.W - 4 ? g.W - 4 : w)) : 0;
  // shift by (w - wl) bytes, right if positive, left if negative, zero fill:
  // ((v << 24) >> (24 + 8 (w - wl))) in 64 bits; |w - wl| >= 4 means no overlap
  const int dw = w - wl;
  const bool overlap = !kWide || (dw > -4 && dw < 4);
  const int sh = 24 + 8 * (overlap ? dw : 0);
  const int chs = g.H * g.W;
  const int npass = (16 + slots - 1) / slots;
  uint32_t* dump = lds + RB * n * Wc * CBQ;      // 4*CBQ dwords nobody reads
  for (int rs = 0; rs < RB; ++rs) {
    const int r = r0 + rs;
    const int rc = r < R ? r : R - 1;
    const int img = rc / g.TH, th = rc - img * g.TH;
    const int h = th * M - g.pad + j;
    const int hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h);
    const bool rowok = lane_on && r < R && h == hc && overlap;
    const int8_t* base = x + ((size_t)img * g.C + c0) * chs + (size_t)hc * g.W + wl;
    uint32_t* ldsrow = lds + ((rs * n + j) * Wc + lq * 4) * CBQ;
    // One batch of kB passes: all its loads are issued before the first is used.  (The
    // batch size follows the number of passes, so that a workgroup shape with many slots
    // issues no loads for channel quads beyond the block.)
    auto batch = [&](auto kb_tag, int ps0) {
      constexpr int kBatch = decltype(kb_tag)::value;
      uint32_t q[kBatch][4];
      int off[kBatch][4];                    // byte offset from base; 0 for masked lanes
      uint32_t msk[kBatch][4];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int cq = (ps0 + u) * slots + sidx;
        const bool ok = rowok && cq < 16;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int cl = cq * 4 + e;                     // channel inside the block
          const bool cok = ok && c0 + cl < g.C;
          msk[u][e] = 0u - (uint32_t)cok;
          off[u][e] = (cl * chs) & (int)msk[u][e];
        }
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if constexpr (kWide)
            q[u][e] = ((const UnalignedU32*)(base + off[u][e]))->v;
          else
            q[u][e] = load_quad_guarded(base + off[u][e], w, g.W);
        }
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          q[u][e] = (kWide ? (uint32_t)(((uint64_t)q[u][e] << 24) >> sh) : q[u][e]) & msk[u][e];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int cq = (ps0 + u) * slots + sidx;
        const bool live = lane_on && cq < 16;      // others write to the dump area
        // 4x4 byte transpose: q[e] = pixels 0..3 of channel e -> channels 0..3 of pixel k
        const uint32_t t0 = __builtin_amdgcn_perm(q[u][1], q[u][0], 0x05010400u);  // a0 b0 a1 b1
        const uint32_t t1 = __builtin_amdgcn_perm(q[u][1], q[u][0], 0x07030602u);  // a2 b2 a3 b3
        const uint32_t t2 = __builtin_amdgcn_perm(q[u][3], q[u][2], 0x05010400u);  // c0 d0 c1 d1
        const uint32_t t3 = __builtin_amdgcn_perm(q[u][3], q[u][2], 0x07030602u);  // c2 d2 c3 d3
        uint32_t* dst = live ? ldsrow + cq : dump;
        dst[0 * CBQ] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);                 // a0 b0 c0 d0
        dst[1 * CBQ] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);                 // a1 b1 c1 d1
        dst[2 * CBQ] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
        dst[3 * CBQ] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
      }
    };
    int ps0 = 0;
    for (; ps0 + 8 <= npass; ps0 += 8) batch(std::integral_constant<int, 8>{}, ps0);
    if (npass - ps0 >= 4) { batch(std::integral_constant<int, 4>{}, ps0); ps0 += 4; }
    if (npass - ps0 >= 2) { batch(std::integral_constant<int, 2>{}, ps0); ps0 += 2; }
    if (npass - ps0 >= 1) batch(std::integral_constant<int, 1>{}, ps0);
  }
}

// Phase 2 for one (tile, channel quad), in two steps so that a kernel may reuse the
// staging area between them.  load_quad_patch: src points at the tile's top-left staged
// pixel for this quad.  transform_raw: out[p] receives the four int8 codes of position p
// (channel e in byte e); raw is consumed.
template <int M>
__device__ __forceinline__ void load_quad_patch(const uint32_t* src, int Wc,
                                                uint32_t (&raw)[M + 2][M + 2]) {
  constexpr int n = M + 2, CBQ = InCfg<M>::kCBQ;
#pragma unroll
  for (int j = 0; j < n; ++j)
#pragma unroll
    for (int l = 0; l < n; ++l) raw[j][l] = src[(j * Wc + l) * CBQ];
}

// kPos: one quantizer factor per Winograd position (rvp.r[p]) instead of r_v.
template <int M, bool kSparse, bool kPos = false>
__device__ __forceinline__ void transform_raw(uint32_t (&raw)[M + 2][M + 2], const MatBT& bt,
                                              float r_v, float lo, float hi,
                                              uint32_t (&out)[(M + 2) * (M + 2)],
                                              const PosScale* rvp = nullptr) {
  constexpr int n = M + 2, P = n * n;
#pragma unroll
  for (int p = 0; p < P; ++p) out[p] = 0u;
  // A real loop over the channels (not unrolled): the code stays small enough to be
  // fetched quickly by a launch that runs it only once per wavefront.  Each pass
  // consumes byte 0 of raw and shifts the result into the top byte of out, so after
  // four passes channel e sits in byte e.
#pragma unroll 1
  for (int e = 0; e < 4; ++e) {
    float d[n][n], Vt[n][n];
#pragma unroll
    for (int j = 0; j < n; ++j)
#pragma unroll
      for (int l = 0; l < n; ++l) {
        d[j][l] = (float)(int)(int8_t)(raw[j][l] & 0xff);
        raw[j][l] >>= 8;
      }
    transform_patch<M, kSparse>(d, bt, Vt);
#pragma unroll
    for (int i = 0; i < n; ++i)
#pragma unroll
      for (int k = 0; k < n; ++k) {
        const uint32_t bits = quantize_bits(Vt[i][k], kPos ? rvp->r[i * n + k] : r_v, lo, hi);
        out[i * n + k] = __builtin_amdgcn_perm(bits, out[i * n + k], 0x04030201u);
      }
  }
}

template <int M, bool kSparse, bool kPos = false>
__device__ __forceinline__ void transform_quad(const uint32_t* src, int Wc, const MatBT& bt,
                                               float r_v, float lo, float hi,
                                               uint32_t (&out)[(M + 2) * (M + 2)],
                                               const PosScale* rvp = nullptr) {
  uint32_t raw[M + 2][M + 2];
  load_quad_patch<M>(src, Wc, raw);
  transform_raw<M, kSparse, kPos>(raw, bt, r_v, lo, hi, out, rvp);
}

#endif  // __HIPCC__

}  // namespace wino
