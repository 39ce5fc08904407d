// Output side shared by the fused kernels: MFMA accumulator types, the lane-local
// output transform of the four (tile, k) pairs a lane holds after the last Winograd
// position, and the NCHW store of one m x m tile (Eq. 1, Sec. 3.1; quantizer of
// Sec. 3.2).
#pragma once
#include <type_traits>

#include "transform_math.h"

namespace wino {

#if defined(__HIPCC__)

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

template <bool I8> struct Acc { typedef v4i type; };
template <> struct Acc<false> { typedef v4f type; };

// One row of six output codes of F(6x6,3x3) as a dword and a pair instead of three pairs:
// tile columns start at w0 = 6 tw, so a row begins on a dword boundary (even tw: dword at
// w0, pair at w0 + 4) or in mid-dword (odd tw: pair at w0, dword at w0 + 2).  For row
// pitches that are multiples of 4 and planes that start dword-aligned: then a dword, like a
// pair, is inside the image or outside it as a whole.  b0 .. b5: the codes in the low bytes.
__device__ __forceinline__ void store_row6(int8_t* row, int w0, int Wo, uint32_t b0, uint32_t b1,
                                           uint32_t b2, uint32_t b3, uint32_t b4, uint32_t b5) {
  const uint32_t lo4 = pack_codes(b0, b1, b2, b3);
  const uint32_t hi2 = __builtin_amdgcn_perm(b5, b4, 0x0c0c0400u);
  const bool odd = (w0 & 3) != 0;
  const uint32_t dv = odd ? __builtin_amdgcn_alignbit(hi2, lo4, 16) : lo4;
  const uint32_t sv = odd ? lo4 : hi2;
  const int doff = odd ? 2 : 0, soff = odd ? 0 : 4;
  if (w0 + doff + 4 <= Wo) *(uint32_t*)(row + doff) = dv;
  if (w0 + soff + 2 <= Wo) *(uint16_t*)(row + soff) = (uint16_t)sv;
}

// Stores one m x m output tile of channel k; (h0, w0) is its top-left corner.
// kFast: the host has checked that m divides Ho and Wo (every tile is whole and every
// row keeps the alignment of the vector stores; for fp32 also that y itself is 16-byte
// aligned), so no per-lane decisions are left.
template <int M, bool I8, bool kFast = false>
__device__ __forceinline__ void store_tile(const Geom& g, void* __restrict__ yv, size_t plane,
                                           int h0, int w0, const float (&Y)[M][M], float r_y,
                                           float lo, float hi) {
  if (I8) {
    int8_t* y = (int8_t*)yv + plane;
    uint32_t q[M][M];
#pragma unroll
    for (int a = 0; a < M; ++a)
#pragma unroll
      for (int b = 0; b < M; ++b) q[a][b] = quantize_bits(Y[a][b], r_y, lo, hi);
    const bool full = kFast || (h0 + M <= g.Ho && w0 + M <= g.Wo);
    if (kFast || (full && (g.Wo & 1) == 0)) {
      // rows start at even addresses (w0 = tw*m is even): 2-byte stores, or one
      // dword per row when m == 4 and the row pitch keeps it aligned
#pragma unroll
      for (int a = 0; a < M; ++a) {
        int8_t* row = y + (size_t)(h0 + a) * g.Wo + w0;
        bool dword_row = false;
        if constexpr (M == 4) {
          dword_row = kFast || (g.Wo & 3) == 0;
          if (dword_row) {
            uint32_t lo16 = __builtin_amdgcn_perm(q[a][1], q[a][0], 0x0c0c0400u);
            uint32_t hi16 = __builtin_amdgcn_perm(q[a][3], q[a][2], 0x04000c0cu);
            *(uint32_t*)row = lo16 | hi16;
          }
        }
        if (!dword_row) {
#pragma unroll
          for (int b = 0; b < M; b += 2)
            *(uint16_t*)(row + b) =
                (uint16_t)__builtin_amdgcn_perm(q[a][b + 1], q[a][b], 0x0c0c0400u);
        }
      }
    } else if (M == 6 && (g.Wo & 3) == 0 && (((uintptr_t)yv + plane) & 3) == 0) {
      // six codes per row as a dword and a pair (store_row6)
      if constexpr (M == 6) {
#pragma unroll
        for (int a = 0; a < M; ++a)
          if (h0 + a < g.Ho)
            store_row6(y + (size_t)(h0 + a) * g.Wo + w0, w0, g.Wo, q[a][0], q[a][1], q[a][2], q[a][3],
                       q[a][4], q[a][5]);
      }
    } else if ((g.Wo & 1) == 0) {
      // ragged tile, even row pitch: a pair of codes is inside the image or outside it as
      // a whole (w0 is even), so the rows go out in 2-byte stores -- the L1 pays per lane
      // and store, not per byte
#pragma unroll
      for (int a = 0; a < M; ++a)
#pragma unroll
        for (int b = 0; b < M; b += 2)
          if (h0 + a < g.Ho && w0 + b < g.Wo)
            *(uint16_t*)(y + (size_t)(h0 + a) * g.Wo + w0 + b) =
                (uint16_t)__builtin_amdgcn_perm(q[a][b + 1], q[a][b], 0x0c0c0400u);
    } else {
#pragma unroll
      for (int a = 0; a < M; ++a)
#pragma unroll
        for (int b = 0; b < M; ++b)
          if (h0 + a < g.Ho && w0 + b < g.Wo)
            y[(size_t)(h0 + a) * g.Wo + w0 + b] = (int8_t)(q[a][b] & 0xff);
    }
  } else {
    float* y = (float*)yv + plane;
    if constexpr (kFast && (M == 2 || M == 4)) {
      // whole tiles, and the host has checked that y is 16-byte aligned: one vector store
      // per tile row (rows start at multiples of m floats)
#pragma unroll
      for (int a = 0; a < M; ++a) {
        float* row = y + (size_t)(h0 + a) * g.Wo + w0;
        if constexpr (M == 4) {
          *(v4f*)row = v4f{Y[a][0], Y[a][1], Y[a][2], Y[a][3]};
        } else {
          typedef float v2f __attribute__((ext_vector_type(2)));
          *(v2f*)row = v2f{Y[a][0], Y[a][1]};
        }
      }
    } else {
#pragma unroll
      for (int a = 0; a < M; ++a)
#pragma unroll
        for (int b = 0; b < M; ++b)
          if (h0 + a < g.Ho && w0 + b < g.Wo) y[(size_t)(h0 + a) * g.Wo + w0 + b] = Y[a][b];
    }
  }
}


// A lane of the 16x16 MFMA result holds, for one tile, the accumulators of four
// consecutive output channels k0..k0+3 (vector components) of every position:
// transform each of the four n x n matrices and store its tile.
// kMQ: the optional quantizer after the Hadamard stage is on (r_m > 0).
// kFast: whole tiles only (see store_tile), K a multiple of 4 and k0 < K checked by the
// caller (no channel guard here).
// kPos: per-position scales -- every accumulator is first multiplied by the factor of its
// position (wpos[p], real units per unit of the integer product).
template <int M, bool I8, bool kSparse, bool kMQ, bool kFast = false, bool kPos = false>
__device__ __forceinline__ void finish_lane(const Geom& g, const MatAT& at,
                                            const typename Acc<I8>::type (&acc)[(M + 2) * (M + 2)],
                                            void* __restrict__ yv, int img, int th, int tw, int k0,
                                            float r_m, float r_y, float qmax,
                                            const float* wpos = nullptr) {
  constexpr int n = M + 2;
  const float lo = kMagic - qmax, hi = kMagic + qmax;
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    const int k = k0 + rr;
    if (!kFast && k >= g.K) continue;
    float Mt[n][n], Y[M][M];
#pragma unroll
    for (int i = 0; i < n; ++i)
#pragma unroll
      for (int j = 0; j < n; ++j) {
        if constexpr (I8) {
          float f = (float)acc[i * n + j][rr];
          if constexpr (kPos) f *= wpos[i * n + j];
          if constexpr (kMQ) f = quantize_f(f, r_m, qmax);
          Mt[i][j] = f;
        } else {
          Mt[i][j] = acc[i * n + j][rr];
        }
      }
    transform_result<M, kSparse>(Mt, at, Y);
    store_tile<M, I8, kFast>(g, yv, ((size_t)img * g.K + k) * g.Ho * g.Wo, th * M, tw * M, Y, r_y,
                             lo, hi);
  }
}

// The int8 output side with the quantizer options decided at run time (both uniform):
// r_m > 0 turns the Hadamard-stage quantizer on, `pos` the per-position factors w[p].
// One copy of the code per combination, so that none pays for the others' instructions.
template <int M, bool kSparse, bool kFast>
__device__ __forceinline__ void finish_lane_any(const Geom& g, const MatAT& at,
                                                const v4i (&acc)[(M + 2) * (M + 2)],
                                                void* __restrict__ yv, int img, int th, int tw,
                                                int k0, float r_m, float r_y, float qmax,
                                                bool pos, const float* wpos) {
  if (pos) {
    if (r_m > 0.0f)
      finish_lane<M, true, kSparse, true, kFast, true>(g, at, acc, yv, img, th, tw, k0, r_m, r_y, qmax, wpos);
    else
      finish_lane<M, true, kSparse, false, kFast, true>(g, at, acc, yv, img, th, tw, k0, r_m, r_y, qmax, wpos);
  } else {
    if (r_m > 0.0f)
      finish_lane<M, true, kSparse, true, kFast>(g, at, acc, yv, img, th, tw, k0, r_m, r_y, qmax);
    else
      finish_lane<M, true, kSparse, false, kFast>(g, at, acc, yv, img, th, tw, k0, r_m, r_y, qmax);
  }
}

// Stores one m x m tile of output codes; (h0, w0) is its top-left corner in the plane.
// fast (uniform): m divides Ho and Wo and Y is 8-byte aligned, so every tile is whole and
// every tile row is one aligned piece of m codes.
template <int M, typename YT>
__device__ __forceinline__ void store_codes(YT* __restrict__ plane, const Geom& g, int h0, int w0,
                                            const int (&q)[M][M], bool fast) {
  if (fast) {
#pragma unroll
    for (int a = 0; a < M; ++a) {
      YT* row = plane + (size_t)(h0 + a) * g.Wo + w0;
      if constexpr (sizeof(YT) == 2) {
        uint32_t wd[M / 2];
#pragma unroll
        for (int e = 0; e < M / 2; ++e)
          wd[e] = ((uint32_t)q[a][2 * e] & 0xffffu) | ((uint32_t)q[a][2 * e + 1] << 16);
        if constexpr (M == 4) {
          typedef uint32_t v2u __attribute__((ext_vector_type(2)));
          *(v2u*)row = v2u{wd[0], wd[1]};
        } else {
#pragma unroll
          for (int e = 0; e < M / 2; ++e) ((uint32_t*)row)[e] = wd[e];
        }
      } else {
        if constexpr (M == 4) {
          *(uint32_t*)row = ((uint32_t)q[a][0] & 0xffu) | (((uint32_t)q[a][1] & 0xffu) << 8) |
                            (((uint32_t)q[a][2] & 0xffu) << 16) | ((uint32_t)q[a][3] << 24);
        } else {
#pragma unroll
          for (int e = 0; e < M / 2; ++e)
            ((uint16_t*)row)[e] =
                (uint16_t)(((uint32_t)q[a][2 * e] & 0xffu) | (((uint32_t)q[a][2 * e + 1] & 0xffu) << 8));
        }
      }
    }
  } else if (M == 6 && sizeof(YT) == 1 && (g.Wo & 3) == 0 && ((uintptr_t)plane & 3) == 0) {
    // six codes per row as a dword and a pair (store_row6)
    if constexpr (M == 6 && sizeof(YT) == 1) {
#pragma unroll
      for (int a = 0; a < M; ++a)
        if (h0 + a < g.Ho)
          store_row6((int8_t*)plane + (size_t)(h0 + a) * g.Wo + w0, w0, g.Wo, (uint32_t)q[a][0],
                     (uint32_t)q[a][1], (uint32_t)q[a][2], (uint32_t)q[a][3], (uint32_t)q[a][4],
                     (uint32_t)q[a][5]);
    }
  } else if ((g.Wo & 1) == 0 && ((uintptr_t)plane & (2 * sizeof(YT) - 1)) == 0) {
    // ragged tile, even row pitch: a pair of codes is inside the image or outside it as a
    // whole (w0 is even): one store per pair -- the L1 pays per lane and store, not per byte
    typedef typename std::conditional<sizeof(YT) == 2, uint32_t, uint16_t>::type pair_t;
#pragma unroll
    for (int a = 0; a < M; ++a)
#pragma unroll
      for (int b = 0; b < M; b += 2)
        if (h0 + a < g.Ho && w0 + b < g.Wo) {
          constexpr int EB = 8 * (int)sizeof(YT);
          const uint32_t mask = (1u << EB) - 1u;
          *(pair_t*)(plane + (size_t)(h0 + a) * g.Wo + w0 + b) =
              (pair_t)(((uint32_t)q[a][b] & mask) | ((uint32_t)q[a][b + 1] << EB));
        }
  } else {
#pragma unroll
    for (int a = 0; a < M; ++a)
#pragma unroll
      for (int b = 0; b < M; ++b)
        if (h0 + a < g.Ho && w0 + b < g.Wo) plane[(size_t)(h0 + a) * g.Wo + w0 + b] = (YT)q[a][b];
  }
}

#endif  // __HIPCC__

}  // namespace wino
