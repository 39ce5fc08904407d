// Device-side arithmetic shared by the transform kernels: the two-sided
// transforms of Eq. 1 (Sec. 3.1) and the stage quantizer (Sec. 3.2, Sec. 5.1).
//
// Arithmetic contract of the int8 mode (what makes an integer result well defined
// for arbitrary real matrices): IEEE fp32; every sum is the chain
// acc = +0; acc = fma(a_j, b_j, acc) over ascending j; the left product of a
// two-sided transform comes first (B^T d, G g, A^T M); a quantizer rounds the exact
// product of its input and its reciprocal step once, half to even, and saturates to
// [-qmax, qmax].
//
// Terms whose matrix entry is exactly zero may be skipped: fma(0, x, acc) == acc
// for finite x (a +0/-0 difference disappears when the integer is taken, and
// compares equal in the float path).  Which entries are zero is a compile-time
// pattern (kSparse kernels); the host selects such a kernel only after checking
// that the caller's matrix really is zero there.  The values always come from the
// kernel arguments.
#pragma once
#include "wino_internal.h"

namespace wino {

// Nonzero structure (bit r*cols + c) of the Cook-Toom matrices built from a point
// list that starts 0, +a, -a, +b, -b, ... and ends with the point at infinity:
// even/odd symmetry of the Lagrange polynomials leaves these zeros whatever the
// values a, b are.
template <int M> struct CookToomMask;
template <> struct CookToomMask<2> {
  static constexpr uint64_t bt = 0xa665ull, at = 0xe7ull;
};
template <> struct CookToomMask<4> {
  static constexpr uint64_t bt = 0xa9e79e795ull, at = 0xf9e79full;
};
template <> struct CookToomMask<6> {
  static constexpr uint64_t bt = 0xaa7e7e7e7e7e7e55ull, at = 0xfe7e7e7e7e7full;
};

template <int M, bool kSparse>
__host__ __device__ constexpr bool bt_nonzero(int i, int j) {
  return !kSparse || ((CookToomMask<M>::bt >> (i * (M + 2) + j)) & 1ull);
}
template <int M, bool kSparse>
__host__ __device__ constexpr bool at_nonzero(int a, int i) {
  return !kSparse || ((CookToomMask<M>::at >> (a * (M + 2) + i)) & 1ull);
}

// Host: true if every entry outside the pattern is exactly zero.
inline bool fits_mask(const float* mat, int count, uint64_t mask) {
  for (int i = 0; i < count; ++i)
    if (!((mask >> i) & 1ull) && mat[i] != 0.0f) return false;
  return true;
}

// First column of row a of A^T that the Cook-Toom pattern leaves nonzero (column 0 for the
// first row, the first nonzero point's column for the others).
template <int M>
__host__ __device__ constexpr int at_lead(int a) {
  for (int i = 0; i < M + 2; ++i)
    if ((CookToomMask<M>::at >> (a * (M + 2) + i)) & 1ull) return i;
  return 0;
}

// Host: A^T has the pattern's zeros AND a leading 1 in every row (x^a at the point x = 1, and
// the row of ones: true of every point list that starts 0, 1, -1).  The kSparse forms of the
// output transform rely on both: a chain's first term fma(1, x, +0) is x itself, so they
// start the chain with x instead of issuing it (at most the sign of a zero differs, which
// no result shows, see above).  Any other A^T takes the dense forms.
template <int M>
inline bool sparse_at(const float* at) {
  if (!fits_mask(at, M * (M + 2), CookToomMask<M>::at)) return false;
  for (int a = 0; a < M; ++a)
    if (at[a * (M + 2) + at_lead<M>(a)] != 1.0f) return false;
  return true;
}

#if defined(__HIPCC__)

// The stage quantizer q = sat(rne(v * r)), product taken exactly and rounded once: the
// fused multiply-add v * r + 1.5 * 2^23 rounds the exact sum to fp32, and in [2^23, 2^24)
// the fp32 numbers are the integers, so for |v r| < 2^22 the result is 1.5 * 2^23 plus the
// integer nearest to v * r, ties to even (1.5 * 2^23 is even).  Beyond that range the sum
// is past the clamp bounds anyway.  The low mantissa bits hold the two's-complement
// integer: bits(1.5 * 2^23 + q) = 0x4B400000 + q.
constexpr float kMagic = 12582912.0f;
constexpr uint32_t kMagicBits = 0x4B400000u;
// ... left in the low bits of a float's bit pattern (lo = kMagic - qmax, hi = kMagic + qmax)
__device__ __forceinline__ uint32_t quantize_bits(float v, float r, float lo, float hi) {
  float u = __builtin_fmaf(v, r, kMagic);
  u = __builtin_amdgcn_fmed3f(u, lo, hi);
  return __float_as_uint(u);
}
// ... as an integer in [-qmax, qmax]
__device__ __forceinline__ int quantize(float v, float r, float qmax) {
  return (int)(quantize_bits(v, r, kMagic - qmax, kMagic + qmax) - kMagicBits);
}
// ... as a float holding that integer
__device__ __forceinline__ float quantize_f(float v, float r, float qmax) {
  return __uint_as_float(quantize_bits(v, r, kMagic - qmax, kMagic + qmax)) - kMagic;
}

// The low bytes of four such bit patterns as one dword, b0 lowest (v_perm_b32: selector
// values 0..3 pick bytes of the second operand, 4..7 bytes of the first, 0x0c is zero).
__device__ __forceinline__ uint32_t pack_codes(uint32_t b0, uint32_t b1, uint32_t b2, uint32_t b3) {
  const uint32_t lo2 = __builtin_amdgcn_perm(b1, b0, 0x0c0c0400u);
  const uint32_t hi2 = __builtin_amdgcn_perm(b3, b2, 0x04000c0cu);
  return __builtin_amdgcn_perm(hi2, lo2, 0x07060100u);
}

// out with byte `e` replaced by the low byte of `bits` (v_perm_b32: selector
// values 0..3 pick bytes of the second operand, 4..7 bytes of the first).
template <int e>
__device__ __forceinline__ uint32_t insert_byte(uint32_t out, uint32_t bits) {
  constexpr uint32_t sel = e == 0 ? 0x03020104u : e == 1 ? 0x03020400u
                         : e == 2 ? 0x03040100u : 0x04020100u;
  return __builtin_amdgcn_perm(bits, out, sel);
}

// One step of a chain z = sum_i A^T[a][i] * f_i in ascending i: z after the term i.  kSparse:
// skipped zeros and the unit leading entry (sparse_at); before the leading entry z is unused.
template <int M, bool kSparse>
__device__ __forceinline__ float at_step(const MatAT& at, int a, int i, float f, float z) {
  constexpr int n = M + 2;
  if constexpr (kSparse) {
    if (i < at_lead<M>(a)) return 0.0f;
    if (i == at_lead<M>(a)) return f;
    if (!at_nonzero<M, true>(a, i)) return z;
    return __builtin_fmaf(at.v[a * n + i], f, z);
  } else {
    return __builtin_fmaf(at.v[a * n + i], f, i == 0 ? 0.0f : z);
  }
}

// V = B^T d B for one n x n patch in registers.
template <int M, bool kSparse>
__device__ __forceinline__ void transform_patch(const float (&d)[M + 2][M + 2], const MatBT& bt,
                                                float (&V)[M + 2][M + 2]) {
  constexpr int n = M + 2;
  float w[n][n];
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int l = 0; l < n; ++l) {
      float acc = 0.0f;
#pragma unroll
      for (int j = 0; j < n; ++j)
        if (bt_nonzero<M, kSparse>(i, j)) acc = __builtin_fmaf(bt.v[i * n + j], d[j][l], acc);
      w[i][l] = acc;
    }
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int k = 0; k < n; ++k) {
      float acc = 0.0f;
#pragma unroll
      for (int l = 0; l < n; ++l)
        if (bt_nonzero<M, kSparse>(k, l)) acc = __builtin_fmaf(w[i][l], bt.v[k * n + l], acc);
      V[i][k] = acc;
    }
}

// U = G g G^T for one 3 x 3 filter.
template <int n>
__device__ __forceinline__ void transform_filter(const float (&gk)[3][3], const MatG& mg,
                                                 float (&U)[n][n]) {
  float t[n][3];
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int b = 0; b < 3; ++b) {
      float acc = 0.0f;
#pragma unroll
      for (int a = 0; a < 3; ++a) acc = __builtin_fmaf(mg.v[i * 3 + a], gk[a][b], acc);
      t[i][b] = acc;
    }
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int j = 0; j < n; ++j) {
      float acc = 0.0f;
#pragma unroll
      for (int b = 0; b < 3; ++b) acc = __builtin_fmaf(t[i][b], mg.v[j * 3 + b], acc);
      U[i][j] = acc;
    }
}

// Yt = A^T Mt A for one (tile, output channel).
template <int M, bool kSparse>
__device__ __forceinline__ void transform_result(const float (&Mt)[M + 2][M + 2], const MatAT& at,
                                                 float (&Y)[M][M]) {
  constexpr int n = M + 2;
  float z[M][n];
#pragma unroll
  for (int a = 0; a < M; ++a)
#pragma unroll
    for (int j = 0; j < n; ++j) {
      float acc = 0.0f;
#pragma unroll
      for (int i = 0; i < n; ++i) acc = at_step<M, kSparse>(at, a, i, Mt[i][j], acc);
      z[a][j] = acc;
    }
#pragma unroll
  for (int a = 0; a < M; ++a)
#pragma unroll
    for (int b = 0; b < M; ++b) {
      float acc = 0.0f;
#pragma unroll
      for (int j = 0; j < n; ++j) acc = at_step<M, kSparse>(at, b, j, z[a][j], acc);
      Y[a][b] = acc;
    }
}

#endif  // __HIPCC__

}  // namespace wino
