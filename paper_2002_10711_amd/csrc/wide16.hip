// Wider Winograd domain: the quantized forward with up to 16-bit codes after every stage
// (Sec. 3.2, "quantization diversity": each intermediate of Eq. 1 may have its own
// bit-width; Sec. 5.1 runs INT8, INT10 and INT16; Sec. 7 names wider intermediate stages as
// the way to recover F4/F6 accuracy).
//
// The matrix cores have no 16-bit integer instruction, but int8 at twice the fp16 rate.  A
// code v in [-32767, 32767] is stored as two int8 digits of v - 128,
//
//     v = 256 a + b + 128,   a = floor(v / 256),  b = v mod 256 - 128,   a, b in [-128, 127]
//
// (the offset makes both digits fit: a plain balanced split needs a = 128 for the largest
// codes).  With u~ = u - 128, v~ = v - 128 the per-position GEMM of Sec. 5.3 becomes
//
//     sum_c u v = sum u~ v~ + 128 sum u~ + 128 sum v~ + 16384 Cp,
//     sum u~ v~ = 2^16 sum a_u a_v + 2^8 (sum a_u b_v + sum b_u a_v) + sum b_u b_v,
//
// all sums over the Cp padded channels (padding encodes v = 0 like any other code): four
// v_mfma_i32_16x16x64_i8 per 64 channels for the digit pairs, and four more against an
// operand of ones for sum u~ (per output channel) and sum v~ (per tile), which land in the
// same lanes as the accumulators they correct.  Every partial sum is an exact int32
// (|.| <= 2^15 Cp); the recombination runs in 64-bit integers or in fp64 below 2^53.  The
// result is the exact integer M of the int16 pipeline.
//
// Device layouts of this mode (int8 digit planes, plane 0 = a, plane 1 = b):
//   V [P][2][Tp][Cp]   plain rows, channel fastest
//   U [P][Kp/16][Cp/64][2][64 lanes][16]  1 KB blocks in the order an MFMA wavefront loads
//                      its "A" operand: lane = (c % 64 / 16) * 16 + k % 16 holds 16 channels
//   M [P][Tp][Kp]      int64
// with Tp, Kp, Cp rounded up to 64.
#include <type_traits>

#include "output_stage.h"

namespace wino {
namespace {

typedef uint32_t v4u __attribute__((ext_vector_type(4)));

__host__ __device__ inline size_t u8w_index(int Kp, int Cp, int p, int plane, int k, int c) {
  const size_t blk = ((size_t)p * (Kp >> 4) + (k >> 4)) * (Cp >> 6) + (c >> 6);
  return ((blk * 2 + plane) * 64 + (size_t)(((c & 63) >> 4) * 16 + (k & 15))) * 16 + (c & 15);
}
__host__ __device__ inline size_t v8w_index(int Tp, int Cp, int p, int plane, int t, int c) {
  return (((size_t)p * 2 + plane) * Tp + t) * Cp + c;
}

// v = 256 a + b + 128 on the code as a float (an integer, |v| <= 32767); a, b in [-128, 127]
__device__ __forceinline__ void split_code(float v, int& a, int& b) {
  const float hi = __builtin_floorf(v * 0.00390625f);
  a = (int)hi;
  b = (int)(__builtin_fmaf(hi, -256.0f, v) - 128.0f);
}
__device__ __forceinline__ int join_code(int8_t a, int8_t b) { return (int)a * 256 + (int)b + 128; }

constexpr int kOnes = 0x01010101;                      // sixteen int8 ones: v4i{kOnes, ...}

// M from the seven int32 sums of one (tile, output channel): digit pairs hh, mid
// (= a_u b_v + b_u a_v), ll; digit sums of v~ (sva, svb) and of u~ (sua, sub).
__device__ __forceinline__ long long combine_i64(int hh, int mid, int ll, int sva, int svb,
                                                 int sua, int sub, int Cp) {
  return (long long)hh * 65536 + ((long long)mid + 128ll * ((long long)sva + sua)) * 256 +
         (long long)ll + 128ll * ((long long)svb + sub) + 16384ll * Cp;
}

// Weight stage (Eq. 1: U = G g G^T; quantizer of Sec. 3.2): one thread per (k, c) of the
// padded matrix, codes split into the two digit planes.
template <int M>
__global__ __launch_bounds__(256) void weight_transform_w16(Geom g, MatG mg,
                                                            const float* __restrict__ w,
                                                            int8_t* __restrict__ U, PosScale ru,
                                                            float qmax) {
  constexpr int n = M + 2;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= g.Kp * g.Cp) return;
  const int k = idx / g.Cp, c = idx - k * g.Cp;
  float gk[3][3];
#pragma unroll
  for (int a = 0; a < 3; ++a)
#pragma unroll
    for (int b = 0; b < 3; ++b) gk[a][b] = 0.0f;
  if (k < g.K && c < g.C) {
    const float* src = w + ((size_t)k * g.C + c) * 9;
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
      for (int b = 0; b < 3; ++b) gk[a][b] = src[a * 3 + b];
  }
  float Uf[n][n];
  transform_filter<n>(gk, mg, Uf);
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int j = 0; j < n; ++j) {
      const int p = i * n + j;
      int a, b;
      split_code(quantize_f(Uf[i][j], ru.r[p], qmax), a, b);
      U[u8w_index(g.Kp, g.Cp, p, 0, k, c)] = (int8_t)a;
      U[u8w_index(g.Kp, g.Cp, p, 1, k, c)] = (int8_t)b;
    }
}

// Input stage (Eq. 1: V = B^T d B on every patch, Sec. 3.2): a workgroup owns 8
// consecutive tiles x 32 channels, one (tile, channel) per thread with the tiles along the
// lanes: neighbouring patches overlap, so the eight lanes of a channel read one run of an
// image row (one cache access instead of eight).  The digits go through LDS so that the
// rows of V are written in pieces of 32 bytes.
// kRow: every image row holds at least one load window (W >= 8 elements): a
// lane fetches each of its n patch rows with ONE load of a window clamped into the row and
// shifts the patch out of it, instead of n loads of one element -- the L1 spends its
// cycles per lane and load, not per byte.
template <int M, typename XT, bool kSparse, bool kRow>
__global__ __launch_bounds__(256) void input_transform_w16(Geom g, MatBT bt,
                                                           const XT* __restrict__ x,
                                                           int8_t* __restrict__ V, PosScale rv,
                                                           float qmax) {
  constexpr int n = M + 2, P = n * n;
  constexpr int kPitch = 48;                           // bytes per staged row (32 used)
  __shared__ __attribute__((aligned(16))) int8_t sm[P * 8 * kPitch];
  const int tid = threadIdx.x, r = tid & 7, cc = tid >> 3;
  const int t = blockIdx.x * 8 + r, c = blockIdx.y * 32 + cc;
  float d[n][n];
  {
    // branch-free: every lane loads from an address clamped into an image that exists and
    // zeroes what fell outside (loads under a branch would be waited for one by one)
    const bool live = t < g.T && c < g.C;
    const int tc = t < g.T ? t : g.T - 1, ch = c < g.C ? c : g.C - 1;
    const int tw = tc % g.TW, th = (tc / g.TW) % g.TH, img = tc / (g.TW * g.TH);
    const XT* base = x + ((size_t)img * g.C + ch) * g.H * g.W;
    if constexpr (kRow) {
      constexpr int NW = (sizeof(XT) == 2 && M == 2) ? 4 : 8;   // elements per window (>= n)
      constexpr int EB = 8 * (int)sizeof(XT);          // bits per element
      typedef uint32_t wdw __attribute__((ext_vector_type(NW * sizeof(XT) / 4)));
      struct __attribute__((packed, aligned(sizeof(XT)))) Window { wdw v; };
      const int c0 = tw * M - g.pad;                   // first patch column
      const int ws = c0 < 0 ? 0 : (c0 > g.W - NW ? g.W - NW : c0);
      const int sh = c0 - ws;                          // -1 at the left edge, > 0 at the right
      Window raw[n];
#pragma unroll
      for (int j = 0; j < n; ++j) {
        const int h = th * M - g.pad + j;
        const int hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h);
        raw[j] = *(const Window*)(base + hc * g.W + ws);
      }
      const unsigned rs = sh > 0 ? (unsigned)sh * EB : 0u;          // right shift, bits
#pragma unroll
      for (int j = 0; j < n; ++j) {
        const int h = th * M - g.pad + j;
        const bool hok = live && h >= 0 && h < g.H;
        // the window as one little-endian integer (64 or 128 bits), patch column l at
        // element l + sh: shift right by sh elements (zero fill = columns >= W, because a
        // positive sh means the window ends at the row's end), or left by one (column -1)
        unsigned long long lo, hi = 0;
        if constexpr (sizeof(wdw) == 8) {
          lo = ((unsigned long long)raw[j].v[1] << 32) | raw[j].v[0];
        } else {
          lo = ((unsigned long long)raw[j].v[1] << 32) | raw[j].v[0];
          hi = ((unsigned long long)raw[j].v[3] << 32) | raw[j].v[2];
        }
        const unsigned s1 = rs & 63u;
        const unsigned long long a = rs >= 64 ? hi : lo, b = rs >= 64 ? 0ull : hi;
        unsigned long long r0 = (a >> s1) | (s1 ? b << (64u - s1) : 0ull), r1 = b >> s1;
        if (sh < 0) {
          r1 = (hi << EB) | (lo >> (64 - EB));
          r0 = lo << EB;
        }
#pragma unroll
        for (int l = 0; l < n; ++l) {
          const int bit = l * EB;
          const unsigned long long word = bit < 64 ? r0 >> bit : r1 >> (bit - 64);
          const int e = sizeof(XT) == 2 ? (int)(short)word : (int)(signed char)word;
          d[j][l] = hok ? (float)e : 0.0f;
        }
      }
    } else {
      XT raw[n][n];
#pragma unroll
      for (int j = 0; j < n; ++j) {
        const int h = th * M - g.pad + j;
        const int hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h);
#pragma unroll
        for (int l = 0; l < n; ++l) {
          const int ww = tw * M - g.pad + l;
          const int wc = ww < 0 ? 0 : (ww >= g.W ? g.W - 1 : ww);
          raw[j][l] = base[hc * g.W + wc];
        }
      }
#pragma unroll
      for (int j = 0; j < n; ++j) {
        const int h = th * M - g.pad + j;
        const bool hok = live && h >= 0 && h < g.H;
#pragma unroll
        for (int l = 0; l < n; ++l) {
          const int ww = tw * M - g.pad + l;
          d[j][l] = (hok && ww >= 0 && ww < g.W) ? (float)raw[j][l] : 0.0f;
        }
      }
    }
  }
  float Vf[n][n];
  transform_patch<M, kSparse>(d, bt, Vf);
  // The code c sits in the low 16 bits of the quantizer's bit pattern (two's complement);
  // its digits as bytes: a = floor(c / 256) is byte 1, b = c mod 256 - 128 is byte 0 with
  // its top bit flipped.
  uint32_t code[P];
  const float qlo = kMagic - qmax, qhi = kMagic + qmax;
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int k = 0; k < n; ++k) code[i * n + k] = quantize_bits(Vf[i][k], rv.r[i * n + k], qlo, qhi);
#pragma unroll
  for (int digit = 0; digit < 2; ++digit) {
    if (digit) __syncthreads();                        // the first plane has left LDS
#pragma unroll
    for (int p = 0; p < P; ++p)
      sm[(p * 8 + r) * kPitch + cc] = (int8_t)(digit ? (code[p] ^ 0x80u) : (code[p] >> 8));
    __syncthreads();
    // P * 8 rows of 32 channels = P * 16 pieces of 16 bytes
    for (int idx = tid; idx < P * 16; idx += 256) {
      const int p = idx >> 4, row = (idx & 15) >> 1, piece = idx & 1;
      *(v4u*)(V + v8w_index(g.Tp, g.Cp, p, digit, blockIdx.x * 8 + row,
                            blockIdx.y * 32 + piece * 16)) =
          *(const v4u*)&sm[(p * 8 + row) * kPitch + piece * 16];
    }
  }
}

// Hadamard/GEMM stage (Sec. 5.3: one GEMM per Winograd position, channels summed in the
// Winograd domain), exact in 64-bit integers.  Workgroup = 64 tiles x 64 output channels
// of one position; wavefront = 32 x 32 = 2 x 2 MFMA tiles with three accumulators each
// (the digit pairs) plus the digit sums of its two tile blocks and two channel blocks.
// Operands go straight from global memory into the MFMA, one 64-channel step ahead.
__global__ __launch_bounds__(256) void gemm_w16_kernel(int Tp, int Kp, int Cp,
                                                       const int8_t* __restrict__ V,
                                                       const int8_t* __restrict__ U,
                                                       long long* __restrict__ Mo) {
  const int p = blockIdx.z, tb = blockIdx.x * 64, kb = blockIdx.y * 64;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, grp = lane >> 4;
  const int wave = tid >> 6, wt = wave & 1, wk = wave >> 1;
  const int nch = Cp >> 6;
  const v4i* ua[2][2];
  const v4i* vb[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const int kt = kb + wk * 32 + a * 16;
    const size_t blk = ((size_t)p * (Kp >> 4) + (kt >> 4)) * (Cp >> 6);
#pragma unroll
    for (int dg = 0; dg < 2; ++dg) ua[a][dg] = (const v4i*)(U + (blk * 2 + dg) * 1024) + lane;
  }
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int t = tb + wt * 32 + b * 16 + r;
#pragma unroll
    for (int dg = 0; dg < 2; ++dg)
      vb[b][dg] = (const v4i*)(V + v8w_index(Tp, Cp, p, dg, t, grp * 16));
  }
  // per 64-channel step: U advances by one block pair (2 KB = 128 pieces of 16 bytes), V by
  // 64 bytes = 4 pieces
  v4i A[2][2], B[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int dg = 0; dg < 2; ++dg) {
      A[a][dg] = ua[a][dg][0];
      B[a][dg] = vb[a][dg][0];
    }
  const v4i zero = v4i{0, 0, 0, 0}, ones = v4i{kOnes, kOnes, kOnes, kOnes};
  v4i hh[2][2], mid[2][2], ll[2][2], sv[2][2], su[2][2];       // sv[b][dg], su[a][dg]
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) hh[a][b] = mid[a][b] = ll[a][b] = sv[a][b] = su[a][b] = zero;
  for (int ch = 0; ch < nch; ++ch) {
    const int nx = ch + 1 < nch ? ch + 1 : ch;         // (the last step reloads itself)
    v4i nA[2][2], nB[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int dg = 0; dg < 2; ++dg) {
        nA[a][dg] = ua[a][dg][(size_t)nx * 128];
        nB[a][dg] = vb[a][dg][(size_t)nx * 4];
      }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        hh[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[a][0], B[b][0], hh[a][b], 0, 0, 0);
        mid[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[a][0], B[b][1], mid[a][b], 0, 0, 0);
        mid[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[a][1], B[b][0], mid[a][b], 0, 0, 0);
        ll[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[a][1], B[b][1], ll[a][b], 0, 0, 0);
      }
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int dg = 0; dg < 2; ++dg) {
        sv[x][dg] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, B[x][dg], sv[x][dg], 0, 0, 0);
        su[x][dg] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[x][dg], ones, su[x][dg], 0, 0, 0);
      }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int dg = 0; dg < 2; ++dg) {
        A[a][dg] = nA[a][dg];
        B[a][dg] = nB[a][dg];
      }
  }
  // lane: tile t (column), output channels k0 .. k0 + 3 (rows grp*4 + rr); the digit sums
  // of v~ are the same in every row, those of u~ the same in every column
  typedef long long v2ll __attribute__((ext_vector_type(2)));
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int t = tb + wt * 32 + b * 16 + r, k0 = kb + wk * 32 + a * 16 + grp * 4;
      long long m[4];
#pragma unroll
      for (int rr = 0; rr < 4; ++rr)
        m[rr] = combine_i64(hh[a][b][rr], mid[a][b][rr], ll[a][b][rr], sv[b][0][rr], sv[b][1][rr],
                            su[a][0][rr], su[a][1][rr], Cp);
      long long* dst = Mo + ((size_t)p * Tp + t) * Kp + k0;
      *(v2ll*)dst = v2ll{m[0], m[1]};
      *(v2ll*)(dst + 2) = v2ll{m[2], m[3]};
    }
}

// Output stage (Eq. 1: A^T M A; quantizers of Sec. 3.2 after the Hadamard stage and on the
// output, each with its own range): one thread per (tile, output channel), channels along
// the lanes.
template <int M, typename YT, bool kSparse, bool kPos>
__global__ __launch_bounds__(256) void output_transform_w16(Geom g, MatAT at,
                                                            const long long* __restrict__ Mi,
                                                            YT* __restrict__ y, PosScale w,
                                                            float r_m, float r_y, float qmax_m,
                                                            float qmax_y, int fast) {
  constexpr int n = M + 2;
  const int k = blockIdx.y * 64 + (threadIdx.x & 63), t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= g.T || k >= g.K) return;
  float Mt[n][n], Y[M][M];
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int j = 0; j < n; ++j) {
      const int p = i * n + j;
      float f = (float)Mi[((size_t)p * g.Tp + t) * g.Kp + k];   // correctly rounded
      if (kPos) f = f * w.r[p];
      if (r_m > 0.0f) f = quantize_f(f, r_m, qmax_m);
      Mt[i][j] = f;
    }
  transform_result<M, kSparse>(Mt, at, Y);
  const int tw = t % g.TW, th = (t / g.TW) % g.TH, img = t / (g.TW * g.TH);
  int q[M][M];
#pragma unroll
  for (int a = 0; a < M; ++a)
#pragma unroll
    for (int b = 0; b < M; ++b) q[a][b] = quantize(Y[a][b], r_y, qmax_y);
  store_codes<M, YT>(y + ((size_t)img * g.K + k) * g.Ho * g.Wo, g, th * M, tw * M, q, fast != 0);
}

// Hadamard/GEMM stage and output stage in one kernel: M never reaches memory.  A wavefront
// owns 16 tiles x 16 output channels (the MFMA result: lane = tile, four channels); the
// workgroup's four wavefronts share the tiles.  The Winograd positions are visited column
// by column (j outer, i inner), which lets the output transform run along with them in
// exactly the pinned order: z[a] = fma(A^T[a][i], M[i][j], z[a]) as the accumulators of
// column j arrive (ascending i), then Y[a][b] = fma(z[a], A^T[b][j], Y[a][b]) once the
// column is complete (ascending j).  A lane therefore keeps m + m*m floats per channel
// instead of all n*n accumulators, which leaves room for the seven integer sums of a
// position and a ring of U operands loaded kDepth steps ahead.  The column loop is a real
// loop (it bounds how far the compiler may hoist loads); inside it everything is unrolled,
// so NCH = Cp / 64 is a compile-time constant and the ring slots are static.  kSparse:
// entries of A^T that are zero in the Cook-Toom pattern are skipped along i (compile
// time); along j they are multiplied out (fma(z, 0, Y) == Y).
// V reaches the four wavefronts through LDS: the workgroup loads each position's operands
// once (16 tiles x Cp channels x 2 planes, 16 bytes per thread and load) instead of once
// per wavefront -- the L1's access rate, about 44 cycles per 16-byte-per-lane wavefront
// load, is what bounds such a kernel.  The loads run kPos positions ahead in registers;
// two LDS buffers alternate, one barrier per position.
template <int M, typename YT, int NCH, bool kSparse>
__global__ __launch_bounds__(256) void gemm_out_w16_kernel(Geom g, MatAT at,
                                                           const int8_t* __restrict__ V,
                                                           const int8_t* __restrict__ U,
                                                           YT* __restrict__ y, PosScale w,
                                                           float r_m, float r_y, float qmax_m,
                                                           float qmax_y, int fast) {
  constexpr int n = M + 2;
  constexpr int SJ = n * NCH;                          // steps (64 channels each) per column
  constexpr int kDepth = SJ % 8 == 0 ? 8 : SJ % 6 == 0 ? 6 : 4;  // U ring, in steps
  static_assert(SJ % kDepth == 0 && kDepth <= SJ, "ring depth must divide a column's steps");
  constexpr int kBlocks = NCH * 2;                     // 1 KB operand blocks of V per position
  constexpr int kLd = (kBlocks + 3) / 4;               // 16-byte loads per thread and position
  constexpr int kPos = kLd > 1 ? 2 : NCH >= 2 ? n / 2 : n;        // positions ahead
  static_assert(n % kPos == 0 && n % 2 == 0, "position ring and buffer parity must be static");
  constexpr int kBufPieces = kBlocks * 64;             // 16-byte pieces of one position
  __shared__ v4u vlds[2 * kBufPieces];
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, grp = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tb = blockIdx.x * 16, kb = blockIdx.y * 64;
  const int t = tb + r;
  // Addresses = uniform byte offset (position, channel step: scalar registers, recomputed
  // per load and hidden from the optimiser, which would otherwise keep one 64-bit vector
  // pointer per load site of the unrolled column) + one 32-bit per-lane offset per tensor.
  // U: block pair of (position, 16 channels k, 64 channels c) = 2 KB, the planes 1 KB
  // apart, the lane's piece at lane * 16.
  const char* Ub = (const char*)U;
  const char* Vb = (const char*)V;
  const size_t ublock = (size_t)((kb + wave * 16) >> 4) * NCH * 2048;
  const size_t ustep_p = (size_t)(g.Kp >> 4) * NCH * 2048;
  const size_t vplane = (size_t)g.Tp * g.Cp;           // bytes of one digit plane of a position
  const uint32_t ulane = (uint32_t)lane * 16u;
  // V piece e = tid + 256 k of a position, in operand order [channel step][plane][tile
  // row][16 bytes]: e & 3 = piece of the 64-byte row, (e >> 2) & 15 = tile, e >> 6 =
  // channel step * 2 + plane (wave + 4 k: the plane and the low bit of the step come from
  // the wavefront, the rest of the step from k)
  const uint32_t vthr = (uint32_t)(wave & 1) * (uint32_t)vplane +
                        (uint32_t)(tb + ((tid >> 2) & 15)) * (uint32_t)g.Cp +
                        (uint32_t)(wave >> 1) * 64u + (uint32_t)(tid & 3) * 16u;

  v4i rua[kDepth], rub[kDepth];
  v4u vst[kPos][kLd];
  // step sj of column j: position p = (sj / NCH) * n + j, channel step sj % NCH
  auto fetch = [&](int sj, int j, int slot) {
    const int p = (sj / NCH) * n + j, ch = sj % NCH;
    size_t uo = ublock + (size_t)p * ustep_p + (size_t)ch * 2048;
    asm volatile("" : "+s"(uo));
    rua[slot] = *(const v4i*)(Ub + uo + ulane);
    rub[slot] = *(const v4i*)(Ub + uo + 1024 + ulane);
  };
  // the workgroup's share of position (i, j) into ring slot `slot` (wavefronts beyond the
  // last operand block of a short reduction load nothing)
  auto vfetch = [&](int i, int j, int slot) {
    const int p = i * n + j;
#pragma unroll
    for (int k = 0; k < kLd; ++k) {
      if (wave + 4 * k < kBlocks) {
        size_t vo = (size_t)(2 * p) * vplane + (size_t)k * 128;
        asm volatile("" : "+s"(vo));
        vst[slot][k] = *(const v4u*)(Vb + vo + vthr);
      }
    }
  };
  auto vstore = [&](int slot, int buf) {
#pragma unroll
    for (int k = 0; k < kLd; ++k)
      if (wave + 4 * k < kBlocks) vlds[buf * kBufPieces + tid + 256 * k] = vst[slot][k];
  };
  // position 0 straight into buffer 0, positions 1 .. kPos into the ring (position x in
  // slot x % kPos), the first kDepth steps of U into theirs
  vfetch(0, 0, 0);
  vstore(0, 0);
#pragma unroll
  for (int x = 1; x <= kPos; ++x) vfetch(x % n, x / n, x % kPos);
#pragma unroll
  for (int s = 0; s < kDepth; ++s) fetch(s, 0, s);

  float z[M][4], Y[M][M][4];
#pragma unroll
  for (int a = 0; a < M; ++a)
#pragma unroll
    for (int b = 0; b < M; ++b)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) Y[a][b][rr] = 0.0f;
  const v4i zero = v4i{0, 0, 0, 0}, ones = v4i{kOnes, kOnes, kOnes, kOnes};
  const int cbias = 16384 * g.Cp;

  // (one copy of the loop per setting of the Hadamard-stage quantizer: a test per
  // accumulator would cut the loop body into pieces the scheduler cannot overlap)
  auto columns = [&](auto mq_tag) {
    constexpr bool kMQ = decltype(mq_tag)::value;
#pragma unroll 1
    for (int j = 0; j < n; ++j) {
      // (columns past the last: the loads repeat valid addresses, their data is never used)
      const int jn = j + 1 < n ? j + 1 : j, jnn = j + 2 < n ? j + 2 : n - 1;
#pragma unroll
      for (int i = 0; i < n; ++i) {
        // Every wavefront has finished the previous position, whose buffer the next
        // position's operands may now overwrite; this position's buffer is complete.
        __syncthreads();
        vstore((i + 1) % kPos, (i + 1) & 1);
        constexpr int kAhead = 1 + kPos;
        static_assert(kAhead <= n + 1, "at most two columns ahead");
        vfetch((i + kAhead) % n, (i + kAhead) / n == 0 ? j : (i + kAhead) / n == 1 ? jn : jnn,
               (i + 1) % kPos);
        const v4i* vops = (const v4i*)(vlds + (i & 1) * kBufPieces) + (r * 4 + grp);
        v4i hh = zero, mid = zero, ll = zero, sva = zero, svb = zero, sua = zero, sub = zero;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
          const int sj = i * NCH + ch, slot = sj % kDepth;
          const v4i ua = rua[slot], ub = rub[slot];
          const v4i va = vops[(ch * 2) * 64], vb = vops[(ch * 2 + 1) * 64];
          hh = __builtin_amdgcn_mfma_i32_16x16x64_i8(ua, va, hh, 0, 0, 0);
          mid = __builtin_amdgcn_mfma_i32_16x16x64_i8(ua, vb, mid, 0, 0, 0);
          mid = __builtin_amdgcn_mfma_i32_16x16x64_i8(ub, va, mid, 0, 0, 0);
          ll = __builtin_amdgcn_mfma_i32_16x16x64_i8(ub, vb, ll, 0, 0, 0);
          sva = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, va, sva, 0, 0, 0);
          svb = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, vb, svb, 0, 0, 0);
          sua = __builtin_amdgcn_mfma_i32_16x16x64_i8(ua, ones, sua, 0, 0, 0);
          sub = __builtin_amdgcn_mfma_i32_16x16x64_i8(ub, ones, sub, 0, 0, 0);
          // refill the slot once its operands have been issued (the loads may then land in
          // the same registers); the compiler-level fence keeps later steps' loads behind
          // this one, so that the ring, not the scheduler, decides what is in flight
          if (sj + kDepth < SJ) fetch(sj + kDepth, j, slot);
          else fetch(sj + kDepth - SJ, jn, slot);
          asm volatile("" ::: "memory");
        }
        const float wp = w.r[i * n + j];               // 1 with per-tensor scales: exact
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          // M = 2^16 hh + 2^8 (mid + 128 (sva + sua)) + (ll + 128 (svb + sub) + 16384 Cp):
          // the brackets fit int32 (|.| <= 2^16 Cp), the sum is exact in fp64 (below
          // 2^53), and one rounding to fp32 is the conversion of the integer M
          const int m1 = mid[rr] + (sva[rr] + sua[rr]) * 128;
          const int m0 = ll[rr] + (svb[rr] + sub[rr]) * 128 + cbias;
          const double dm = __builtin_fma((double)hh[rr], 65536.0,
                                          __builtin_fma((double)m1, 256.0, (double)m0));
          float f = (float)dm * wp;
          if constexpr (kMQ) f = quantize_f(f, r_m, qmax_m);
#pragma unroll
          for (int a = 0; a < M; ++a) {
            if (i == 0) z[a][rr] = 0.0f;
            if (at_nonzero<M, kSparse>(a, i))
              z[a][rr] = __builtin_fmaf(at.v[a * n + i], f, z[a][rr]);
          }
        }
      }
#pragma unroll
      for (int b = 0; b < M; ++b) {
        const float abj = at.v[b * n + j];
#pragma unroll
        for (int a = 0; a < M; ++a)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) Y[a][b][rr] = __builtin_fmaf(z[a][rr], abj, Y[a][b][rr]);
      }
    }
  };
  if (r_m > 0.0f) columns(std::true_type{});
  else columns(std::false_type{});

  if (t >= g.T) return;
  const int tw = t % g.TW, th = (t / g.TW) % g.TH, img = t / (g.TW * g.TH);
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    const int k = kb + wave * 16 + grp * 4 + rr;
    if (k >= g.K) continue;
    int q[M][M];
#pragma unroll
    for (int a = 0; a < M; ++a)
#pragma unroll
      for (int b = 0; b < M; ++b) q[a][b] = quantize(Y[a][b][rr], r_y, qmax_y);
    store_codes<M, YT>(y + ((size_t)img * g.K + k) * g.Ho * g.Wo, g, th * M, tw * M, q, fast != 0);
  }
}

// Taps: canonical dense order, int16 codes (U, V) or the int64 accumulators (M).
__global__ __launch_bounds__(256) void export_u_w16(const int8_t* __restrict__ U,
                                                    int16_t* __restrict__ out, Geom g) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)g.P * g.K * g.C) return;
  const int c = (int)(i % g.C), k = (int)((i / g.C) % g.K), p = (int)(i / ((size_t)g.C * g.K));
  out[i] = (int16_t)join_code(U[u8w_index(g.Kp, g.Cp, p, 0, k, c)],
                              U[u8w_index(g.Kp, g.Cp, p, 1, k, c)]);
}
__global__ __launch_bounds__(256) void export_v_w16(const int8_t* __restrict__ V,
                                                    int16_t* __restrict__ out, Geom g) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)g.P * g.T * g.C) return;
  const int c = (int)(i % g.C), t = (int)((i / g.C) % g.T), p = (int)(i / ((size_t)g.C * g.T));
  out[i] = (int16_t)join_code(V[v8w_index(g.Tp, g.Cp, p, 0, t, c)],
                              V[v8w_index(g.Tp, g.Cp, p, 1, t, c)]);
}
__global__ __launch_bounds__(256) void export_m_w16(const long long* __restrict__ Mi,
                                                    long long* __restrict__ out, Geom g) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)g.P * g.T * g.K) return;
  const int k = (int)(i % g.K), t = (int)((i / g.K) % g.T), p = (int)(i / ((size_t)g.K * g.T));
  out[i] = Mi[((size_t)p * g.Tp + t) * g.Kp + k];
}

template <int M>
hipError_t input_m(const Geom& g, const MatBT& bt, const void* x, void* V, const PosScale& rv,
                   float qmax, hipStream_t s) {
  dim3 grid(g.Tp / 8, g.Cp / 32);
  const bool sparse = fits_mask(bt.v, g.n * g.n, CookToomMask<M>::bt);
  const bool row = g.W >= 8;
  int8_t* Vh = (int8_t*)V;
#define WINO_W16_IN(XT, SP, RW) \
  input_transform_w16<M, XT, SP, RW><<<grid, 256, 0, s>>>(g, bt, (const XT*)x, Vh, rv, qmax)
#define WINO_W16_IN2(XT, SP) do { if (row) WINO_W16_IN(XT, SP, true); else WINO_W16_IN(XT, SP, false); } while (0)
  if (g.x16) {
    if (sparse) WINO_W16_IN2(int16_t, true); else WINO_W16_IN2(int16_t, false);
  } else {
    if (sparse) WINO_W16_IN2(int8_t, true); else WINO_W16_IN2(int8_t, false);
  }
#undef WINO_W16_IN2
#undef WINO_W16_IN
  return hipGetLastError();
}

template <int M, typename YT>
hipError_t output_my(const Geom& g, const MatAT& at, const void* Mi, void* y, const PosScale* w,
                     float r_m, float r_y, float qmax_m, float qmax_y, hipStream_t s) {
  dim3 grid(g.Tp / 4, g.Kp / 64);
  const bool sparse = sparse_at<M>(at.v);
  PosScale one;
  for (int p = 0; p < 64; ++p) one.r[p] = 1.0f;
  const long long* Ml = (const long long*)Mi;
  YT* yo = (YT*)y;
  const int fast = g.Ho % M == 0 && g.Wo % M == 0 && ((uintptr_t)y & 7) == 0;
  if (w) {
    if (sparse) output_transform_w16<M, YT, true, true><<<grid, 256, 0, s>>>(g, at, Ml, yo, *w, r_m, r_y, qmax_m, qmax_y, fast);
    else output_transform_w16<M, YT, false, true><<<grid, 256, 0, s>>>(g, at, Ml, yo, *w, r_m, r_y, qmax_m, qmax_y, fast);
  } else {
    if (sparse) output_transform_w16<M, YT, true, false><<<grid, 256, 0, s>>>(g, at, Ml, yo, one, r_m, r_y, qmax_m, qmax_y, fast);
    else output_transform_w16<M, YT, false, false><<<grid, 256, 0, s>>>(g, at, Ml, yo, one, r_m, r_y, qmax_m, qmax_y, fast);
  }
  return hipGetLastError();
}

template <int M>
hipError_t output_m(const Geom& g, const MatAT& at, const void* Mi, void* y, const PosScale* w,
                    float r_m, float r_y, float qmax_m, float qmax_y, hipStream_t s) {
  return g.x16 ? output_my<M, int16_t>(g, at, Mi, y, w, r_m, r_y, qmax_m, qmax_y, s)
               : output_my<M, int8_t>(g, at, Mi, y, w, r_m, r_y, qmax_m, qmax_y, s);
}

}  // namespace

hipError_t launch_w16_weights(const Geom& g, const MatG& mg, const float* w, void* U,
                              const PosScale& ru, float qmax, hipStream_t s) {
  const unsigned nb = (unsigned)(((size_t)g.Kp * g.Cp + 255) / 256);
  int8_t* Uh = (int8_t*)U;
  switch (g.m) {
    case 2: weight_transform_w16<2><<<nb, 256, 0, s>>>(g, mg, w, Uh, ru, qmax); break;
    case 4: weight_transform_w16<4><<<nb, 256, 0, s>>>(g, mg, w, Uh, ru, qmax); break;
    default: weight_transform_w16<6><<<nb, 256, 0, s>>>(g, mg, w, Uh, ru, qmax); break;
  }
  return hipGetLastError();
}

hipError_t launch_w16_input(const Geom& g, const MatBT& bt, const void* x, void* V,
                            const PosScale& rv, float qmax, hipStream_t s) {
  switch (g.m) {
    case 2: return input_m<2>(g, bt, x, V, rv, qmax, s);
    case 4: return input_m<4>(g, bt, x, V, rv, qmax, s);
    default: return input_m<6>(g, bt, x, V, rv, qmax, s);
  }
}

hipError_t launch_w16_gemm(const Geom& g, const void* V, const void* U, void* M, hipStream_t s) {
  if (g.Kp / 64 > 65535 || g.Cp > 1024) return hipErrorInvalidValue;
  dim3 grid(g.Tp / 64, g.Kp / 64, g.P);
  gemm_w16_kernel<<<grid, 256, 0, s>>>(g.Tp, g.Kp, g.Cp, (const int8_t*)V, (const int8_t*)U,
                                       (long long*)M);
  return hipGetLastError();
}

hipError_t launch_w16_output(const Geom& g, const MatAT& at, const void* M, void* y,
                             const PosScale* w_pos, float r_m, float r_y, float qmax_m,
                             float qmax_y, hipStream_t s) {
  if (g.Kp / 64 > 65535) return hipErrorInvalidValue;
  switch (g.m) {
    case 2: return output_m<2>(g, at, M, y, w_pos, r_m, r_y, qmax_m, qmax_y, s);
    case 4: return output_m<4>(g, at, M, y, w_pos, r_m, r_y, qmax_m, qmax_y, s);
    default: return output_m<6>(g, at, M, y, w_pos, r_m, r_y, qmax_m, qmax_y, s);
  }
}

// GEMM + output in one kernel: 64..512 padded channels in powers of two, every offset in
// 32 bits -- and enough tiles: with few, its long workgroups leave most of the chip idle and
// the two separate kernels measure faster (64 tiles: 18.0 vs 12.7 us at 64 channels, 28.8 vs
// 18.3 at 256; F6 at 288 tiles 51.6 vs 33.7; from 512 tiles on the fused kernel wins).
bool w16_gemm_out_supported(const Geom& g, const MatAT&) {
  const bool nch_ok = g.Cp == 64 || g.Cp == 128 || g.Cp == 256 || g.Cp == 512;
  // (the per-thread part of a V address, up to two digit planes, must fit 32 bits)
  return nch_ok && g.T >= (g.m == 6 ? 1024 : 512) && g.Kp / 64 <= 65535 &&
         (size_t)g.Tp * g.Cp * 2 < 0xffffffffull;
}

namespace {
template <int M, typename YT, bool kSparse>
hipError_t gemm_out_mys(const Geom& g, const MatAT& at, const void* V, const void* U, void* y,
                        const PosScale* w, float r_m, float r_y, float qmax_m, float qmax_y,
                        hipStream_t s) {
  PosScale one;
  for (int p = 0; p < 64; ++p) one.r[p] = 1.0f;
  const PosScale& ws = w ? *w : one;
  const int8_t* Vi = (const int8_t*)V;
  const int8_t* Ui = (const int8_t*)U;
  YT* yo = (YT*)y;
  const int fast = g.Ho % M == 0 && g.Wo % M == 0 && ((uintptr_t)y & 7) == 0;
  const dim3 grid(g.Tp / 16, g.Kp / 64);
#define WINO_W16_GO(NCHV)                                                                  \
  gemm_out_w16_kernel<M, YT, NCHV, kSparse><<<grid, 256, 0, s>>>(g, at, Vi, Ui, yo, ws, r_m, \
                                                                  r_y, qmax_m, qmax_y, fast)
  switch (g.Cp) {
    case 64: WINO_W16_GO(1); break;
    case 128: WINO_W16_GO(2); break;
    case 256: WINO_W16_GO(4); break;
    default: WINO_W16_GO(8); break;
  }
#undef WINO_W16_GO
  return hipGetLastError();
}
template <int M>
hipError_t gemm_out_m(const Geom& g, const MatAT& at, const void* V, const void* U, void* y,
                      const PosScale* w, float r_m, float r_y, float qmax_m, float qmax_y,
                      hipStream_t s) {
  const bool sparse = sparse_at<M>(at.v);
  if (g.x16)
    return sparse ? gemm_out_mys<M, int16_t, true>(g, at, V, U, y, w, r_m, r_y, qmax_m, qmax_y, s)
                  : gemm_out_mys<M, int16_t, false>(g, at, V, U, y, w, r_m, r_y, qmax_m, qmax_y, s);
  return sparse ? gemm_out_mys<M, int8_t, true>(g, at, V, U, y, w, r_m, r_y, qmax_m, qmax_y, s)
                : gemm_out_mys<M, int8_t, false>(g, at, V, U, y, w, r_m, r_y, qmax_m, qmax_y, s);
}
}  // namespace

hipError_t launch_w16_gemm_out(const Geom& g, const MatAT& at, const void* V, const void* U,
                               void* y, const PosScale* w_pos, float r_m, float r_y, float qmax_m,
                               float qmax_y, hipStream_t s) {
  if (!w16_gemm_out_supported(g, at)) return hipErrorInvalidValue;
  switch (g.m) {
    case 2: return gemm_out_m<2>(g, at, V, U, y, w_pos, r_m, r_y, qmax_m, qmax_y, s);
    case 4: return gemm_out_m<4>(g, at, V, U, y, w_pos, r_m, r_y, qmax_m, qmax_y, s);
    default: return gemm_out_m<6>(g, at, V, U, y, w_pos, r_m, r_y, qmax_m, qmax_y, s);
  }
}

hipError_t launch_w16_export(const Geom& g, int which, const void* src, void* out, hipStream_t s) {
  if (which == WINO_TAP_U) {
    const size_t tot = (size_t)g.P * g.K * g.C;
    export_u_w16<<<(unsigned)((tot + 255) / 256), 256, 0, s>>>((const int8_t*)src, (int16_t*)out, g);
  } else if (which == WINO_TAP_V) {
    const size_t tot = (size_t)g.P * g.T * g.C;
    export_v_w16<<<(unsigned)((tot + 255) / 256), 256, 0, s>>>((const int8_t*)src, (int16_t*)out, g);
  } else {
    const size_t tot = (size_t)g.P * g.T * g.K;
    export_m_w16<<<(unsigned)((tot + 255) / 256), 256, 0, s>>>((const long long*)src, (long long*)out, g);
  }
  return hipGetLastError();
}

}  // namespace wino
