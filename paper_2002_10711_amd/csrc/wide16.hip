// Wider Winograd domain: the quantized forward with up to 16-bit codes after every stage
// (Sec. 3.2, "quantization diversity": each intermediate of Eq. 1 may have its own
// bit-width; Sec. 5.1 runs INT8, INT10 and INT16; Sec. 6 names wider intermediate stages as
// the way to recover F4/F6 accuracy).
//
// The matrix cores have no 16-bit integer instruction.  A code v in [-32767, 32767] is
// split into two balanced base-256 digits, v = 256 a + b with b in [-128, 127] and
// a in [-128, 128], both exact in fp16, and the per-position GEMM of Sec. 5.3 becomes four
// fp16 MFMAs per 32 channels,
//
//     sum_c u v = 2^16 sum a_u a_v + 2^8 (sum a_u b_v + sum b_u a_v) + sum b_u b_v .
//
// Every product is an integer of magnitude <= 2^14 and every partial sum stays an integer
// below 2^24 for up to 1024 channels (512 where the two middle sums share one
// accumulator), so the fp32 accumulators of the MFMA hold them exactly; the four sums are
// recombined in 64-bit integers.  The result is the exact integer M of the int16 pipeline.
//
// Device layouts of this mode (fp16 digit planes, digit 0 = a, digit 1 = b):
//   V [P][2][Tp][Cp]   plain rows, channel fastest
//   U [P][Kp/16][Cp/32][2][64 lanes][8]  blocks in the order an MFMA wavefront loads its "A"
//                      operand: lane = (c % 32 / 8) * 16 + k % 16 holds channels c % 8
//   M [P][Tp][Kp]      int64
// with Tp, Kp, Cp rounded up to 64; padding channels hold zero.
#include "output_stage.h"

namespace wino {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

__host__ __device__ inline size_t u16_index(int Kp, int Cp, int p, int digit, int k, int c) {
  const size_t blk = ((size_t)p * (Kp >> 4) + (k >> 4)) * (Cp >> 5) + (c >> 5);
  return ((blk * 2 + digit) * 64 + (size_t)(((c & 31) >> 3) * 16 + (k & 15))) * 8 + (c & 7);
}
__host__ __device__ inline size_t v16_index(int Tp, int Cp, int p, int digit, int t, int c) {
  return (((size_t)p * 2 + digit) * Tp + t) * Cp + c;
}

// v = 256 a + b, b in [-128, 127]
__device__ __forceinline__ void split_code(int v, _Float16& a, _Float16& b) {
  const int lo = ((v + 128) & 255) - 128;
  a = (_Float16)(float)((v - lo) >> 8);
  b = (_Float16)(float)lo;
}
__device__ __forceinline__ int join_code(_Float16 a, _Float16 b) {
  return (int)(float)a * 256 + (int)(float)b;
}

// Weight stage (Eq. 1: U = G g G^T; quantizer of Sec. 3.2): one thread per (k, c) of the
// padded matrix, codes split into the two digit planes.
template <int M>
__global__ __launch_bounds__(256) void weight_transform_w16(Geom g, MatG mg,
                                                            const float* __restrict__ w,
                                                            _Float16* __restrict__ U, PosScale ru,
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
      _Float16 a, b;
      split_code(quantize(Uf[i][j], ru.r[p], qmax), a, b);
      U[u16_index(g.Kp, g.Cp, p, 0, k, c)] = a;
      U[u16_index(g.Kp, g.Cp, p, 1, k, c)] = b;
    }
}

// Input stage (Eq. 1: V = B^T d B on every patch, Sec. 3.2): a workgroup owns 16
// consecutive tiles x 16 channels, one (tile, channel) per thread with the tiles along the
// lanes (neighbouring patches overlap: the loads of a wavefront fall into a few runs of
// an image row).  The codes go through LDS so that the rows of V are written in pieces of
// 32 bytes.
template <int M, typename XT, bool kSparse>
__global__ __launch_bounds__(256) void input_transform_w16(Geom g, MatBT bt,
                                                           const XT* __restrict__ x,
                                                           _Float16* __restrict__ V, PosScale rv,
                                                           float qmax) {
  constexpr int n = M + 2, P = n * n;
  __shared__ __attribute__((aligned(16))) _Float16 sm[P * 256];
  const int tid = threadIdx.x, r = tid & 15, cc = tid >> 4;
  const int t = blockIdx.x * 16 + r, c = blockIdx.y * 16 + cc;
  float d[n][n];
#pragma unroll
  for (int j = 0; j < n; ++j)
#pragma unroll
    for (int l = 0; l < n; ++l) d[j][l] = 0.0f;
  if (t < g.T && c < g.C) {
    const int tw = t % g.TW, th = (t / g.TW) % g.TH, img = t / (g.TW * g.TH);
    const XT* base = x + ((size_t)img * g.C + c) * g.H * g.W;
#pragma unroll
    for (int j = 0; j < n; ++j)
#pragma unroll
      for (int l = 0; l < n; ++l) {
        const int h = th * M - g.pad + j, ww = tw * M - g.pad + l;
        if (h >= 0 && h < g.H && ww >= 0 && ww < g.W) d[j][l] = (float)base[h * g.W + ww];
      }
  }
  float Vf[n][n];
  transform_patch<M, kSparse>(d, bt, Vf);
  int code[P];
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int k = 0; k < n; ++k) code[i * n + k] = quantize(Vf[i][k], rv.r[i * n + k], qmax);
#pragma unroll
  for (int digit = 0; digit < 2; ++digit) {
    if (digit) __syncthreads();                        // the first plane has left LDS
#pragma unroll
    for (int p = 0; p < P; ++p) {
      _Float16 a, b;
      split_code(code[p], a, b);
      sm[(p * 16 + r) * 16 + cc] = digit ? b : a;
    }
    __syncthreads();
    // P * 16 rows of 16 channels = P * 32 pieces of 16 bytes
    for (int idx = tid; idx < P * 32; idx += 256) {
      const int p = idx >> 5, row = (idx & 31) >> 1, piece = idx & 1;
      *(v4u*)(V + v16_index(g.Tp, g.Cp, p, digit, blockIdx.x * 16 + row,
                            blockIdx.y * 16 + piece * 8)) =
          *(const v4u*)&sm[(p * 16 + row) * 16 + piece * 8];
    }
  }
}

// Hadamard/GEMM stage (Sec. 5.3: one GEMM per Winograd position, channels summed in the
// Winograd domain), exact in 64-bit integers.  Workgroup = 64 tiles x 64 output channels
// of one position; wavefront = 32 x 32 = 2 x 2 MFMA tiles with four accumulators each
// (the digit pairs).  Operands go straight from global memory into the MFMA, one 32-channel
// step ahead of their use.
__global__ __launch_bounds__(256) void gemm_w16_kernel(int Tp, int Kp, int Cp,
                                                       const _Float16* __restrict__ V,
                                                       const _Float16* __restrict__ U,
                                                       long long* __restrict__ Mo) {
  const int p = blockIdx.z, tb = blockIdx.x * 64, kb = blockIdx.y * 64;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, grp = lane >> 4;
  const int wave = tid >> 6, wt = wave & 1, wk = wave >> 1;
  const int nch = Cp >> 5;
  const half8* ua[2][2];
  const half8* vb[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const int kt = kb + wk * 32 + a * 16;
    const size_t blk = ((size_t)p * (Kp >> 4) + (kt >> 4)) * (Cp >> 5);
#pragma unroll
    for (int dg = 0; dg < 2; ++dg) ua[a][dg] = (const half8*)(U + (blk * 2 + dg) * 512) + lane;
  }
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int t = tb + wt * 32 + b * 16 + r;
#pragma unroll
    for (int dg = 0; dg < 2; ++dg)
      vb[b][dg] = (const half8*)(V + v16_index(Tp, Cp, p, dg, t, grp * 8));
  }
  // per 32-channel step: U advances by one block pair (2 * 512 halfs = 128 pieces), V by
  // 32 halfs = 4 pieces
  half8 A[2][2], B[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int dg = 0; dg < 2; ++dg) {
      A[a][dg] = ua[a][dg][0];
      B[a][dg] = vb[a][dg][0];
    }
  v4f hh[2][2], hl[2][2], lh[2][2], ll[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) hh[a][b] = hl[a][b] = lh[a][b] = ll[a][b] = v4f{0, 0, 0, 0};
  for (int ch = 0; ch < nch; ++ch) {
    const int nx = ch + 1 < nch ? ch + 1 : ch;         // (the last step reloads itself)
    half8 nA[2][2], nB[2][2];
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
        hh[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[a][0], B[b][0], hh[a][b], 0, 0, 0);
        hl[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[a][0], B[b][1], hl[a][b], 0, 0, 0);
        lh[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[a][1], B[b][0], lh[a][b], 0, 0, 0);
        ll[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[a][1], B[b][1], ll[a][b], 0, 0, 0);
      }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int dg = 0; dg < 2; ++dg) {
        A[a][dg] = nA[a][dg];
        B[a][dg] = nB[a][dg];
      }
  }
  // lane: tile t (column), output channels k0 .. k0 + 3 (rows grp*4 + rr)
  typedef long long v2ll __attribute__((ext_vector_type(2)));
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int t = tb + wt * 32 + b * 16 + r, k0 = kb + wk * 32 + a * 16 + grp * 4;
      long long m[4];
#pragma unroll
      for (int rr = 0; rr < 4; ++rr)
        m[rr] = ((long long)(int)hh[a][b][rr] << 16) +
                (((long long)(int)hl[a][b][rr] + (long long)(int)lh[a][b][rr]) << 8) +
                (long long)(int)ll[a][b][rr];
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
                                                            float qmax_y) {
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
      if (r_m > 0.0f) f = (float)quantize(f, r_m, qmax_m);
      Mt[i][j] = f;
    }
  transform_result<M, kSparse>(Mt, at, Y);
  const int tw = t % g.TW, th = (t / g.TW) % g.TH, img = t / (g.TW * g.TH);
  YT* plane = y + ((size_t)img * g.K + k) * g.Ho * g.Wo;
#pragma unroll
  for (int a = 0; a < M; ++a)
#pragma unroll
    for (int b = 0; b < M; ++b) {
      const int h = th * M + a, x = tw * M + b;
      if (h < g.Ho && x < g.Wo) plane[(size_t)h * g.Wo + x] = (YT)quantize(Y[a][b], r_y, qmax_y);
    }
}

// Taps: canonical dense order, int16 codes (U, V) or the int64 accumulators (M).
__global__ __launch_bounds__(256) void export_u_w16(const _Float16* __restrict__ U,
                                                    int16_t* __restrict__ out, Geom g) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)g.P * g.K * g.C) return;
  const int c = (int)(i % g.C), k = (int)((i / g.C) % g.K), p = (int)(i / ((size_t)g.C * g.K));
  out[i] = (int16_t)join_code(U[u16_index(g.Kp, g.Cp, p, 0, k, c)],
                              U[u16_index(g.Kp, g.Cp, p, 1, k, c)]);
}
__global__ __launch_bounds__(256) void export_v_w16(const _Float16* __restrict__ V,
                                                    int16_t* __restrict__ out, Geom g) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)g.P * g.T * g.C) return;
  const int c = (int)(i % g.C), t = (int)((i / g.C) % g.T), p = (int)(i / ((size_t)g.C * g.T));
  out[i] = (int16_t)join_code(V[v16_index(g.Tp, g.Cp, p, 0, t, c)],
                              V[v16_index(g.Tp, g.Cp, p, 1, t, c)]);
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
  dim3 grid(g.Tp / 16, g.Cp / 16);
  const bool sparse = fits_mask(bt.v, g.n * g.n, CookToomMask<M>::bt);
  _Float16* Vh = (_Float16*)V;
  if (g.x16) {
    if (sparse) input_transform_w16<M, int16_t, true><<<grid, 256, 0, s>>>(g, bt, (const int16_t*)x, Vh, rv, qmax);
    else input_transform_w16<M, int16_t, false><<<grid, 256, 0, s>>>(g, bt, (const int16_t*)x, Vh, rv, qmax);
  } else {
    if (sparse) input_transform_w16<M, int8_t, true><<<grid, 256, 0, s>>>(g, bt, (const int8_t*)x, Vh, rv, qmax);
    else input_transform_w16<M, int8_t, false><<<grid, 256, 0, s>>>(g, bt, (const int8_t*)x, Vh, rv, qmax);
  }
  return hipGetLastError();
}

template <int M, typename YT>
hipError_t output_my(const Geom& g, const MatAT& at, const void* Mi, void* y, const PosScale* w,
                     float r_m, float r_y, float qmax_m, float qmax_y, hipStream_t s) {
  dim3 grid(g.Tp / 4, g.Kp / 64);
  const bool sparse = fits_mask(at.v, g.m * g.n, CookToomMask<M>::at);
  PosScale one;
  for (int p = 0; p < 64; ++p) one.r[p] = 1.0f;
  const long long* Ml = (const long long*)Mi;
  YT* yo = (YT*)y;
  if (w) {
    if (sparse) output_transform_w16<M, YT, true, true><<<grid, 256, 0, s>>>(g, at, Ml, yo, *w, r_m, r_y, qmax_m, qmax_y);
    else output_transform_w16<M, YT, false, true><<<grid, 256, 0, s>>>(g, at, Ml, yo, *w, r_m, r_y, qmax_m, qmax_y);
  } else {
    if (sparse) output_transform_w16<M, YT, true, false><<<grid, 256, 0, s>>>(g, at, Ml, yo, one, r_m, r_y, qmax_m, qmax_y);
    else output_transform_w16<M, YT, false, false><<<grid, 256, 0, s>>>(g, at, Ml, yo, one, r_m, r_y, qmax_m, qmax_y);
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
  _Float16* Uh = (_Float16*)U;
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
  gemm_w16_kernel<<<grid, 256, 0, s>>>(g.Tp, g.Kp, g.Cp, (const _Float16*)V, (const _Float16*)U,
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

hipError_t launch_w16_export(const Geom& g, int which, const void* src, void* out, hipStream_t s) {
  if (which == WINO_TAP_U) {
    const size_t tot = (size_t)g.P * g.K * g.C;
    export_u_w16<<<(unsigned)((tot + 255) / 256), 256, 0, s>>>((const _Float16*)src, (int16_t*)out, g);
  } else if (which == WINO_TAP_V) {
    const size_t tot = (size_t)g.P * g.T * g.C;
    export_v_w16<<<(unsigned)((tot + 255) / 256), 256, 0, s>>>((const _Float16*)src, (int16_t*)out, g);
  } else {
    const size_t tot = (size_t)g.P * g.T * g.K;
    export_m_w16<<<(unsigned)((tot + 255) / 256), 256, 0, s>>>((const long long*)src, (long long*)out, g);
  }
  return hipGetLastError();
}

}  // namespace wino
