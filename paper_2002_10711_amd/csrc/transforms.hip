// Transform kernels of the Winograd-aware layer (paper, Sec. 3.1 Eq. 1 and
// Sec. 3.2): input transform B^T d B, weight transform G g G^T, output transform
// A^T M A, each followed by the stage's quantizer in int8 mode, plus the copy
// kernel behind the parity taps.
//
// Arithmetic contract of the int8 mode (what makes an integer result well defined
// for arbitrary real matrices): IEEE fp32; every sum is the chain
// acc = +0; acc = fma(a_j, b_j, acc) over ascending j; the first product of a
// two-sided transform is the left one (B^T d, G g, A^T M); a quantizer rounds the
// exact product of its input and its reciprocal step once, half to even, and
// saturates to [-qmax, qmax] (transform_math.h).
//
// The matrices arrive by value in the kernel arguments (scalar registers), never
// as compiled-in constants, so learned transforms use the same code.
#include <string.h>

#include "input_stage.h"
#include "output_stage.h"

namespace wino {
namespace {

// ------------------------------------------------------------------ input --
// Stand-alone int8 input transform (see input_stage.h): V[p][t][c] to global memory,
// a wavefront storing 256 contiguous bytes per position.
// kPos: per-position quantizer factors rvp (else the one factor r_v).
template <int M, bool kSparse, bool kWide, bool kPos>
__global__ __launch_bounds__(256) void input_transform_i8(Geom g, MatBT bt,
                                                          const int8_t* __restrict__ x,
                                                          uint32_t* __restrict__ V, float r_v,
                                                          float qmax, int RB, int TWB,
                                                          PosScale rvp) {
  constexpr int n = M + 2, P = n * n, CBQ = InCfg<M>::kCBQ;
  extern __shared__ uint32_t lds[];
  const int Wc = stage_cols(M, TWB);
  const int ntwb = (g.TW + TWB - 1) / TWB;
  const int twb = blockIdx.x % ntwb, rb = blockIdx.x / ntwb;
  const int r0 = rb * RB, tw0 = twb * TWB, c0 = blockIdx.y * 64;
  const int R = g.N * g.TH;
  stage_strips<M, kWide>(g, x, lds, c0, r0, tw0, RB, TWB);
  __syncthreads();
  const float lo = kMagic - qmax, hi = kMagic + qmax;
  const int cq_per = g.Cp >> 2;
  const size_t pstride = (size_t)g.Tp * cq_per;
  const int nitem = RB * TWB * 16;
  for (int it = threadIdx.x; it < nitem; it += blockDim.x) {
    const int cq = it & 15, twl = (it >> 4) % TWB, rs = (it >> 4) / TWB;
    const int r = r0 + rs, tw = tw0 + twl;
    if (r >= R || tw >= g.TW) continue;
    uint32_t out[P];
    transform_quad<M, kSparse, kPos>(lds + ((size_t)rs * n * Wc + twl * M) * CBQ + cq, Wc, bt, r_v,
                                     lo, hi, out, &rvp);
    uint32_t* vp = V + ((size_t)r * g.TW + tw) * cq_per + (c0 >> 2) + cq;
#pragma unroll
    for (int p = 0; p < P; ++p) vp[p * pstride] = out[p];
  }
}

// The same for layers with few tiles (less than a wavefront per SIMD): (M + 2) / 2 wavefronts
// share an item, each producing two rows i of V -- w = (B^T d)[i][.] and V[i][.] = w B need
// no other rows -- so the chain of dependent fmas a lane runs is (M + 2) / 2 times shorter.
// blockDim.x = 64 * (M + 2) / 2; wavefront s owns rows 2s, 2s + 1 of every item (one copy
// of the arithmetic per s, so that the rows are compile-time constants and the zero
// pattern of B^T can be skipped in both products).
template <int M, bool kSparse, bool kWide, bool kPos>
__global__ __launch_bounds__(256) void input_transform_i8_rows(Geom g, MatBT bt,
                                                               const int8_t* __restrict__ x,
                                                               uint32_t* __restrict__ V, float r_v,
                                                               float qmax, int RB, int TWB,
                                                               PosScale rvp) {
  constexpr int n = M + 2, CBQ = InCfg<M>::kCBQ;
  extern __shared__ uint32_t lds[];
  const int Wc = stage_cols(M, TWB);
  const int ntwb = (g.TW + TWB - 1) / TWB;
  const int twb = blockIdx.x % ntwb, rb = blockIdx.x / ntwb;
  const int r0 = rb * RB, tw0 = twb * TWB, c0 = blockIdx.y * 64;
  const int R = g.N * g.TH;
  stage_strips<M, kWide>(g, x, lds, c0, r0, tw0, RB, TWB);
  __syncthreads();
  const float lo = kMagic - qmax, hi = kMagic + qmax;
  const int cq_per = g.Cp >> 2;
  const size_t pstride = (size_t)g.Tp * cq_per;
  const int nitem = RB * TWB * 16;
  const int sub = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  auto rows = [&](auto i0_tag) {
  constexpr int i0 = decltype(i0_tag)::value;
  for (int it = threadIdx.x & 63; it < nitem; it += 64) {
    const int cq = it & 15, twl = (it >> 4) % TWB, rs = (it >> 4) / TWB;
    const int r = r0 + rs, tw = tw0 + twl;
    if (r >= R || tw >= g.TW) continue;
    uint32_t raw[n][n];
    load_quad_patch<M>(lds + ((size_t)rs * n * Wc + twl * M) * CBQ + cq, Wc, raw);
    uint32_t out[2][n];
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int k = 0; k < n; ++k) out[ii][k] = 0u;
#pragma unroll 1
    for (int e = 0; e < 4; ++e) {
      float d[n][n];
#pragma unroll
      for (int j = 0; j < n; ++j)
#pragma unroll
        for (int l = 0; l < n; ++l) {
          d[j][l] = (float)(int)(int8_t)(raw[j][l] & 0xff);
          raw[j][l] >>= 8;
        }
#pragma unroll
      for (int ii = 0; ii < 2; ++ii) {
        float w[n];
#pragma unroll
        for (int l = 0; l < n; ++l) {
          float acc = 0.0f;
#pragma unroll
          for (int j = 0; j < n; ++j)
            if (bt_nonzero<M, kSparse>(i0 + ii, j))
              acc = __builtin_fmaf(bt.v[(i0 + ii) * n + j], d[j][l], acc);
          w[l] = acc;
        }
#pragma unroll
        for (int k = 0; k < n; ++k) {
          float acc = 0.0f;
#pragma unroll
          for (int l = 0; l < n; ++l)
            if (bt_nonzero<M, kSparse>(k, l)) acc = __builtin_fmaf(w[l], bt.v[k * n + l], acc);
          const uint32_t bits =
              quantize_bits(acc, kPos ? rvp.r[(i0 + ii) * n + k] : r_v, lo, hi);
          out[ii][k] = __builtin_amdgcn_perm(bits, out[ii][k], 0x04030201u);
        }
      }
    }
    uint32_t* vp = V + ((size_t)r * g.TW + tw) * cq_per + (c0 >> 2) + cq;
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int k = 0; k < n; ++k) vp[(size_t)((i0 + ii) * n + k) * pstride] = out[ii][k];
  }
  };
  switch (sub) {
    case 0: rows(std::integral_constant<int, 0>{}); break;
    case 1: rows(std::integral_constant<int, 2>{}); break;
    case 2: if constexpr (n > 4) rows(std::integral_constant<int, 4>{}); break;
    default: if constexpr (n > 6) rows(std::integral_constant<int, 6>{}); break;
  }
}

// fp32: one thread per (tile, channel), patch gathered straight from global memory.
template <int M, bool kSparse>
__global__ __launch_bounds__(256) void input_transform_f32(Geom g, MatBT bt,
                                                           const float* __restrict__ x,
                                                           float* __restrict__ V) {
  constexpr int n = M + 2, P = n * n;
  const long long item = (long long)blockIdx.x * 256 + threadIdx.x;
  const int t = (int)(item / g.Cp), c = (int)(item % g.Cp);
  if (t >= g.Tp) return;
  float Vt[n][n];
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int k = 0; k < n; ++k) Vt[i][k] = 0.0f;
  if (t < g.T && c < g.C) {
    const int tw = t % g.TW, th = (t / g.TW) % g.TH, img = t / (g.TW * g.TH);
    const int h0 = th * M - g.pad, w0 = tw * M - g.pad;
    const float* xp = x + ((size_t)img * g.C + c) * g.H * g.W;
    float d[n][n];
#pragma unroll
    for (int j = 0; j < n; ++j)
#pragma unroll
      for (int l = 0; l < n; ++l) {
        const int h = h0 + j, w = w0 + l;
        const bool in = h >= 0 && h < g.H && w >= 0 && w < g.W;
        d[j][l] = in ? xp[h * g.W + w] : 0.0f;
      }
    transform_patch<M, kSparse>(d, bt, Vt);
  }
  const size_t pstride = (size_t)g.Tp * g.Cp;
  float* vp = V + (size_t)t * g.Cp + c;
#pragma unroll
  for (int p = 0; p < P; ++p) vp[p * pstride] = Vt[p / n][p % n];
}

// ----------------------------------------------------------------- weights --
template <int M>
__global__ __launch_bounds__(256) void weight_transform_i8(Geom g, MatG mg,
                                                           const float* __restrict__ w,
                                                           uint32_t* __restrict__ U, PosScale ru,
                                                           float qmax) {
  // One thread per (k, channel quad) and rows i = blockIdx.y, blockIdx.y + gridDim.y, ... of
  // U; i is uniform per block, so the matrix entries stay in scalar registers.  Small layers
  // are launched with one row per block (n times more wavefronts for a latency-bound
  // kernel), large ones with all rows in one thread (the filters are read once).
  // Lanes run over (channel quad & 3, k & 15, the rest): a wavefront's 64 dwords of one
  // position are then 256 consecutive bytes of the blocked layout (see u_byte_index).
  constexpr int n = M + 2;
  const int cq_per = g.Cp >> 2;
  const long long item = (long long)blockIdx.x * 256 + threadIdx.x;
  const int lo6 = (int)(item & 63);
  const long long hi = item >> 6;                      // (k >> 4, cq >> 2), cq >> 2 fastest
  const int cqh = (int)(hi % (cq_per >> 2)), kh = (int)(hi / (cq_per >> 2));
  const int k = kh * 16 + (lo6 >> 2), cq = cqh * 4 + (lo6 & 3);
  if (k >= g.Kp) return;
  float wv[4][9];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int c = cq * 4 + e;
    const bool ok = k < g.K && c < g.C;               // padding: zero filters give zero codes
    const float* wp = w + ((size_t)(ok ? k : 0) * g.C + (ok ? c : 0)) * 9;
#pragma unroll
    for (int a = 0; a < 9; ++a) {
      const float v = wp[a];
      wv[e][a] = ok ? v : 0.0f;
    }
  }
  const size_t pstride = (size_t)g.Kp * cq_per;        // dwords per position
  uint32_t* ub = U + u_byte_index(g.Kp, g.Cp, 1, 0, k, cq * 4) / 4;
  for (int i = blockIdx.y; i < n; i += gridDim.y) {
    const float gi0 = mg.v[i * 3 + 0], gi1 = mg.v[i * 3 + 1], gi2 = mg.v[i * 3 + 2];
    uint32_t out[n];
#pragma unroll
    for (int j = 0; j < n; ++j) out[j] = 0u;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float t[3];
#pragma unroll
      for (int b = 0; b < 3; ++b) {        // t[b] = (G g)[i][b]
        float acc = 0.0f;
        acc = __builtin_fmaf(gi0, wv[e][0 * 3 + b], acc);
        acc = __builtin_fmaf(gi1, wv[e][1 * 3 + b], acc);
        acc = __builtin_fmaf(gi2, wv[e][2 * 3 + b], acc);
        t[b] = acc;
      }
#pragma unroll
      for (int j = 0; j < n; ++j) {        // U[i][j] = sum_b t[b] G[j][b]
        float acc = 0.0f;
#pragma unroll
        for (int b = 0; b < 3; ++b) acc = __builtin_fmaf(t[b], mg.v[j * 3 + b], acc);
        const int q = quantize(acc, ru.r[i * n + j], qmax);   // one factor per position
        out[j] |= (uint32_t)(q & 0xff) << (8 * e);
      }
    }
    // blocked layout: same place in every position's slab
    uint32_t* up = ub + (size_t)i * n * pstride;
#pragma unroll
    for (int j = 0; j < n; ++j) up[j * pstride] = out[j];
  }
}

// kBF: results rounded to bf16 (nearest even) and stored in the layout of ubf_index.
template <int M, bool kBF = false>
__global__ __launch_bounds__(256) void weight_transform_f32(Geom g, MatG mg,
                                                            const float* __restrict__ w,
                                                            float* __restrict__ U) {
  constexpr int n = M + 2, P = n * n;
  const long long item = (long long)blockIdx.x * 256 + threadIdx.x;
  const int k = (int)(item / g.Cp), c = (int)(item % g.Cp);
  if (k >= g.Kp) return;
  float Ut[n][n];
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int j = 0; j < n; ++j) Ut[i][j] = 0.0f;
  if (k < g.K && c < g.C) {
    const float* wp = w + ((size_t)k * g.C + c) * 9;
    float gk[3][3];
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
      for (int b = 0; b < 3; ++b) gk[a][b] = wp[a * 3 + b];
    transform_filter<n>(gk, mg, Ut);
  }
  // blocked layout (see u_byte_index / ubf_index): same place in every position's slab
  const size_t pstride = (size_t)g.Kp * g.Cp;
  if constexpr (kBF) {
    __bf16* up = (__bf16*)U + ubf_index(g.Kp, g.Cp, 0, k, c);
#pragma unroll
    for (int p = 0; p < P; ++p) up[p * pstride] = (__bf16)Ut[p / n][p % n];
  } else {
    float* up = U + u_byte_index(g.Kp, g.Cp, 4, 0, k, c) / 4;
#pragma unroll
    for (int p = 0; p < P; ++p) up[p * pstride] = Ut[p / n][p % n];
  }
}

// ------------------------------------------------------------------ output --
// Stand-alone output transform, used when M is materialised (layers whose accumulators
// do not fit the fused kernels, per-stage calls, the parity tap).  One thread per
// (tile, output channel); lanes run along k so that the reads of M are contiguous.
// kPos: per-position scales -- every accumulator is first brought to real units,
// (float)M * wp.r[p], before the optional quantizer and the transform.
template <int M, bool I8, bool kSparse, bool kMQ, bool kPos = false>
__global__ __launch_bounds__(256) void output_transform(Geom g, MatAT at,
                                                        const void* __restrict__ Mv,
                                                        void* __restrict__ yv, float r_m,
                                                        float r_y, float qmax, PosScale wp) {
  constexpr int n = M + 2;
  const long long item = (long long)blockIdx.x * 256 + threadIdx.x;
  const int t = (int)(item / g.Kp), k = (int)(item % g.Kp);
  if (t >= g.T || k >= g.K) return;
  const size_t pstride = (size_t)g.Tp * g.Kp;
  const size_t base = (size_t)t * g.Kp + k;
  float Mt[n][n], Y[M][M];
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int j = 0; j < n; ++j) {
      if (I8) {
        float f = (float)((const int32_t*)Mv)[(i * n + j) * pstride + base];
        if constexpr (kPos) f = f * wp.r[i * n + j];
        if constexpr (kMQ) f = quantize_f(f, r_m, qmax);
        Mt[i][j] = f;
      } else {
        Mt[i][j] = ((const float*)Mv)[(i * n + j) * pstride + base];
      }
    }
  transform_result<M, kSparse>(Mt, at, Y);
  const int tw = t % g.TW, th = (t / g.TW) % g.TH, img = t / (g.TW * g.TH);
  store_tile<M, I8>(g, yv, ((size_t)img * g.K + k) * g.Ho * g.Wo, th * M, tw * M, Y, r_y,
                    kMagic - qmax, kMagic + qmax);
}

// ------------------------------------------------------------------- taps --
// out[p][r][c] (dense rows x cols) <- src[p][r][c] (padded rowsP x colsP).
template <typename T>
__global__ __launch_bounds__(256) void export_kernel(const T* __restrict__ src,
                                                     T* __restrict__ out, int P, int rows, int cols,
                                                     int rowsP, int colsP) {
  const long long total = (long long)P * rows * cols;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total;
       i += (long long)gridDim.x * 256) {
    const int c = (int)(i % cols);
    const long long pr = i / cols;
    const int r = (int)(pr % rows), p = (int)(pr / rows);
    out[i] = src[((size_t)p * rowsP + r) * colsP + c];
  }
}

// The same for the transformed weights, which live in the blocked layout.
template <typename T>
__global__ __launch_bounds__(256) void export_u_kernel(const T* __restrict__ src,
                                                       T* __restrict__ out, int P, int K, int C,
                                                       int Kp, int Cp) {
  const long long total = (long long)P * K * C;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total;
       i += (long long)gridDim.x * 256) {
    const int c = (int)(i % C);
    const long long pk = i / C;
    const int k = (int)(pk % K), p = (int)(pk / K);
    out[i] = src[u_byte_index(Kp, Cp, (int)sizeof(T), p, k, c) / sizeof(T)];
  }
}

unsigned blocks_for(long long items) { return (unsigned)((items + 255) / 256); }

// Block shape of the int8 input transform: TWB tiles of RB tile rows per workgroup,
// about 16 tiles (256 threads x 1 item), LDS kept under 64 KB.
template <int M, bool kSparse>
hipError_t launch_input_i8(const Geom& g, const MatBT& bt, const int8_t* x, uint32_t* V, float r_v,
                           float qmax, hipStream_t s, const PosScale* rv_pos) {
  constexpr int n = M + 2;
  const int R = g.N * g.TH;
  // 16, 8 or 4 tiles per workgroup: the largest that still gives every CU several
  // workgroups to overlap one's loads with another's math.
  const long long tc = (long long)R * g.TW * (g.Cp / 64);      // tiles x channel blocks
  int tiles = 16;
  while (tiles > 4 && tc / tiles < 1024) tiles >>= 1;
  int TWB = g.TW < tiles ? g.TW : tiles;
  int RB = tiles / TWB;
  if (RB > R) RB = R;
  if (RB < 1) RB = 1;
  auto lds_bytes = [&](int rb, int twb) { return (size_t)stage_dwords<M>(rb, twb) * 4; };
  while (lds_bytes(RB, TWB) > 65536 && RB > 1) --RB;
  while (lds_bytes(RB, TWB) > 65536 && TWB > 1) --TWB;
  const int ntwb = (g.TW + TWB - 1) / TWB, nrb = (R + RB - 1) / RB;
  if ((long long)ntwb * nrb > 0x7fffffffLL || g.Cp / 64 > 65535) return hipErrorInvalidValue;
  dim3 grid((unsigned)(ntwb * nrb), (unsigned)(g.Cp / 64));
  int threads = RB * TWB * 16;
  threads = threads <= 64 ? 64 : threads <= 128 ? 128 : 256;
  const int strip = n * (stage_cols(M, TWB) / 4);          // staging lanes one strip needs
  while (threads < strip) threads *= 2;
  if (threads > 256) return hipErrorInvalidValue;          // cannot happen for TWB <= 16
  const size_t lb = lds_bytes(RB, TWB);
  PosScale none;
  memset(&none, 0, sizeof none);
  // few tiles (one wavefront per workgroup, less than one per SIMD): split the rows of V
  // over (M + 2) / 2 wavefronts (with more wavefronts the kernel is bound by its
  // instruction count, which the split raises: every wavefront unpacks the whole patch)
  if (threads == 64 && (long long)ntwb * nrb * (g.Cp / 64) < 1024) {
#define WINO_LAUNCH_INR(WIDE, POS)                                                         \
  input_transform_i8_rows<M, kSparse, WIDE, POS><<<grid, 32 * n, lb, s>>>(                  \
      g, bt, x, V, r_v, qmax, RB, TWB, POS ? *rv_pos : none)
    if (g.W >= 4) {
      if (rv_pos) WINO_LAUNCH_INR(true, true); else WINO_LAUNCH_INR(true, false);
    } else {
      if (rv_pos) WINO_LAUNCH_INR(false, true); else WINO_LAUNCH_INR(false, false);
    }
#undef WINO_LAUNCH_INR
    return hipGetLastError();
  }
#define WINO_LAUNCH_IN(WIDE, POS)                                                          \
  input_transform_i8<M, kSparse, WIDE, POS><<<grid, threads, lb, s>>>(g, bt, x, V, r_v, qmax, RB, \
                                                                       TWB, POS ? *rv_pos : none)
  if (g.W >= 4) {
    if (rv_pos) WINO_LAUNCH_IN(true, true); else WINO_LAUNCH_IN(true, false);
  } else {
    if (rv_pos) WINO_LAUNCH_IN(false, true); else WINO_LAUNCH_IN(false, false);
  }
#undef WINO_LAUNCH_IN
  return hipGetLastError();
}

template <int M>
hipError_t launch_input_m(const Geom& g, const MatBT& bt, const void* x, void* V, float r_v,
                          float qmax, hipStream_t s, const PosScale* rv_pos) {
  const bool sparse = fits_mask(bt.v, g.n * g.n, CookToomMask<M>::bt);
  if (g.i8) {
    return sparse ? launch_input_i8<M, true>(g, bt, (const int8_t*)x, (uint32_t*)V, r_v, qmax, s,
                                             rv_pos)
                  : launch_input_i8<M, false>(g, bt, (const int8_t*)x, (uint32_t*)V, r_v, qmax, s,
                                              rv_pos);
  }
  const unsigned nb = blocks_for((long long)g.Tp * g.Cp);
  if (sparse)
    input_transform_f32<M, true><<<nb, 256, 0, s>>>(g, bt, (const float*)x, (float*)V);
  else
    input_transform_f32<M, false><<<nb, 256, 0, s>>>(g, bt, (const float*)x, (float*)V);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_input_transform(const Geom& g, const MatBT& bt, const void* x, void* V, float r_v,
                                  float qmax, hipStream_t s, const PosScale* rv_pos) {
  switch (g.m) {
    case 2: return launch_input_m<2>(g, bt, x, V, r_v, qmax, s, rv_pos);
    case 4: return launch_input_m<4>(g, bt, x, V, r_v, qmax, s, rv_pos);
    default: return launch_input_m<6>(g, bt, x, V, r_v, qmax, s, rv_pos);
  }
}

hipError_t launch_weight_transform(const Geom& g, const MatG& mg, const float* w, void* U, float r_u,
                                   float qmax, hipStream_t s, const PosScale* ru_pos) {
  if (g.i8) {
    PosScale ru;                                       // per-tensor: the same factor everywhere
    for (int p = 0; p < 64; ++p) ru.r[p] = ru_pos ? ru_pos->r[p] : r_u;
    const unsigned nb = blocks_for((long long)g.Kp * (g.Cp / 4));
    uint32_t* Uo = (uint32_t*)U;
    // rows per block: one for small layers; with many blocks, all rows in one thread
    const unsigned ny = nb >= 1024 ? 1u : nb >= 256 ? 2u : (unsigned)g.n;
    switch (g.m) {
      case 2: weight_transform_i8<2><<<dim3(nb, ny), 256, 0, s>>>(g, mg, w, Uo, ru, qmax); break;
      case 4: weight_transform_i8<4><<<dim3(nb, ny), 256, 0, s>>>(g, mg, w, Uo, ru, qmax); break;
      default: weight_transform_i8<6><<<dim3(nb, ny), 256, 0, s>>>(g, mg, w, Uo, ru, qmax); break;
    }
  } else {
    const unsigned nb = blocks_for((long long)g.Kp * g.Cp);
    float* Uo = (float*)U;
    if (g.bf16) {
      if (g.m == 2) weight_transform_f32<2, true><<<nb, 256, 0, s>>>(g, mg, w, Uo);
      else if (g.m == 4) weight_transform_f32<4, true><<<nb, 256, 0, s>>>(g, mg, w, Uo);
      else return hipErrorInvalidValue;
      return hipGetLastError();
    }
    switch (g.m) {
      case 2: weight_transform_f32<2><<<nb, 256, 0, s>>>(g, mg, w, Uo); break;
      case 4: weight_transform_f32<4><<<nb, 256, 0, s>>>(g, mg, w, Uo); break;
      default: weight_transform_f32<6><<<nb, 256, 0, s>>>(g, mg, w, Uo); break;
    }
  }
  return hipGetLastError();
}

namespace {
// Output transform, four channels per lane: the lane layout of the MFMA result (lane =
// tile r of 16, channel quad grp; wavefront w = channels 16 w .. 16 w + 15 of a 64-channel
// block), so every load moves 16 bytes per lane, the four wavefronts of a workgroup read
// 256 contiguous bytes per tile and position, and the lane-local transform and the tile
// stores are the ones of the fused kernels (16 consecutive tiles store side by side).
// For m = 2 and 4; the 8 x 8 accumulator sets of m = 6 do not fit beside the temporaries.
template <int M, bool I8, bool kSparse, bool kMQ, bool kFast>
__global__ __launch_bounds__(256) void output_transform_quad(Geom g, MatAT at,
                                                             const void* __restrict__ Mv,
                                                             void* __restrict__ yv, float r_m,
                                                             float r_y, float qmax) {
  constexpr int n = M + 2, P = n * n;
  typedef typename Acc<I8>::type acc_t;
  const int lane = threadIdx.x & 63, r = lane & 15, grp = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int t = blockIdx.x * 16 + r, k0 = blockIdx.y * 64 + wave * 16 + grp * 4;
  // uniform base per position + one 32-bit lane offset (the host checks the range);
  // rows t < Tp and channels k0 + 3 < Kp exist in M whatever T and K are
  const size_t pstride = (size_t)g.Tp * g.Kp * 4;
  const uint32_t off = ((uint32_t)t * (uint32_t)g.Kp + (uint32_t)k0) * 4u;
  const char* Mb = (const char*)Mv;
  acc_t acc[P];
#pragma unroll
  for (int p = 0; p < P; ++p) acc[p] = *(const acc_t*)(Mb + p * pstride + off);
  if (t >= g.T || k0 >= g.K) return;
  const int tw = t % g.TW, th = (t / g.TW) % g.TH, img = t / (g.TW * g.TH);
  finish_lane<M, I8, kSparse, kMQ, kFast>(g, at, acc, yv, img, th, tw, k0, r_m, r_y, qmax);
}

template <int M, bool I8>
hipError_t launch_output_quad(const Geom& g, const MatAT& at, const void* Mv, void* y, float r_m,
                              float r_y, float qmax, hipStream_t s) {
  if (g.Kp / 64 > 65535) return hipErrorInvalidValue;
  dim3 grid(g.Tp / 16, g.Kp / 64);
  const bool sparse = sparse_at<M>(at.v);
  const bool mq = I8 && r_m > 0.0f;
  const bool fast = I8 && !mq && sparse && g.Ho % M == 0 && g.Wo % M == 0 && g.K % 4 == 0;
  if (fast)
    output_transform_quad<M, I8, true, false, I8><<<grid, 256, 0, s>>>(g, at, Mv, y, r_m, r_y, qmax);
  else if (mq && sparse)
    output_transform_quad<M, I8, true, I8, false><<<grid, 256, 0, s>>>(g, at, Mv, y, r_m, r_y, qmax);
  else if (mq)
    output_transform_quad<M, I8, false, I8, false><<<grid, 256, 0, s>>>(g, at, Mv, y, r_m, r_y, qmax);
  else if (sparse)
    output_transform_quad<M, I8, true, false, false><<<grid, 256, 0, s>>>(g, at, Mv, y, r_m, r_y, qmax);
  else
    output_transform_quad<M, I8, false, false, false><<<grid, 256, 0, s>>>(g, at, Mv, y, r_m, r_y, qmax);
  return hipGetLastError();
}
}  // namespace

namespace {
template <int M, bool I8>
hipError_t launch_output_m(const Geom& g, const MatAT& at, const void* Mv, void* y, float r_m,
                           float r_y, float qmax, hipStream_t s, const PosScale* w_pos) {
  const unsigned nb = blocks_for((long long)g.T * g.Kp);
  const bool sparse = sparse_at<M>(at.v);
  const bool mq = I8 && r_m > 0.0f;
  PosScale none;
  memset(&none, 0, sizeof none);
#define WINO_LAUNCH_OUT(SP, MQ, POS)                                                         \
  output_transform<M, I8, SP, MQ, POS><<<nb, 256, 0, s>>>(g, at, Mv, y, r_m, r_y, qmax,        \
                                                          POS ? *w_pos : none)
  if (I8 && w_pos) {
    if (mq) { if (sparse) WINO_LAUNCH_OUT(true, I8, I8); else WINO_LAUNCH_OUT(false, I8, I8); }
    else    { if (sparse) WINO_LAUNCH_OUT(true, false, I8); else WINO_LAUNCH_OUT(false, false, I8); }
  } else if (mq) {
    if (sparse) WINO_LAUNCH_OUT(true, I8, false); else WINO_LAUNCH_OUT(false, I8, false);
  } else {
    if (sparse) WINO_LAUNCH_OUT(true, false, false); else WINO_LAUNCH_OUT(false, false, false);
  }
#undef WINO_LAUNCH_OUT
  return hipGetLastError();
}
}  // namespace

hipError_t launch_output_transform(const Geom& g, const MatAT& at, const void* M, void* y, float r_m,
                                   float r_y, float qmax, hipStream_t s, const PosScale* w_pos) {
  // four channels per lane: needs 32-bit lane offsets, and enough workgroups (16 tiles x
  // 64 channels each) for one per compute unit; below that the thread-per-(tile,
  // channel) kernel spreads the work further
  const bool quad = !w_pos && (unsigned long long)g.Tp * g.Kp * 4 < 0x100000000ull &&
                    (long long)(g.Tp / 16) * (g.Kp / 64) >= 256;
  if (g.i8) {
    switch (g.m) {
      case 2: return quad ? launch_output_quad<2, true>(g, at, M, y, r_m, r_y, qmax, s)
                          : launch_output_m<2, true>(g, at, M, y, r_m, r_y, qmax, s, w_pos);
      case 4: return quad ? launch_output_quad<4, true>(g, at, M, y, r_m, r_y, qmax, s)
                          : launch_output_m<4, true>(g, at, M, y, r_m, r_y, qmax, s, w_pos);
      default: return launch_output_m<6, true>(g, at, M, y, r_m, r_y, qmax, s, w_pos);
    }
  }
  switch (g.m) {
    case 2: return quad ? launch_output_quad<2, false>(g, at, M, y, r_m, r_y, qmax, s)
                        : launch_output_m<2, false>(g, at, M, y, r_m, r_y, qmax, s, w_pos);
    case 4: return quad ? launch_output_quad<4, false>(g, at, M, y, r_m, r_y, qmax, s)
                        : launch_output_m<4, false>(g, at, M, y, r_m, r_y, qmax, s, w_pos);
    default: return launch_output_m<6, false>(g, at, M, y, r_m, r_y, qmax, s, w_pos);
  }
}

hipError_t launch_export(const Geom& g, int which, const void* src, void* out, hipStream_t s) {
  int rows, cols, rowsP, colsP, esz;
  if (which == WINO_TAP_U) {
    rows = g.K; cols = g.C; rowsP = g.Kp; colsP = g.Cp; esz = g.i8 ? 1 : 4;
  } else if (which == WINO_TAP_V) {
    rows = g.T; cols = g.C; rowsP = g.Tp; colsP = g.Cp; esz = g.i8 ? 1 : 4;
  } else {
    rows = g.T; cols = g.K; rowsP = g.Tp; colsP = g.Kp; esz = 4;
  }
  const long long total = (long long)g.P * rows * cols;
  const unsigned nb = (unsigned)((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
  if (which == WINO_TAP_U && g.i8)
    export_u_kernel<int8_t><<<nb, 256, 0, s>>>((const int8_t*)src, (int8_t*)out, g.P, g.K, g.C, g.Kp, g.Cp);
  else if (which == WINO_TAP_U)
    export_u_kernel<uint32_t><<<nb, 256, 0, s>>>((const uint32_t*)src, (uint32_t*)out, g.P, g.K, g.C, g.Kp, g.Cp);
  else if (esz == 1)
    export_kernel<int8_t><<<nb, 256, 0, s>>>((const int8_t*)src, (int8_t*)out, g.P, rows, cols,
                                              rowsP, colsP);
  else
    export_kernel<uint32_t><<<nb, 256, 0, s>>>((const uint32_t*)src, (uint32_t*)out, g.P, rows,
                                                cols, rowsP, colsP);
  return hipGetLastError();
}

}  // namespace wino
