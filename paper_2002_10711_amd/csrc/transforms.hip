// Transform kernels of the Winograd-aware layer (paper, Sec. 3.1 Eq. 1 and
// Sec. 3.2): input transform B^T d B, weight transform G g G^T, output transform
// A^T M A, each followed by the stage's quantizer in int8 mode, plus the copy
// kernel behind the parity taps.
//
// Arithmetic contract of the int8 mode (what makes an integer result well defined
// for arbitrary real matrices): IEEE fp32; every sum is the chain
// acc = +0; acc = fma(a_j, b_j, acc) over ascending j; the first product of a
// two-sided transform is the left one (B^T d, G g, A^T M); the scale is applied
// by one fp32 multiplication; rounding is half-to-even; saturation to
// [-qmax, qmax] is done in float before the integer conversion.
//
// The matrices arrive by value in the kernel arguments (scalar registers), never
// as compiled-in constants, so learned transforms use the same code.
#include "wino_internal.h"

namespace wino {
namespace {

__device__ __forceinline__ int quantize(float v, float r, float qmax) {
  float s = v * r;
  s = __builtin_rintf(s);
  s = fminf(fmaxf(s, -qmax), qmax);
  return (int)s;
}

// ------------------------------------------------------------------ input --
// V = B^T d B for one n x n patch held in registers.
template <int n>
__device__ __forceinline__ void transform_patch(const float (&d)[n][n], const MatBT& bt,
                                                float (&V)[n][n]) {
  float w[n][n];
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int l = 0; l < n; ++l) {
      float acc = 0.0f;
#pragma unroll
      for (int j = 0; j < n; ++j) acc = __builtin_fmaf(bt.v[i * n + j], d[j][l], acc);
      w[i][l] = acc;
    }
#pragma unroll
  for (int i = 0; i < n; ++i)
#pragma unroll
    for (int k = 0; k < n; ++k) {
      float acc = 0.0f;
#pragma unroll
      for (int l = 0; l < n; ++l) acc = __builtin_fmaf(w[i][l], bt.v[k * n + l], acc);
      V[i][k] = acc;
    }
}

// int8: one thread per (tile, group of 4 channels); the four int8 results of a
// Winograd position are packed into one dword so that a wavefront writes 256
// contiguous bytes per position.
template <int M>
__global__ __launch_bounds__(256) void input_transform_i8(Geom g, MatBT bt,
                                                          const int8_t* __restrict__ x,
                                                          uint32_t* __restrict__ V, float r_v,
                                                          float qmax) {
  constexpr int n = M + 2, P = n * n;
  const int cq_per = g.Cp >> 2;
  const long long item = (long long)blockIdx.x * 256 + threadIdx.x;
  const int t = (int)(item / cq_per), cq = (int)(item % cq_per);
  if (t >= g.Tp) return;
  uint32_t out[P];
#pragma unroll
  for (int p = 0; p < P; ++p) out[p] = 0u;
  if (t < g.T) {
    const int tw = t % g.TW, th = (t / g.TW) % g.TH, img = t / (g.TW * g.TH);
    const int h0 = th * M - g.pad, w0 = tw * M - g.pad;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int c = cq * 4 + e;
      if (c < g.C) {
        const int8_t* xp = x + ((size_t)img * g.C + c) * g.H * g.W;
        float d[n][n], Vt[n][n];
#pragma unroll
        for (int j = 0; j < n; ++j)
#pragma unroll
          for (int l = 0; l < n; ++l) {
            const int h = h0 + j, w = w0 + l;
            const bool in = h >= 0 && h < g.H && w >= 0 && w < g.W;
            d[j][l] = in ? (float)xp[h * g.W + w] : 0.0f;
          }
        transform_patch<n>(d, bt, Vt);
#pragma unroll
        for (int i = 0; i < n; ++i)
#pragma unroll
          for (int k = 0; k < n; ++k) {
            const int q = quantize(Vt[i][k], r_v, qmax);
            out[i * n + k] |= (uint32_t)(q & 0xff) << (8 * e);
          }
      }
    }
  }
  const size_t pstride = (size_t)g.Tp * cq_per;
  uint32_t* vp = V + (size_t)t * cq_per + cq;
#pragma unroll
  for (int p = 0; p < P; ++p) vp[p * pstride] = out[p];
}

// fp32: one thread per (tile, channel).
template <int M>
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
    transform_patch<n>(d, bt, Vt);
  }
  const size_t pstride = (size_t)g.Tp * g.Cp;
  float* vp = V + (size_t)t * g.Cp + c;
#pragma unroll
  for (int p = 0; p < P; ++p) vp[p * pstride] = Vt[p / n][p % n];
}

// ----------------------------------------------------------------- weights --
// U = G g G^T for one (k, c).
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

template <int M>
__global__ __launch_bounds__(256) void weight_transform_i8(Geom g, MatG mg,
                                                           const float* __restrict__ w,
                                                           uint32_t* __restrict__ U, float r_u,
                                                           float qmax) {
  constexpr int n = M + 2, P = n * n;
  const int cq_per = g.Cp >> 2;
  const long long item = (long long)blockIdx.x * 256 + threadIdx.x;
  const int k = (int)(item / cq_per), cq = (int)(item % cq_per);
  if (k >= g.Kp) return;
  uint32_t out[P];
#pragma unroll
  for (int p = 0; p < P; ++p) out[p] = 0u;
  if (k < g.K) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int c = cq * 4 + e;
      if (c < g.C) {
        const float* wp = w + ((size_t)k * g.C + c) * 9;
        float gk[3][3], Ut[n][n];
#pragma unroll
        for (int a = 0; a < 3; ++a)
#pragma unroll
          for (int b = 0; b < 3; ++b) gk[a][b] = wp[a * 3 + b];
        transform_filter<n>(gk, mg, Ut);
#pragma unroll
        for (int i = 0; i < n; ++i)
#pragma unroll
          for (int j = 0; j < n; ++j) {
            const int q = quantize(Ut[i][j], r_u, qmax);
            out[i * n + j] |= (uint32_t)(q & 0xff) << (8 * e);
          }
      }
    }
  }
  const size_t pstride = (size_t)g.Kp * cq_per;
  uint32_t* up = U + (size_t)k * cq_per + cq;
#pragma unroll
  for (int p = 0; p < P; ++p) up[p * pstride] = out[p];
}

template <int M>
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
  const size_t pstride = (size_t)g.Kp * g.Cp;
  float* up = U + (size_t)k * g.Cp + c;
#pragma unroll
  for (int p = 0; p < P; ++p) up[p * pstride] = Ut[p / n][p % n];
}

// ------------------------------------------------------------------ output --
// Yt = A^T Mt A for one (tile, output channel).
template <int M>
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
      for (int i = 0; i < n; ++i) acc = __builtin_fmaf(at.v[a * n + i], Mt[i][j], acc);
      z[a][j] = acc;
    }
#pragma unroll
  for (int a = 0; a < M; ++a)
#pragma unroll
    for (int b = 0; b < M; ++b) {
      float acc = 0.0f;
#pragma unroll
      for (int j = 0; j < n; ++j) acc = __builtin_fmaf(z[a][j], at.v[b * n + j], acc);
      Y[a][b] = acc;
    }
}

// One thread per (tile, output channel); lanes run along k so that the reads of M
// are contiguous.
template <int M, bool I8>
__global__ __launch_bounds__(256) void output_transform(Geom g, MatAT at,
                                                        const void* __restrict__ Mv,
                                                        void* __restrict__ yv, float r_m,
                                                        float r_y, float qmax) {
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
        if (r_m > 0.0f) f = (float)quantize(f, r_m, qmax);
        Mt[i][j] = f;
      } else {
        Mt[i][j] = ((const float*)Mv)[(i * n + j) * pstride + base];
      }
    }
  transform_result<M>(Mt, at, Y);
  const int tw = t % g.TW, th = (t / g.TW) % g.TH, img = t / (g.TW * g.TH);
  const size_t ybase = ((size_t)img * g.K + k) * g.Ho * g.Wo;
#pragma unroll
  for (int a = 0; a < M; ++a)
#pragma unroll
    for (int b = 0; b < M; ++b) {
      const int h = th * M + a, w = tw * M + b;
      if (h < g.Ho && w < g.Wo) {
        if (I8)
          ((int8_t*)yv)[ybase + (size_t)h * g.Wo + w] = (int8_t)quantize(Y[a][b], r_y, qmax);
        else
          ((float*)yv)[ybase + (size_t)h * g.Wo + w] = Y[a][b];
      }
    }
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

unsigned blocks_for(long long items) { return (unsigned)((items + 255) / 256); }

}  // namespace

hipError_t launch_input_transform(const Geom& g, const MatBT& bt, const void* x, void* V, float r_v,
                                  float qmax, hipStream_t s) {
  if (g.i8) {
    const unsigned nb = blocks_for((long long)g.Tp * (g.Cp / 4));
    const int8_t* xi = (const int8_t*)x;
    uint32_t* Vo = (uint32_t*)V;
    switch (g.m) {
      case 2: input_transform_i8<2><<<nb, 256, 0, s>>>(g, bt, xi, Vo, r_v, qmax); break;
      case 4: input_transform_i8<4><<<nb, 256, 0, s>>>(g, bt, xi, Vo, r_v, qmax); break;
      default: input_transform_i8<6><<<nb, 256, 0, s>>>(g, bt, xi, Vo, r_v, qmax); break;
    }
  } else {
    const unsigned nb = blocks_for((long long)g.Tp * g.Cp);
    const float* xf = (const float*)x;
    float* Vo = (float*)V;
    switch (g.m) {
      case 2: input_transform_f32<2><<<nb, 256, 0, s>>>(g, bt, xf, Vo); break;
      case 4: input_transform_f32<4><<<nb, 256, 0, s>>>(g, bt, xf, Vo); break;
      default: input_transform_f32<6><<<nb, 256, 0, s>>>(g, bt, xf, Vo); break;
    }
  }
  return hipGetLastError();
}

hipError_t launch_weight_transform(const Geom& g, const MatG& mg, const float* w, void* U, float r_u,
                                   float qmax, hipStream_t s) {
  if (g.i8) {
    const unsigned nb = blocks_for((long long)g.Kp * (g.Cp / 4));
    uint32_t* Uo = (uint32_t*)U;
    switch (g.m) {
      case 2: weight_transform_i8<2><<<nb, 256, 0, s>>>(g, mg, w, Uo, r_u, qmax); break;
      case 4: weight_transform_i8<4><<<nb, 256, 0, s>>>(g, mg, w, Uo, r_u, qmax); break;
      default: weight_transform_i8<6><<<nb, 256, 0, s>>>(g, mg, w, Uo, r_u, qmax); break;
    }
  } else {
    const unsigned nb = blocks_for((long long)g.Kp * g.Cp);
    float* Uo = (float*)U;
    switch (g.m) {
      case 2: weight_transform_f32<2><<<nb, 256, 0, s>>>(g, mg, w, Uo); break;
      case 4: weight_transform_f32<4><<<nb, 256, 0, s>>>(g, mg, w, Uo); break;
      default: weight_transform_f32<6><<<nb, 256, 0, s>>>(g, mg, w, Uo); break;
    }
  }
  return hipGetLastError();
}

hipError_t launch_output_transform(const Geom& g, const MatAT& at, const void* M, void* y, float r_m,
                                   float r_y, float qmax, hipStream_t s) {
  const unsigned nb = blocks_for((long long)g.T * g.Kp);
  if (g.i8) {
    switch (g.m) {
      case 2: output_transform<2, true><<<nb, 256, 0, s>>>(g, at, M, y, r_m, r_y, qmax); break;
      case 4: output_transform<4, true><<<nb, 256, 0, s>>>(g, at, M, y, r_m, r_y, qmax); break;
      default: output_transform<6, true><<<nb, 256, 0, s>>>(g, at, M, y, r_m, r_y, qmax); break;
    }
  } else {
    switch (g.m) {
      case 2: output_transform<2, false><<<nb, 256, 0, s>>>(g, at, M, y, r_m, r_y, qmax); break;
      case 4: output_transform<4, false><<<nb, 256, 0, s>>>(g, at, M, y, r_m, r_y, qmax); break;
      default: output_transform<6, false><<<nb, 256, 0, s>>>(g, at, M, y, r_m, r_y, qmax); break;
    }
  }
  return hipGetLastError();
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
  if (esz == 1)
    export_kernel<int8_t><<<nb, 256, 0, s>>>((const int8_t*)src, (int8_t*)out, g.P, rows, cols,
                                              rowsP, colsP);
  else
    export_kernel<uint32_t><<<nb, 256, 0, s>>>((const uint32_t*)src, (uint32_t*)out, g.P, rows,
                                                cols, rowsP, colsP);
  return hipGetLastError();
}

}  // namespace wino
