// The baseline the paper measures Winograd against (Sec. 5.3, Table 3): im2row
// convolution.  Every output pixel becomes a row of the 9*C input taps it reads
// (tap-major, channel fastest), the filters become rows of the same order, one
// GEMM multiplies them, and an epilogue requantizes and scatters to NCHW.
// Stride 1 or 2, 3x3 filters, zero padding.
#include "wino_internal.h"

namespace wino {
namespace {

// wp[k][rs*Cp + c] <- w[k][c][rs]; zero in the padding.
template <typename T>
__global__ __launch_bounds__(256) void ref_pack_weights_kernel(const T* __restrict__ w,
                                                               T* __restrict__ wp, int C, int K,
                                                               int Cp, int Kp) {
  const long long total = (long long)Kp * 9 * Cp;
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % Cp), rs = (int)((i / Cp) % 9), k = (int)(i / (9LL * Cp));
  T v = 0;
  if (k < K && c < C) v = w[((size_t)k * C + c) * 9 + rs];
  wp[i] = v;
}

// rows[t][rs*Cp + c] <- x[img][c][ho*stride + r - pad][wo*stride + s - pad].
// VEC channels per thread (4 int8 packed into a dword, or 1 float).
template <typename T, int VEC>
__global__ __launch_bounds__(256) void im2row_kernel(RefGeom g, const T* __restrict__ x,
                                                     T* __restrict__ rows) {
  const int cv_per = g.Cp / VEC;
  const long long total = (long long)g.Tp * 9 * cv_per;
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int cv = (int)(i % cv_per), rs = (int)((i / cv_per) % 9), t = (int)(i / (9LL * cv_per));
  T v[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) v[e] = 0;
  if (t < g.T) {
    const int wo = t % g.Wo, ho = (t / g.Wo) % g.Ho, img = t / (g.Wo * g.Ho);
    const int h = ho * g.stride + rs / 3 - g.pad, w = wo * g.stride + rs % 3 - g.pad;
    if (h >= 0 && h < g.H && w >= 0 && w < g.W) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const int c = cv * VEC + e;
        if (c < g.C) v[e] = x[(((size_t)img * g.C + c) * g.H + h) * g.W + w];
      }
    }
  }
  T* o = rows + (size_t)i * VEC;
#pragma unroll
  for (int e = 0; e < VEC; ++e) o[e] = v[e];
}

// y[img][k][ho][wo] <- M[t][k], requantized in int8 mode.
template <bool I8>
__global__ __launch_bounds__(256) void ref_epilogue_kernel(RefGeom g, const void* __restrict__ Mv,
                                                           void* __restrict__ yv, float r_y,
                                                           float qmax) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  const int t = (int)(i / g.Kp), k = (int)(i % g.Kp);
  if (t >= g.T || k >= g.K) return;
  const int hw = g.Ho * g.Wo, img = t / hw, pix = t % hw;
  const size_t o = ((size_t)img * g.K + k) * hw + pix;
  if (I8) {
    float s = (float)((const int32_t*)Mv)[(size_t)t * g.Kp + k] * r_y;
    s = __builtin_rintf(s);
    s = fminf(fmaxf(s, -qmax), qmax);
    ((int8_t*)yv)[o] = (int8_t)(int)s;
  } else {
    ((float*)yv)[o] = ((const float*)Mv)[(size_t)t * g.Kp + k];
  }
}

unsigned blocks_for(long long items) { return (unsigned)((items + 255) / 256); }

}  // namespace

hipError_t launch_ref_pack_weights(int C, int K, int Cp, int Kp, int i8, const void* w, void* wp,
                                   hipStream_t s) {
  const unsigned nb = blocks_for((long long)Kp * 9 * Cp);
  if (i8)
    ref_pack_weights_kernel<int8_t><<<nb, 256, 0, s>>>((const int8_t*)w, (int8_t*)wp, C, K, Cp, Kp);
  else
    ref_pack_weights_kernel<float><<<nb, 256, 0, s>>>((const float*)w, (float*)wp, C, K, Cp, Kp);
  return hipGetLastError();
}

hipError_t launch_im2row(const RefGeom& g, const void* x, void* rows, hipStream_t s) {
  if (g.i8) {
    const unsigned nb = blocks_for((long long)g.Tp * 9 * (g.Cp / 4));
    im2row_kernel<int8_t, 4><<<nb, 256, 0, s>>>(g, (const int8_t*)x, (int8_t*)rows);
  } else {
    const unsigned nb = blocks_for((long long)g.Tp * 9 * g.Cp);
    im2row_kernel<float, 1><<<nb, 256, 0, s>>>(g, (const float*)x, (float*)rows);
  }
  return hipGetLastError();
}

hipError_t launch_ref_epilogue(const RefGeom& g, const void* M, void* y, float r_y, float qmax,
                               hipStream_t s) {
  const unsigned nb = blocks_for((long long)g.T * g.Kp);
  if (g.i8)
    ref_epilogue_kernel<true><<<nb, 256, 0, s>>>(g, M, y, r_y, qmax);
  else
    ref_epilogue_kernel<false><<<nb, 256, 0, s>>>(g, M, y, r_y, qmax);
  return hipGetLastError();
}

}  // namespace wino
