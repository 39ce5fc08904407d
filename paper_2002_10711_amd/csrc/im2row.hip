// The baseline the paper measures Winograd against (Sec. 5.3, Table 3): im2row
// convolution.  Every output pixel becomes a row of the 9*C input taps it reads
// (tap-major, channel fastest), the filters become rows of the same order, one
// GEMM multiplies them, and an epilogue requantizes and scatters to NCHW.
// Stride 1 or 2, 3x3 filters, zero padding.
#include "transform_math.h"

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

// The same int8 weights once more in the order the one-kernel form reads them: 1 KB blocks,
// one per (16 output channels, 64 input channels, tap), [k/16][c/64][tap]; inside a block
// lane (c % 64 / 16) * 16 + k % 16 owns the 16 bytes c % 16 = 0..15 -- the B operand of
// v_mfma_i32_16x16x64_i8, so that a wavefront's load is one contiguous kilobyte (rows of
// 9*Cp bytes made it 16 half cache lines).
__global__ __launch_bounds__(256) void ref_pack_weights_operand_kernel(const int8_t* __restrict__ w,
                                                                       int8_t* __restrict__ wo,
                                                                       int C, int K, int Cp,
                                                                       int Kp) {
  const long long total = (long long)Kp * 9 * Cp;
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int nch = Cp >> 6;
  const int byte = (int)(i & 15), lane = (int)((i >> 4) & 63);
  const long long blk = i >> 10;
  const int tap = (int)(blk % 9), ch = (int)((blk / 9) % nch), kb = (int)(blk / (9LL * nch));
  const int k = kb * 16 + (lane & 15), c = ch * 64 + (lane >> 4) * 16 + byte;
  int8_t v = 0;
  if (k < K && c < C) v = w[((size_t)k * C + c) * 9 + tap];
  wo[i] = v;
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
    ((int8_t*)yv)[o] =
        (int8_t)quantize((float)((const int32_t*)Mv)[(size_t)t * g.Kp + k], r_y, qmax);
  } else {
    ((float*)yv)[o] = ((const float*)Mv)[(size_t)t * g.Kp + k];
  }
}

// The same gather, one workgroup per (image, output row, block of 64 channels): the
// three input rows the output row reads are staged in LDS with loads that run along the
// image rows, then every (pixel, tap) row segment of 64 channels is written as one
// contiguous run (VEC channels per thread).  For rows that fit LDS; the kernel above
// serves the rest.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void im2row_rows_kernel(RefGeom g, const T* __restrict__ x,
                                                          T* __restrict__ rows) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  T* Xs = (T*)lds_raw;                                 // [3][64][Wl], column = w + pad
  const int Wl = g.W + 2;
  const int row = blockIdx.x, cb = blockIdx.y * 64;
  const int img = row / g.Ho, ho = row - img * g.Ho;
  const int tid = threadIdx.x;
  // lanes along the image row (coalesced), wavefronts over the 3 x 64 (row, channel) pairs
  const int tx = tid & 63, ty = tid >> 6;
  for (int col0 = 0; col0 < Wl; col0 += 64) {
    const int col = col0 + tx, w = col - g.pad;
    const bool wok = col < Wl && w >= 0 && w < g.W;
    // (loads from clamped addresses, selected afterwards, eight in flight per lane: a load
    // inside a conditional would wait for each one in turn)
    for (int rc0 = ty; rc0 < 3 * 64; rc0 += 32) {
      T v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int rc = rc0 + 4 * u;
        const int r = rc >> 6, c = rc & 63;
        const int h = ho * g.stride + r - g.pad;
        const bool ok = wok && h >= 0 && h < g.H && cb + c < g.C;
        const size_t off = ok ? (((size_t)img * g.C + cb + c) * g.H + h) * g.W + w : 0;
        const T t = x[off];
        v[u] = ok ? t : (T)0;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (col < Wl) Xs[(rc0 + 4 * u) * Wl + col] = v[u];
    }
  }
  __syncthreads();
  constexpr int CV = 64 / VEC;                         // threads per (pixel, tap)
  const size_t t0 = (size_t)row * g.Wo;
  for (int i = tid; i < g.Wo * 9 * CV; i += 256) {
    const int cv = i % CV, tap = (i / CV) % 9, wo = i / (CV * 9);
    const int r = tap / 3, col = wo * g.stride + tap % 3;          // column index incl. pad
    T v[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[e] = Xs[(r * 64 + cv * VEC + e) * Wl + col];
    T* o = rows + ((t0 + wo) * 9 + tap) * g.Cp + cb + cv * VEC;
    if constexpr (VEC == 4 && sizeof(T) == 1) {
      *(uint32_t*)o = (uint32_t)(uint8_t)v[0] | ((uint32_t)(uint8_t)v[1] << 8) |
                      ((uint32_t)(uint8_t)v[2] << 16) | ((uint32_t)(uint8_t)v[3] << 24);
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) o[e] = v[e];
    }
  }
}

// y <- M through an LDS tile of 64 pixels x 64 channels: M is read along k (its fastest
// axis), y is written along the pixels of one channel (its fastest axis).
template <bool I8>
__global__ __launch_bounds__(256) void ref_epilogue_tiled_kernel(RefGeom g,
                                                                 const void* __restrict__ Mv,
                                                                 void* __restrict__ yv, float r_y,
                                                                 float qmax) {
  __shared__ float tile[64][65];                       // [k][pixel], padded
  const int t0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
  const int tid = threadIdx.x;
  for (int i = tid; i < 64 * 64; i += 256) {
    const int k = i & 63, tl = i >> 6;
    const int t = t0 + tl;
    float s = 0.0f;
    if (t < g.T) {
      if (I8) {
        s = quantize_f((float)((const int32_t*)Mv)[(size_t)t * g.Kp + k0 + k], r_y, qmax);
      } else {
        s = ((const float*)Mv)[(size_t)t * g.Kp + k0 + k];
      }
    }
    tile[k][tl] = s;
  }
  __syncthreads();
  const int hw = g.Ho * g.Wo;
  for (int i = tid; i < 64 * 64; i += 256) {
    const int tl = i & 63, k = i >> 6;
    const int t = t0 + tl;
    if (t >= g.T || k0 + k >= g.K) continue;
    const int img = t / hw, pix = t - img * hw;
    const size_t o = ((size_t)img * g.K + k0 + k) * hw + pix;
    if (I8) ((int8_t*)yv)[o] = (int8_t)(int)tile[k][tl];
    else ((float*)yv)[o] = tile[k][tl];
  }
}

unsigned blocks_for(long long items) { return (unsigned)((items + 255) / 256); }

}  // namespace

hipError_t launch_ref_pack_weights(int C, int K, int Cp, int Kp, int i8, const void* w, void* wp,
                                   hipStream_t s) {
  const unsigned nb = blocks_for((long long)Kp * 9 * Cp);
  if (i8) {
    ref_pack_weights_kernel<int8_t><<<nb, 256, 0, s>>>((const int8_t*)w, (int8_t*)wp, C, K, Cp, Kp);
    ref_pack_weights_operand_kernel<<<nb, 256, 0, s>>>(
        (const int8_t*)w, (int8_t*)wp + ref_operand_weights_offset(Cp, Kp), C, K, Cp, Kp);
  } else
    ref_pack_weights_kernel<float><<<nb, 256, 0, s>>>((const float*)w, (float*)wp, C, K, Cp, Kp);
  return hipGetLastError();
}

hipError_t launch_im2row(const RefGeom& g, const void* x, void* rows, hipStream_t s) {
  // rows of up to 64 KB of LDS: staged kernel (the rows between T and Tp stay unwritten:
  // the GEMM's results for them are never read)
  const size_t lb = (size_t)3 * 64 * (g.W + 2) * (g.i8 ? 1 : 4);
  if (lb <= 65536 && (long long)g.N * g.Ho <= 0x7fffffffLL && g.Cp / 64 >= 1 && g.Cp % 64 == 0 &&
      g.Cp / 64 <= 65535) {
    dim3 grid((unsigned)(g.N * g.Ho), (unsigned)(g.Cp / 64));
    if (g.i8)
      im2row_rows_kernel<int8_t, 4><<<grid, 256, lb, s>>>(g, (const int8_t*)x, (int8_t*)rows);
    else
      im2row_rows_kernel<float, 1><<<grid, 256, lb, s>>>(g, (const float*)x, (float*)rows);
    return hipGetLastError();
  }
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
  if (g.Kp / 64 <= 65535) {
    dim3 grid((unsigned)(g.Tp / 64), (unsigned)(g.Kp / 64));
    if (g.i8)
      ref_epilogue_tiled_kernel<true><<<grid, 256, 0, s>>>(g, M, y, r_y, qmax);
    else
      ref_epilogue_tiled_kernel<false><<<grid, 256, 0, s>>>(g, M, y, r_y, qmax);
    return hipGetLastError();
  }
  const unsigned nb = blocks_for((long long)g.T * g.Kp);
  if (g.i8)
    ref_epilogue_kernel<true><<<nb, 256, 0, s>>>(g, M, y, r_y, qmax);
  else
    ref_epilogue_kernel<false><<<nb, 256, 0, s>>>(g, M, y, r_y, qmax);
  return hipGetLastError();
}

}  // namespace wino
