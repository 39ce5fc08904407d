// CPU oracle for the Winograd-aware convolution forward path.
//
// TEST INFRASTRUCTURE, NOT PRODUCT.  Slow, plain and meant to be checked against
// the paper by eye.  It is called only by the tests, by the smoke check and by
// the CPU-baseline leg of the benchmark.  It shares no code, header, table or
// helper with the HIP library and is never used as a fallback for it.
//
// What it computes (paper, Sec. 3.1, Eq. 1, applied as Sec. 3.2 describes to
// every patch of the activations):
//
//     Y = A^T [ (G g G^T) (.) (B^T d B) ] A
//
// for F(m x m, 3 x 3): d is an n x n input patch, n = m + 2, patches step by m
// and overlap by 2, Y is the m x m output tile.  For many channels the
// element-wise products are summed over the input channels in the Winograd
// domain (the "GEMM" formulation the paper deploys, Sec. 5.3), then one output
// transform is applied per (tile, output channel).
//
// Three parts:
//   O1  direct 3x3 cross-correlation in fp64 (the plain definition that an
//       unquantized Winograd convolution reaches up to rounding).
//   O2  the literal per-tile evaluation of Eq. 1 in fp64, matrices supplied by
//       the caller (Cook-Toom or perturbed/learned ones).
//   O3  the quantized pipeline of Sec. 3.2 / Fig. 2 (a quantizer after every
//       stage; per-layer symmetric uniform quantization, Sec. 5.1), stage by
//       stage with every intermediate exposed.  Arithmetic is pinned so that an
//       integer result is well defined for arbitrary real matrices:
//       IEEE fp32, every sum a chain acc = +0; acc = fmaf(a_j, b_j, acc) over
//       ascending j; a quantizer rounds the EXACT product of its fp32 input and its
//       fp32 reciprocal step once, to the nearest integer, ties to even, and then
//       saturates to [-qmax, qmax].
//
// Canonical tensor orders (row-major, last index fastest):
//   X[N][C][H][W], g[K][C][3][3], Y[N][K][Ho][Wo], Ho = H + 2 pad - 2,
//   U[p][k][c], V[p][t][c], M[p][t][k] with Winograd position p = i*n + j and
//   tile index t = (img*TH + th)*TW + tw, TH = ceil(Ho/m), TW = ceil(Wo/m).
//   Tile (th, tw) reads input rows th*m - pad + j, columns tw*m - pad + l
//   (zero outside the image) and writes output rows th*m + a, columns tw*m + b
//   (dropped where they fall outside the output).
//
// Parity status: every function here is pinned by tests/test_oracle_pins.py
// (closed forms, brute force, exact identities, the counts the paper prints).
// The one exception is stated there: with perturbed ("flex") matrices there is
// no independent definition of the result, so O2/O3 with such matrices are
// "parity unpinned" beyond the limit noise -> 0.
//
// Build: g++ -O2 -ffp-contract=off -fopenmp -shared -fPIC (no fast-math).

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// C[ar x bc] = A[ar x ac] * B[ac x bc], fp64, plain triple loop.
void matmul(const double* A, int ar, int ac, const double* B, int bc, double* C) {
  for (int i = 0; i < ar; ++i)
    for (int j = 0; j < bc; ++j) {
      double s = 0.0;
      for (int k = 0; k < ac; ++k) s += A[i * ac + k] * B[k * bc + j];
      C[i * bc + j] = s;
    }
}

// C[ar x br] = A[ar x ac] * B^T, with B stored [br x ac].
void matmul_bt(const double* A, int ar, int ac, const double* B, int br, double* C) {
  for (int i = 0; i < ar; ++i)
    for (int j = 0; j < br; ++j) {
      double s = 0.0;
      for (int k = 0; k < ac; ++k) s += A[i * ac + k] * B[j * ac + k];
      C[i * br + j] = s;
    }
}

// Symmetric uniform quantizer q = sat(rne(v * r)) (Sec. 5.1: per-layer symmetric uniform
// quantization; r is the reciprocal step, an fp32 number from the host).  The product is
// taken exactly -- two fp32 numbers multiply without error in fp64 -- and rounded once, to
// the nearest integer, ties to even; then saturated to [-qmax, qmax].
inline int32_t quantize(float v, float r, float qmax) {
  double q = nearbyint((double)v * (double)r);
  q = fmin(fmax(q, -(double)qmax), (double)qmax);
  return (int32_t)q;
}

}  // namespace

extern "C" {

// ---------------------------------------------------------------- O1 ------
// Direct 3x3 cross-correlation (no filter flip), fp64:
//   Y[n,k,h,w] = sum_c sum_{i,j<3} X[n,c,h*stride+i-pad, w*stride+j-pad] g[k,c,i,j]
// zero outside the image.  Ho = (H + 2 pad - 3)/stride + 1.
int oracle_conv2d_direct_f64(int N, int C, int K, int H, int W, int stride, int pad,
                             const double* X, const double* g, double* Y) {
  if (N < 1 || C < 1 || K < 1 || H < 1 || W < 1 || stride < 1 || pad < 0) return -1;
  const int Ho = (H + 2 * pad - 3) / stride + 1, Wo = (W + 2 * pad - 3) / stride + 1;
  if (Ho < 1 || Wo < 1) return -1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int k = 0; k < K; ++k)
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          double s = 0.0;
          for (int c = 0; c < C; ++c)
            for (int i = 0; i < 3; ++i)
              for (int j = 0; j < 3; ++j) {
                const int hi = h * stride + i - pad, wj = w * stride + j - pad;
                if (hi < 0 || hi >= H || wj < 0 || wj >= W) continue;
                s += X[(((size_t)n * C + c) * H + hi) * W + wj] *
                     g[(((size_t)k * C + c) * 3 + i) * 3 + j];
              }
          Y[(((size_t)n * K + k) * Ho + h) * Wo + w] = s;
        }
  return 0;
}

// Same definition on integers: int8-range activations and weights, exact
// accumulation, then one requantization  y = sat(rne( (float)acc * r_y )).
// The baseline (im2row) convolution of the quantized network, Sec. 5.3.
int oracle_conv2d_direct_q(int N, int C, int K, int H, int W, int stride, int pad,
                           const int32_t* Xq, const int32_t* gq, float r_y, int qmax,
                           int64_t* acc_out /* may be null */, int32_t* Yq) {
  if (N < 1 || C < 1 || K < 1 || H < 1 || W < 1 || stride < 1 || pad < 0) return -1;
  const int Ho = (H + 2 * pad - 3) / stride + 1, Wo = (W + 2 * pad - 3) / stride + 1;
  if (Ho < 1 || Wo < 1) return -1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int k = 0; k < K; ++k)
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          int64_t s = 0;
          for (int c = 0; c < C; ++c)
            for (int i = 0; i < 3; ++i)
              for (int j = 0; j < 3; ++j) {
                const int hi = h * stride + i - pad, wj = w * stride + j - pad;
                if (hi < 0 || hi >= H || wj < 0 || wj >= W) continue;
                s += (int64_t)Xq[(((size_t)n * C + c) * H + hi) * W + wj] *
                     (int64_t)gq[(((size_t)k * C + c) * 3 + i) * 3 + j];
              }
          const size_t o = (((size_t)n * K + k) * Ho + h) * Wo + w;
          if (acc_out) acc_out[o] = s;
          Yq[o] = quantize((float)s, r_y, (float)qmax);
        }
  return 0;
}

// ---------------------------------------------------------------- O2 ------
// Literal Winograd, fp64.  BT is n x n, G is n x 3, AT is m x n (row-major).
// For every tile and output channel:
//   Yt = A^T [ sum_c (G g_{k,c} G^T) (.) (B^T d_c B) ] A.
int oracle_winograd_f64(int N, int C, int K, int H, int W, int pad, int m,
                        const double* BT, const double* G, const double* AT,
                        const double* X, const double* g, double* Y) {
  if (N < 1 || C < 1 || K < 1 || H < 1 || W < 1 || pad < 0 || m < 1) return -1;
  const int n = m + 2, P = n * n;
  const int Ho = H + 2 * pad - 2, Wo = W + 2 * pad - 2;
  if (Ho < 1 || Wo < 1) return -1;
  const int TH = ceil_div(Ho, m), TW = ceil_div(Wo, m);

  // Winograd-domain filters U[k][c] = G g G^T  (n x n each).
  std::vector<double> U((size_t)K * C * P);
#pragma omp parallel for schedule(static)
  for (int kc = 0; kc < K * C; ++kc) {
    std::vector<double> Gg(n * 3);
    matmul(G, n, 3, g + (size_t)kc * 9, 3, Gg.data());        // G g      (n x 3)
    matmul_bt(Gg.data(), n, 3, G, n, U.data() + (size_t)kc * P);  // (G g) G^T (n x n)
  }

#pragma omp parallel for collapse(2) schedule(static)
  for (int img = 0; img < N; ++img)
    for (int th = 0; th < TH; ++th) {
      std::vector<double> V((size_t)C * P), d(P), Btd(P), acc(P), AtM(m * n), Yt(m * m);
      for (int tw = 0; tw < TW; ++tw) {
        // Winograd-domain patches V[c] = B^T d_c B.
        for (int c = 0; c < C; ++c) {
          for (int j = 0; j < n; ++j)
            for (int l = 0; l < n; ++l) {
              const int h = th * m - pad + j, w = tw * m - pad + l;
              d[j * n + l] = (h < 0 || h >= H || w < 0 || w >= W)
                                 ? 0.0
                                 : X[(((size_t)img * C + c) * H + h) * W + w];
            }
          matmul(BT, n, n, d.data(), n, Btd.data());                    // B^T d
          matmul_bt(Btd.data(), n, n, BT, n, V.data() + (size_t)c * P);  // (B^T d) B
        }
        for (int k = 0; k < K; ++k) {
          for (int p = 0; p < P; ++p) {
            double s = 0.0;
            for (int c = 0; c < C; ++c) s += U[((size_t)k * C + c) * P + p] * V[(size_t)c * P + p];
            acc[p] = s;
          }
          matmul(AT, m, n, acc.data(), n, AtM.data());       // A^T M     (m x n)
          matmul_bt(AtM.data(), m, n, AT, m, Yt.data());     // (A^T M) A (m x m)
          for (int a = 0; a < m; ++a)
            for (int b = 0; b < m; ++b) {
              const int h = th * m + a, w = tw * m + b;
              if (h < Ho && w < Wo) Y[(((size_t)img * K + k) * Ho + h) * Wo + w] = Yt[a * m + b];
            }
        }
      }
    }
  return 0;
}

// ---------------------------------------------------------------- O3 ------
// Host scalars of the quantized pipeline, all in fp32.  s_x, s_v, s_u, s_y are
// the scales of the input, the transformed input, the transformed weights and
// the output; s_m > 0 switches on the quantizer after the Hadamard stage.
//   r_u = 1/s_u            U  -> Uq
//   r_v = s_x/s_v          B^T x_q B -> Vq   (x_q carries the factor 1/s_x)
//   r_m = (s_u s_v)/s_m    M  -> Mq          (only if s_m > 0)
//   r_y = (s_u s_v)/s_y    A^T M A -> y_q    (s_m/s_y if the M quantizer is on)
void oracle_q_scalars(float s_x, float s_v, float s_u, float s_y, float s_m,
                      float* r_u, float* r_v, float* r_m, float* r_y) {
  *r_u = 1.0f / s_u;
  *r_v = s_x / s_v;
  const float suv = s_u * s_v;
  if (s_m > 0.0f) {
    *r_m = suv / s_m;
    *r_y = s_m / s_y;
  } else {
    *r_m = 0.0f;
    *r_y = suv / s_y;
  }
}

// Weight stage:  t = G g (n x 3), U = t G^T (n x n), Uq = sat(rne(U * r_u)).
// U_f32 (optional) receives the unscaled fp32 U, Uq (optional) the integers;
// both in the order [p][k][c].
// Per-position variant (Sec. 7 names other kinds of quantization as the way to recover
// F4/F6 accuracy; one scale per Winograd position is the smallest step from the paper's
// one scale per tensor): r_u_pos[p] multiplies position p = i*n + j.  The per-tensor entry
// point below is this one with all factors equal.
int oracle_q_weights_pos(int K, int C, int m, const float* G, const float* g,
                         const float* r_u_pos, int qmax, float* U_f32, int32_t* Uq) {
  if (K < 1 || C < 1 || m < 1 || m > 6 || !r_u_pos) return -1;
  const int n = m + 2;
#pragma omp parallel for schedule(static)
  for (int k = 0; k < K; ++k)
    for (int c = 0; c < C; ++c) {
      const float* gk = g + ((size_t)k * C + c) * 9;
      float t[8][3];
      for (int i = 0; i < n; ++i)
        for (int b = 0; b < 3; ++b) {
          float acc = 0.0f;
          for (int a = 0; a < 3; ++a) acc = fmaf(G[i * 3 + a], gk[a * 3 + b], acc);
          t[i][b] = acc;
        }
      for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
          float acc = 0.0f;
          for (int b = 0; b < 3; ++b) acc = fmaf(t[i][b], G[j * 3 + b], acc);
          const size_t o = ((size_t)(i * n + j) * K + k) * C + c;
          if (U_f32) U_f32[o] = acc;
          if (Uq) Uq[o] = quantize(acc, r_u_pos[i * n + j], (float)qmax);
        }
    }
  return 0;
}

int oracle_q_weights(int K, int C, int m, const float* G, const float* g, float r_u, int qmax,
                     float* U_f32, int32_t* Uq) {
  float r[64];
  for (int p = 0; p < 64; ++p) r[p] = r_u;
  return oracle_q_weights_pos(K, C, m, G, g, r, qmax, U_f32, Uq);
}

// Input stage:  d = patch of x_q as floats (+0 outside the image),
//   w = B^T d (n x n), V = w B (n x n), Vq = sat(rne(V * r_v)).
// V_f32 / Vq in the order [p][t][c].
// r_v_pos[p]: one factor per Winograd position p = i*n + k (see oracle_q_weights_pos).
int oracle_q_input_pos(int N, int C, int H, int W, int pad, int m, const float* BT,
                       const int32_t* xq, const float* r_v_pos, int qmax, float* V_f32,
                       int32_t* Vq) {
  if (N < 1 || C < 1 || H < 1 || W < 1 || pad < 0 || m < 1 || m > 6 || !r_v_pos) return -1;
  const int n = m + 2;
  const int Ho = H + 2 * pad - 2, Wo = W + 2 * pad - 2;
  if (Ho < 1 || Wo < 1) return -1;
  const int TH = ceil_div(Ho, m), TW = ceil_div(Wo, m);
  const size_t T = (size_t)N * TH * TW;
#pragma omp parallel for collapse(2) schedule(static)
  for (int img = 0; img < N; ++img)
    for (int th = 0; th < TH; ++th)
      for (int tw = 0; tw < TW; ++tw) {
        const size_t t = ((size_t)img * TH + th) * TW + tw;
        for (int c = 0; c < C; ++c) {
          float d[8][8], w[8][8];
          for (int j = 0; j < n; ++j)
            for (int l = 0; l < n; ++l) {
              const int h = th * m - pad + j, x = tw * m - pad + l;
              d[j][l] = (h < 0 || h >= H || x < 0 || x >= W)
                            ? 0.0f
                            : (float)xq[(((size_t)img * C + c) * H + h) * W + x];
            }
          for (int i = 0; i < n; ++i)
            for (int l = 0; l < n; ++l) {
              float acc = 0.0f;
              for (int j = 0; j < n; ++j) acc = fmaf(BT[i * n + j], d[j][l], acc);
              w[i][l] = acc;
            }
          for (int i = 0; i < n; ++i)
            for (int k = 0; k < n; ++k) {
              float acc = 0.0f;
              for (int l = 0; l < n; ++l) acc = fmaf(w[i][l], BT[k * n + l], acc);
              const size_t o = ((size_t)(i * n + k) * T + t) * C + c;
              if (V_f32) V_f32[o] = acc;
              if (Vq) Vq[o] = quantize(acc, r_v_pos[i * n + k], (float)qmax);
            }
        }
      }
  return 0;
}

int oracle_q_input(int N, int C, int H, int W, int pad, int m, const float* BT,
                   const int32_t* xq, float r_v, int qmax, float* V_f32, int32_t* Vq) {
  float r[64];
  for (int p = 0; p < 64; ++p) r[p] = r_v;
  return oracle_q_input_pos(N, C, H, W, pad, m, BT, xq, r, qmax, V_f32, Vq);
}

// Hadamard stage written as one GEMM per Winograd position (exact integers):
//   M[p][t][k] = sum_c Vq[p][t][c] * Uq[p][k][c].
int oracle_q_hadamard(int P, int64_t T, int C, int K, const int32_t* Vq, const int32_t* Uq,
                      int64_t* M) {
  if (P < 1 || T < 1 || C < 1 || K < 1) return -1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int p = 0; p < P; ++p)
    for (int64_t t = 0; t < T; ++t)
      for (int k = 0; k < K; ++k) {
        int64_t s = 0;
        const int32_t* v = Vq + ((size_t)p * T + t) * C;
        const int32_t* u = Uq + ((size_t)p * K + k) * C;
        for (int c = 0; c < C; ++c) s += (int64_t)v[c] * (int64_t)u[c];
        M[((size_t)p * T + t) * K + k] = s;
      }
  return 0;
}

// Output stage.  Optional quantizer on M first (r_m > 0):  M <- sat(rne((float)M * r_m)).
// Then  z = A^T M (m x n), Yt = z A (m x m), y_q = sat(rne(Yt * r_y)), cropped.
// Y_f32 (optional) receives Yt before the multiplication by r_y.
// Returns the number of accumulators with |M| >= 2^24 (whose float conversion
// is not exact); 0 in every int8 workload (127^2 * 512 < 2^23).
// w_pos (optional): with per-position scales the accumulators of different positions are
// in different units, so each is first brought to real units, Mf = (float)M * w_pos[p]
// (w_pos[p] = s_u[p] * s_v[p]); r_m and r_y then no longer contain s_u * s_v.
// qmax_m / qmax_y: the two quantizers of this stage may have different bit-widths
// (Sec. 3.2, "quantization diversity": every intermediate of Eq. 1 can be quantized to its
// own number of bits; Sec. 5.1 runs INT8, INT10 and INT16): the Hadamard-stage codes
// saturate to [-qmax_m, qmax_m], the output codes to [-qmax_y, qmax_y].  The weight and
// input stages take their own qmax as an argument already.  (float)M is the conversion of
// the exact integer, rounded half to even when |M| >= 2^24.
int64_t oracle_q_output_bits(int N, int K, int H, int W, int pad, int m, const float* AT,
                             const int64_t* M, const float* w_pos, float r_m, float r_y,
                             int qmax_m, int qmax_y, float* Y_f32, int32_t* Yq) {
  if (N < 1 || K < 1 || H < 1 || W < 1 || pad < 0 || m < 1 || m > 6) return -1;
  const int n = m + 2;
  const int Ho = H + 2 * pad - 2, Wo = W + 2 * pad - 2;
  if (Ho < 1 || Wo < 1) return -1;
  const int TH = ceil_div(Ho, m), TW = ceil_div(Wo, m);
  const size_t T = (size_t)N * TH * TW;
  int64_t inexact = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(+ : inexact)
  for (int img = 0; img < N; ++img)
    for (int th = 0; th < TH; ++th)
      for (int tw = 0; tw < TW; ++tw) {
        const size_t t = ((size_t)img * TH + th) * TW + tw;
        for (int k = 0; k < K; ++k) {
          float Mf[8][8], z[8][8];
          for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
              const int64_t v = M[((size_t)(i * n + j) * T + t) * K + k];
              if (v >= (1 << 24) || v <= -(1 << 24)) ++inexact;
              float f = (float)v;
              if (w_pos) f = f * w_pos[i * n + j];
              if (r_m > 0.0f) f = (float)quantize(f, r_m, (float)qmax_m);
              Mf[i][j] = f;
            }
          for (int a = 0; a < m; ++a)
            for (int j = 0; j < n; ++j) {
              float acc = 0.0f;
              for (int i = 0; i < n; ++i) acc = fmaf(AT[a * n + i], Mf[i][j], acc);
              z[a][j] = acc;
            }
          for (int a = 0; a < m; ++a)
            for (int b = 0; b < m; ++b) {
              float acc = 0.0f;
              for (int j = 0; j < n; ++j) acc = fmaf(z[a][j], AT[b * n + j], acc);
              const int h = th * m + a, x = tw * m + b;
              if (h < Ho && x < Wo) {
                const size_t o = (((size_t)img * K + k) * Ho + h) * Wo + x;
                if (Y_f32) Y_f32[o] = acc;
                if (Yq) Yq[o] = quantize(acc, r_y, (float)qmax_y);
              }
            }
        }
      }
  return inexact;
}

int64_t oracle_q_output_pos(int N, int K, int H, int W, int pad, int m, const float* AT,
                            const int64_t* M, const float* w_pos, float r_m, float r_y, int qmax,
                            float* Y_f32, int32_t* Yq) {
  return oracle_q_output_bits(N, K, H, W, pad, m, AT, M, w_pos, r_m, r_y, qmax, qmax, Y_f32, Yq);
}

int64_t oracle_q_output(int N, int K, int H, int W, int pad, int m, const float* AT,
                        const int64_t* M, float r_m, float r_y, int qmax, float* Y_f32,
                        int32_t* Yq) {
  return oracle_q_output_pos(N, K, H, W, pad, m, AT, M, nullptr, r_m, r_y, qmax, Y_f32, Yq);
}

// Host scalars of the per-position variant, each one fp32 operation:
//   r_u[p] = 1 / s_u[p];  r_v[p] = s_x / s_v[p];  w[p] = s_u[p] * s_v[p];
//   s_m > 0:  r_m = 1 / s_m, r_y = s_m / s_y;   else  r_m = 0, r_y = 1 / s_y.
void oracle_q_scalars_pos(int P, float s_x, const float* s_v_pos, const float* s_u_pos, float s_y,
                          float s_m, float* r_u_pos, float* r_v_pos, float* w_pos, float* r_m,
                          float* r_y) {
  for (int p = 0; p < P; ++p) {
    r_u_pos[p] = 1.0f / s_u_pos[p];
    r_v_pos[p] = s_x / s_v_pos[p];
    w_pos[p] = s_u_pos[p] * s_v_pos[p];
  }
  if (s_m > 0.0f) {
    *r_m = 1.0f / s_m;
    *r_y = s_m / s_y;
  } else {
    *r_m = 0.0f;
    *r_y = 1.0f / s_y;
  }
}

// Number of OpenMP threads the loops above will use (for reporting).
int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_num_threads(int nt) {
#ifdef _OPENMP
  if (nt > 0) omp_set_num_threads(nt);
#else
  (void)nt;
#endif
}

}  // extern "C"
