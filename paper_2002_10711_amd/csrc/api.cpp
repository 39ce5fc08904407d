// Host side of libwino: argument validation, geometry, scalar derivation and
// kernel sequencing for the entry points declared in wino.h.  No device memory is
// allocated here and nothing synchronises.
#include <math.h>
#include <string.h>

#include "wino_internal.h"

using namespace wino;

namespace {

bool finite_all(const float* p, int n) {
  for (int i = 0; i < n; ++i)
    if (!isfinite(p[i])) return false;
  return true;
}

// Validates the descriptor and fills the derived geometry.
wino_status make_geom(const wino_desc* d, Geom* g) {
  if (!d) return WINO_E_NULL;
  if (d->m != 2 && d->m != 4 && d->m != 6) return WINO_E_BAD_M;
  if (d->dtype != WINO_F32 && d->dtype != WINO_I8 && d->dtype != WINO_I16 &&
      d->dtype != WINO_I8W16 && d->dtype != WINO_BF16)
    return WINO_E_BAD_DTYPE;
  if (d->dtype == WINO_BF16 && d->m == 6) return WINO_E_BAD_M;
  if (d->N < 1 || d->C < 1 || d->K < 1 || d->H < 1 || d->W < 1) return WINO_E_BAD_SHAPE;
  if (d->pad != 0 && d->pad != 1) return WINO_E_BAD_SHAPE;
  g->N = d->N; g->C = d->C; g->K = d->K; g->H = d->H; g->W = d->W;
  g->pad = d->pad; g->m = d->m; g->n = d->m + 2; g->P = g->n * g->n;
  g->Ho = d->H + 2 * d->pad - 2;
  g->Wo = d->W + 2 * d->pad - 2;
  if (g->Ho < 1 || g->Wo < 1) return WINO_E_BAD_SHAPE;
  g->TH = (g->Ho + d->m - 1) / d->m;
  g->TW = (g->Wo + d->m - 1) / d->m;
  g->i8 = d->dtype == WINO_I8;
  g->w16 = d->dtype == WINO_I16 || d->dtype == WINO_I8W16;
  g->x16 = d->dtype == WINO_I16;
  g->bf16 = d->dtype == WINO_BF16;
  // (wide modes: the int32 sums of digit products and their recombination are sized for
  // reductions of at most 1024 channels)
  if (g->w16 && d->C > 1024) return WINO_E_BAD_SHAPE;
  const long long T = (long long)d->N * g->TH * g->TW;
  const long long limit = 0x7fffffffLL;
  if (T > limit - 64) return WINO_E_BAD_SHAPE;
  g->T = (int)T;
  g->Tp = round_up(g->T, 64);
  g->Cp = round_up(d->C, (g->i8 || g->w16) ? 64 : 16);
  g->Kp = round_up(d->K, 64);
  // every tensor must be indexable with 31-bit element offsets
  const long long e = g->i8 ? 1 : 4;
  // (wide modes: two digit planes per element of U and V)
  if (g->w16 && ((long long)g->P * g->Tp * g->Cp * 2 > limit ||
                 (long long)g->P * g->Kp * g->Cp * 2 > limit))
    return WINO_E_BAD_SHAPE;
  if ((long long)g->P * g->Tp * g->Cp > limit || (long long)g->P * g->Tp * g->Kp > limit ||
      (long long)g->P * g->Kp * g->Cp > limit ||
      (long long)d->N * d->C * d->H * d->W * e > limit * e ||
      (long long)d->N * d->K * g->Ho * g->Wo > limit)
    return WINO_E_BAD_SHAPE;
  if (g->bf16 && !fused_fwd_bf16_supported(*g)) return WINO_E_BAD_SHAPE;
  return WINO_OK;
}

size_t align256(size_t b) { return (b + 255) / 256 * 256; }
// (wide modes: two int8 digit planes per element of U and V, int64 M)
size_t elem_bytes(const Geom& g) { return g.i8 ? 1 : g.w16 ? 2 : 4; }
size_t v_bytes(const Geom& g) { return align256((size_t)g.P * g.Tp * g.Cp * elem_bytes(g)); }
size_t m_bytes(const Geom& g) { return align256((size_t)g.P * g.Tp * g.Kp * (g.w16 ? 8 : 4)); }
size_t u_bytes(const Geom& g) { return align256((size_t)g.P * g.Kp * g.Cp * elem_bytes(g)); }

// Code range of one stage: its own field, else the common qmax.
int stage_qmax(int own, int common) { return own ? own : common; }

wino_status check_quant(const Geom& g, const wino_quant* q) {
  if (!g.i8 && !g.w16) return WINO_OK;
  if (!q) return WINO_E_BAD_SCALE;
  if ((q->s_v_pos != nullptr) != (q->s_u_pos != nullptr)) return WINO_E_BAD_SCALE;
  if (q->s_v_pos) {
    // per-position scales replace s_v and s_u
    if (!isfinite(q->s_x) || !(q->s_x > 0.0f) || !isfinite(q->s_y) || !(q->s_y > 0.0f))
      return WINO_E_BAD_SCALE;
    for (int p = 0; p < g.P; ++p)
      if (!isfinite(q->s_v_pos[p]) || !(q->s_v_pos[p] > 0.0f) || !isfinite(q->s_u_pos[p]) ||
          !(q->s_u_pos[p] > 0.0f))
        return WINO_E_BAD_SCALE;
  } else {
    const float s[4] = {q->s_x, q->s_v, q->s_u, q->s_y};
    for (float v : s)
      if (!isfinite(v) || !(v > 0.0f)) return WINO_E_BAD_SCALE;
  }
  if (!isfinite(q->s_m) || q->s_m < 0.0f) return WINO_E_BAD_SCALE;
  const int wide = g.w16 ? 32767 : 127;
  if (q->qmax < 1 || q->qmax > wide) return WINO_E_BAD_SCALE;
  const int qu = stage_qmax(q->qmax_u, q->qmax), qv = stage_qmax(q->qmax_v, q->qmax),
            qm = stage_qmax(q->qmax_m, q->qmax), qy = stage_qmax(q->qmax_y, q->qmax);
  if (qu < 1 || qu > wide || qv < 1 || qv > wide || qm < 1 || qm > wide || qy < 1 ||
      qy > (g.x16 ? 32767 : 127))
    return WINO_E_BAD_SCALE;
  // the int8 kernels share one range between their stages
  if (g.i8 && (qu != q->qmax || qv != q->qmax || qm != q->qmax || qy != q->qmax))
    return WINO_E_BAD_SCALE;
  return WINO_OK;
}

// fp32 multipliers of the quantized pipeline, derived on the host:
//   r_u = 1/s_u, r_v = s_x/s_v, r_m = (s_u s_v)/s_m, r_y = (s_u s_v)/s_y  (s_m/s_y if the
//   quantizer after the Hadamard stage is on).
// With per-position scales (pos): r_u[p] = 1/s_u[p], r_v[p] = s_x/s_v[p],
//   w[p] = s_u[p] s_v[p] (applied to the accumulators), r_m = 1/s_m, r_y = 1/s_y (s_m/s_y).
struct Scalars {
  float r_u, r_v, r_m, r_y, qmax;
  float qmax_u, qmax_v, qmax_m, qmax_y;   // per stage (all equal to qmax in the int8 mode)
  bool pos;
  PosScale ru_pos, rv_pos, w_pos;
};
Scalars make_scalars(const Geom& g, const wino_quant* q) {
  Scalars s;
  memset(&s, 0, sizeof s);
  s.r_u = s.r_v = s.r_y = 1.0f;
  s.qmax = 127.0f;
  if (!g.i8 && !g.w16) return s;
  s.qmax_u = (float)stage_qmax(q->qmax_u, q->qmax);
  s.qmax_v = (float)stage_qmax(q->qmax_v, q->qmax);
  s.qmax_m = (float)stage_qmax(q->qmax_m, q->qmax);
  s.qmax_y = (float)stage_qmax(q->qmax_y, q->qmax);
  if (q->s_v_pos) {
    s.pos = true;
    s.qmax = (float)q->qmax;
    for (int p = 0; p < g.P; ++p) {
      volatile float w = q->s_u_pos[p] * q->s_v_pos[p];   // one rounded fp32 product
      s.ru_pos.r[p] = 1.0f / q->s_u_pos[p];
      s.rv_pos.r[p] = q->s_x / q->s_v_pos[p];
      s.w_pos.r[p] = w;
    }
    if (q->s_m > 0.0f) {
      s.r_m = 1.0f / q->s_m;
      s.r_y = q->s_m / q->s_y;
    } else {
      s.r_y = 1.0f / q->s_y;
    }
    s.r_u = s.ru_pos.r[0];
    s.r_v = s.rv_pos.r[0];
    return s;
  }
  volatile float suv = q->s_u * q->s_v;  // one rounded fp32 product, never contracted
  s.r_u = 1.0f / q->s_u;
  s.r_v = q->s_x / q->s_v;
  if (q->s_m > 0.0f) {
    s.r_m = suv / q->s_m;
    s.r_y = q->s_m / q->s_y;
  } else {
    s.r_y = suv / q->s_y;
  }
  s.qmax = (float)q->qmax;
  // (the wide kernels always take one factor per position)
  for (int p = 0; p < 64; ++p) {
    s.ru_pos.r[p] = s.r_u;
    s.rv_pos.r[p] = s.r_v;
  }
  return s;
}

bool aligned256(const void* p) { return ((uintptr_t)p & 255) == 0; }

}  // namespace

extern "C" {

const char* wino_status_string(wino_status s) {
  switch (s) {
    case WINO_OK: return "ok";
    case WINO_E_NULL: return "null pointer";
    case WINO_E_BAD_M: return "m must be 2, 4 or 6";
    case WINO_E_BAD_SHAPE: return "bad shape";
    case WINO_E_BAD_DTYPE: return "bad dtype";
    case WINO_E_BAD_SCALE: return "bad quantizer scale, qmax or matrix entry";
    case WINO_E_WORKSPACE: return "workspace too small or misaligned";
    case WINO_E_HIP: return "HIP error";
    case WINO_E_BAD_ARG: return "bad argument";
    case WINO_E_SCRATCH_LIMIT: return "problem needs more scratch than the built-in buffer holds";
  }
  return "unknown status";
}

size_t wino_weights_bytes(const wino_desc* d) {
  Geom g;
  if (make_geom(d, &g) != WINO_OK) return 0;
  return u_bytes(g);
}

size_t wino_workspace_bytes(const wino_desc* d) {
  Geom g;
  if (make_geom(d, &g) != WINO_OK) return 0;
  return v_bytes(g) + m_bytes(g);
}

wino_status wino_transform_weights(const wino_desc* d, const wino_quant* q, const float* g_dev,
                                   void* U_dev, void* stream) {
  Geom g;
  wino_status st = make_geom(d, &g);
  if (st != WINO_OK) return st;
  if (!d->G || !g_dev || !U_dev) return WINO_E_NULL;
  if (!finite_all(d->G, g.n * 3)) return WINO_E_BAD_SCALE;
  if ((st = check_quant(g, q)) != WINO_OK) return st;
  if (!aligned256(U_dev)) return WINO_E_WORKSPACE;
  MatG mg;
  memset(&mg, 0, sizeof mg);
  memcpy(mg.v, d->G, sizeof(float) * g.n * 3);
  const Scalars s = make_scalars(g, q);
  if (g.w16)
    return launch_w16_weights(g, mg, g_dev, U_dev, s.ru_pos, s.qmax_u, (hipStream_t)stream) ==
                   hipSuccess
               ? WINO_OK
               : WINO_E_HIP;
  if (launch_weight_transform(g, mg, g_dev, U_dev, s.r_u, s.qmax, (hipStream_t)stream,
                              s.pos ? &s.ru_pos : nullptr) != hipSuccess)
    return WINO_E_HIP;
  return WINO_OK;
}

int wino_fwd_num_kernels(const wino_desc* d) {
  Geom g;
  if (make_geom(d, &g) != WINO_OK) return 0;
  if (g.w16) {
    MatAT at;
    memset(&at, 0, sizeof at);
    if (d->AT && finite_all(d->AT, g.m * g.n)) {
      memcpy(at.v, d->AT, sizeof(float) * g.m * g.n);
      if (w16_gemm_out_supported(g, at)) return 2;
    }
    return 3;
  }
  if (g.bf16 || fused_fwd_f32_supported(g)) return 1;
  if (g.i8) {
    // as in wino_conv2d_fwd: the sequence the table of measured times names
    MatBT bt;
    const bool have_bt = d->BT && finite_all(d->BT, g.n * g.n);
    if (have_bt) {
      memset(&bt, 0, sizeof bt);
      memcpy(bt.v, d->BT, sizeof(float) * g.n * g.n);
    }
    const int seq = fwd_sequence_auto(g, have_bt ? &bt : nullptr, true);
    return seq == kSeqFused ? 1 : seq == kSeqStaged ? 3 : 2;
  }
  // fp32: GEMM + output transform in one kernel while the reduction is short
  return gemm_out_f32_preferred(g) ? 2 : 3;
}

}  // extern "C"

namespace wino {

// Bytes of workspace the kernel sequence of this problem really touches: nothing for the
// one-kernel forward, V for two kernels, V and M for three.
size_t fwd_workspace_touched(const wino_desc* d) {
  Geom g;
  if (make_geom(d, &g) != WINO_OK) return 0;
  const int nk = wino_fwd_num_kernels(d);
  return nk <= 1 ? 0 : nk == 2 ? v_bytes(g) : v_bytes(g) + m_bytes(g);
}

// The forward behind wino_conv2d_fwd_stages.  exact_need: the workspace only has to hold
// what the kernel sequence touches (fwd_workspace_touched) instead of V and M.
// Every argument check of the forward that needs no workspace: descriptor, pointers of the
// selected stages, matrices, quantizer.  Fills the geometry.
wino_status fwd_check(const wino_desc* d, const wino_quant* q, const void* x_dev,
                      const void* U_dev, const void* y_dev, int stages, Geom* gp) {
  Geom& g = *gp;
  wino_status st = make_geom(d, &g);
  if (st != WINO_OK) return st;
  if (stages < 1 || stages > WINO_STAGE_ALL) return WINO_E_BAD_ARG;
  const bool s_in = stages & WINO_STAGE_INPUT, s_mm = stages & WINO_STAGE_GEMM,
             s_out = stages & WINO_STAGE_OUTPUT;
  if ((s_in && (!d->BT || !x_dev)) || (s_mm && !U_dev) || (s_out && (!d->AT || !y_dev)))
    return WINO_E_NULL;
  if ((s_in && !finite_all(d->BT, g.n * g.n)) || (s_out && !finite_all(d->AT, g.m * g.n)))
    return WINO_E_BAD_SCALE;
  if ((st = check_quant(g, q)) != WINO_OK) return st;
  if (g.w16 && g.x16 && ((s_in && ((uintptr_t)x_dev & 1)) || (s_out && ((uintptr_t)y_dev & 1))))
    return WINO_E_BAD_ARG;
  return WINO_OK;
}

wino_status fwd_stages(const wino_desc* d, const wino_quant* q, const void* x_dev,
                       const void* U_dev, void* y_dev, void* workspace_dev,
                       size_t workspace_bytes, int stages, void* stream, bool exact_need,
                       int forced_seq) {
  Geom g;
  if (!workspace_dev && d && make_geom(d, &g) == WINO_OK && stages >= 1 &&
      stages <= WINO_STAGE_ALL)
    return WINO_E_NULL;
  wino_status st = fwd_check(d, q, x_dev, U_dev, y_dev, stages, &g);
  if (st != WINO_OK) return st;
  const bool s_in = stages & WINO_STAGE_INPUT, s_mm = stages & WINO_STAGE_GEMM,
             s_out = stages & WINO_STAGE_OUTPUT;
  if (workspace_bytes < (exact_need && stages == WINO_STAGE_ALL && d->BT && d->AT
                             ? fwd_workspace_touched(d)
                             : v_bytes(g) + m_bytes(g)) ||
      !aligned256(workspace_dev) || (s_mm && !aligned256(U_dev)))
    return WINO_E_WORKSPACE;
  const Scalars s = make_scalars(g, q);
  hipStream_t hs = (hipStream_t)stream;
  void* V = workspace_dev;
  void* M = (char*)workspace_dev + v_bytes(g);
  MatBT bt;
  MatAT at;
  if (s_in) {
    memset(&bt, 0, sizeof bt);
    memcpy(bt.v, d->BT, sizeof(float) * g.n * g.n);
  }
  if (s_out) {
    memset(&at, 0, sizeof at);
    memcpy(at.v, d->AT, sizeof(float) * g.m * g.n);
  }
  if (g.w16) {
    if (s_in && launch_w16_input(g, bt, x_dev, V, s.rv_pos, s.qmax_v, hs) != hipSuccess)
      return WINO_E_HIP;
    const PosScale* wpw = s.pos ? &s.w_pos : nullptr;
    if (s_mm && s_out && w16_gemm_out_supported(g, at))
      return launch_w16_gemm_out(g, at, V, U_dev, y_dev, wpw, s.r_m, s.r_y, s.qmax_m, s.qmax_y,
                                 hs) == hipSuccess
                 ? WINO_OK
                 : WINO_E_HIP;
    if (s_mm && launch_w16_gemm(g, V, U_dev, M, hs) != hipSuccess) return WINO_E_HIP;
    if (s_out && launch_w16_output(g, at, M, y_dev, s.pos ? &s.w_pos : nullptr, s.r_m, s.r_y,
                                   s.qmax_m, s.qmax_y, hs) != hipSuccess)
      return WINO_E_HIP;
    return WINO_OK;
  }
  // int8: which kernel sequence (measured table, or the caller's choice)
  int seq = kSeqStaged;
  if (g.i8) {
    const MatBT* btp = s_in ? &bt : nullptr;
    if (forced_seq != kSeqAuto) {
      if (stages != WINO_STAGE_ALL || !fwd_sequence_supported(g, btp, forced_seq))
        return WINO_E_BAD_ARG;
      seq = forced_seq;
    } else {
      seq = fwd_sequence_auto(g, btp, stages == WINO_STAGE_ALL);
    }
  }
  bool exact_refused = false;
  if (stages == WINO_STAGE_ALL && seq == kSeqFused) {
    // the whole forward in one kernel: V and M stay on chip, the workspace is untouched
    const bool exact = fused_fwd_exact_supported(g, bt);
    {
      const PosScale* rvq = s.pos ? &s.rv_pos : nullptr;
      const PosScale* wq = s.pos ? &s.w_pos : nullptr;
      hipError_t e =
          exact ? launch_fused_fwd_exact(g, bt, at, x_dev, U_dev, y_dev, s.r_v, s.r_m, s.r_y, s.qmax,
                                         rvq, wq, hs)
                : launch_fused_fwd(g, bt, at, x_dev, U_dev, y_dev, s.r_v, s.r_m, s.r_y, s.qmax, rvq,
                                   wq, hs);
      // The matrix-core launcher refuses, before launching anything, the few inputs its
      // exact scaling cannot carry (a quantizer factor that underflows when divided by
      // 4^s, a tile row count beyond the grid limit): those take the vector-ALU kernels,
      // which handle them -- as one kernel where that is supported, else stage by stage
      // (which needs the workspace after all).
      if (exact && e == hipErrorInvalidValue) {
        if (fused_fwd_generic_preferred(g))
          e = launch_fused_fwd(g, bt, at, x_dev, U_dev, y_dev, s.r_v, s.r_m, s.r_y, s.qmax, rvq, wq,
                               hs);
        else if (workspace_bytes < v_bytes(g) + m_bytes(g))
          return WINO_E_WORKSPACE;
        else
          exact_refused = true;
      }
      if (!exact_refused) return e == hipSuccess ? WINO_OK : WINO_E_HIP;
      seq = fwd_sequence_auto(g, &bt, false);
    }
  }
  if (g.bf16) {
    // bf16 GEMM operands: the one-kernel forward only (make_geom has checked the shape)
    if (stages != WINO_STAGE_ALL) return WINO_E_BAD_ARG;
    return launch_fused_fwd_bf16(g, bt, at, x_dev, U_dev, y_dev, hs) == hipSuccess ? WINO_OK
                                                                                   : WINO_E_HIP;
  }
  if (stages == WINO_STAGE_ALL && fused_fwd_f32_supported(g))
    return launch_fused_fwd_f32(g, bt, at, x_dev, U_dev, y_dev, hs) == hipSuccess ? WINO_OK
                                                                                  : WINO_E_HIP;
  const PosScale* rvp = s.pos ? &s.rv_pos : nullptr;
  const PosScale* wp = s.pos ? &s.w_pos : nullptr;
  if (s_in) {
    hipError_t e = input_exact_preferred(g, bt, x_dev)
                       ? launch_input_exact(g, bt, x_dev, V, s.r_v, s.qmax, hs, rvp)
                   : input_f32_staged_supported(g)
                       ? launch_input_f32_staged(g, bt, x_dev, V, hs)
                       : launch_input_transform(g, bt, x_dev, V, s.r_v, s.qmax, hs, rvp);
    // (the matrix-core input stage refuses what its exact scaling cannot carry, see above)
    if (e == hipErrorInvalidValue && input_exact_preferred(g, bt, x_dev))
      e = launch_input_transform(g, bt, x_dev, V, s.r_v, s.qmax, hs, rvp);
    if (e != hipSuccess) return WINO_E_HIP;
  }
  // (with per-position scales every accumulator is multiplied by its position's factor
  // before the output transform: the GEMM + output kernels for long reductions and the
  // stand-alone output kernel do that, gemm_out_kernel does not)
  // (gemm_out_kernel knows no per-position factors: such calls take the column-wise kernel)
  if (g.i8 && seq == kSeqRegs && s.pos) seq = gemm_out_col_supported(g) ? kSeqCol : kSeqStaged;
  if (!g.i8) seq = gemm_out_f32_preferred(g) ? kSeqRegs : kSeqStaged;
  // (the row-of-tiles kernel stores 16-byte pieces: other alignments of y take the
  // column-wise kernel, which supports every shape that one does)
  if (g.i8 && seq == kSeqTrow && ((uintptr_t)y_dev & 15) != 0) seq = kSeqCol;
  if (s_mm && s_out && seq == kSeqTrow) {
    // F(6x6,3x3), short reductions: the same fusion on whole rows of tiles
    if (launch_gemm_out_trow(g, at, V, U_dev, y_dev, wp, s.r_m, s.r_y, s.qmax, hs) != hipSuccess)
      return WINO_E_HIP;
  } else if (s_mm && s_out && seq == kSeqLds) {
    // F(2x2,3x3), 512 channels, many tiles: the same fusion with squarer workgroup tiles
    if (launch_gemm_out_lds(g, at, V, U_dev, y_dev, wp, s.r_m, s.r_y, s.qmax, hs) != hipSuccess)
      return WINO_E_HIP;
  } else if (s_mm && s_out && (seq == kSeqCol || seq == kSeqCol2)) {
    // GEMM and output transform in one kernel for any reduction length (and with
    // per-position scales): M stays in registers
    if (launch_gemm_out_col(g, at, V, U_dev, y_dev, wp, s.r_m, s.r_y, s.qmax, hs,
                            seq == kSeqCol2) != hipSuccess)
      return WINO_E_HIP;
  } else if (s_mm && s_out && seq == kSeqRegs) {
    // short reductions: GEMM and output transform in one kernel, M stays in registers
    if (launch_gemm_out(g, at, V, U_dev, y_dev, s.r_m, s.r_y, s.qmax, hs) != hipSuccess)
      return WINO_E_HIP;
  } else if (s_mm && s_out) {
    if (launch_gemm(g.P, g.Tp, g.Kp, g.Cp, g.i8, 1, V, U_dev, M, hs) != hipSuccess) return WINO_E_HIP;
    if (launch_output_transform(g, at, M, y_dev, s.r_m, s.r_y, s.qmax, hs, wp) != hipSuccess)
      return WINO_E_HIP;
  } else if (s_mm) {
    if (launch_gemm(g.P, g.Tp, g.Kp, g.Cp, g.i8, 1, V, U_dev, M, hs) != hipSuccess) return WINO_E_HIP;
  } else if (s_out) {
    if (launch_output_transform(g, at, M, y_dev, s.r_m, s.r_y, s.qmax, hs, wp) != hipSuccess)
      return WINO_E_HIP;
  }
  return WINO_OK;
}

}  // namespace wino

extern "C" {

wino_status wino_conv2d_fwd_stages(const wino_desc* d, const wino_quant* q, const void* x_dev,
                                   const void* U_dev, void* y_dev, void* workspace_dev,
                                   size_t workspace_bytes, int stages, void* stream) {
  return fwd_stages(d, q, x_dev, U_dev, y_dev, workspace_dev, workspace_bytes, stages, stream,
                    false, kSeqAuto);
}

wino_status wino_conv2d_fwd_seq(const wino_desc* d, const wino_quant* q, const void* x_dev,
                                const void* U_dev, void* y_dev, void* workspace_dev,
                                size_t workspace_bytes, int seq, void* stream) {
  if (seq < kSeqAuto || seq >= kSeqCount) return WINO_E_BAD_ARG;
  return fwd_stages(d, q, x_dev, U_dev, y_dev, workspace_dev, workspace_bytes, WINO_STAGE_ALL,
                    stream, false, seq);
}

int wino_fwd_sequence(const wino_desc* d, int seq) {
  Geom g;
  if (make_geom(d, &g) != WINO_OK || !g.i8 || seq < kSeqAuto || seq >= kSeqCount) return 0;
  MatBT bt;
  const bool have_bt = d->BT && finite_all(d->BT, g.n * g.n);
  if (have_bt) {
    memset(&bt, 0, sizeof bt);
    memcpy(bt.v, d->BT, sizeof(float) * g.n * g.n);
  }
  if (seq == kSeqAuto) return fwd_sequence_auto(g, have_bt ? &bt : nullptr, true);
  return fwd_sequence_supported(g, have_bt ? &bt : nullptr, seq) ? seq : 0;
}

wino_status wino_conv2d_fwd(const wino_desc* d, const wino_quant* q, const void* x_dev,
                            const void* U_dev, void* y_dev, void* workspace_dev,
                            size_t workspace_bytes, void* stream) {
  return wino_conv2d_fwd_stages(d, q, x_dev, U_dev, y_dev, workspace_dev, workspace_bytes,
                                WINO_STAGE_ALL, stream);
}

wino_status wino_debug_export(const wino_desc* d, int which, const void* src_dev, void* out_dev,
                              void* stream) {
  Geom g;
  wino_status st = make_geom(d, &g);
  if (st != WINO_OK) return st;
  if (!src_dev || !out_dev) return WINO_E_NULL;
  if (which != WINO_TAP_U && which != WINO_TAP_V && which != WINO_TAP_M) return WINO_E_BAD_ARG;
  if (g.bf16) return WINO_E_BAD_DTYPE;                 // no taps in this mode
  const void* src = src_dev;
  if (which == WINO_TAP_M) src = (const char*)src_dev + v_bytes(g);
  if ((g.w16 ? launch_w16_export(g, which, src, out_dev, (hipStream_t)stream)
             : launch_export(g, which, src, out_dev, (hipStream_t)stream)) != hipSuccess)
    return WINO_E_HIP;
  return WINO_OK;
}

// Cook-Toom / Lagrange construction of a minimal F(m,3) algorithm (Sec. 3.1).
// For finite point p_i:  M_i(x) = prod_{j!=i}(x - p_j), N_i = M_i(p_i),
//   BT[i,:] = sign(N_i) coeffs(M_i),  G[i,b] = p_i^b / |N_i|,  AT[a,i] = p_i^a;
// point at infinity: BT[n-1,:] = coeffs(prod_j (x - p_j)), G[n-1,:] = (0,0,1),
//   AT[m-1,n-1] = 1.
wino_status wino_cook_toom(int m, const double* points, float* BT, float* G, float* AT) {
  if (m != 2 && m != 4 && m != 6) return WINO_E_BAD_M;
  if (!BT || !G || !AT) return WINO_E_NULL;
  static const double kDefault[7] = {0.0, 1.0, -1.0, 0.5, -0.5, 2.0, -2.0};
  const int n = m + 2, np = n - 1;
  const double* pts = points ? points : kDefault;
  for (int i = 0; i < np; ++i) {
    if (!isfinite(pts[i])) return WINO_E_BAD_ARG;
    for (int j = 0; j < i; ++j)
      if (pts[i] == pts[j]) return WINO_E_BAD_ARG;
  }
  for (int i = 0; i < n * n; ++i) BT[i] = 0.0f;
  for (int i = 0; i < n * 3; ++i) G[i] = 0.0f;
  for (int i = 0; i < m * n; ++i) AT[i] = 0.0f;
  long double poly[9];
  for (int i = 0; i <= np; ++i) {      // i == np builds the full product (infinity row)
    int deg = 0;
    poly[0] = 1.0L;
    for (int j = 0; j < np; ++j) {
      if (j == i) continue;
      poly[deg + 1] = 0.0L;            // multiply by (x - p_j)
      for (int k = deg + 1; k >= 1; --k) poly[k] = poly[k - 1] - poly[k] * (long double)pts[j];
      poly[0] = -poly[0] * (long double)pts[j];
      ++deg;
    }
    if (i == np) {
      for (int k = 0; k <= deg; ++k) BT[(n - 1) * n + k] = (float)poly[k];
      G[(n - 1) * 3 + 2] = 1.0f;
      AT[(m - 1) * n + (n - 1)] = 1.0f;
      break;
    }
    const long double p = (long double)pts[i];
    long double Ni = 0.0L, pw = 1.0L;
    for (int k = 0; k <= deg; ++k) { Ni += poly[k] * pw; pw *= p; }
    const long double sgn = Ni < 0 ? -1.0L : 1.0L, aN = Ni < 0 ? -Ni : Ni;
    for (int k = 0; k <= deg; ++k) BT[i * n + k] = (float)(sgn * poly[k]);
    pw = 1.0L;
    for (int b = 0; b < 3; ++b) { G[i * 3 + b] = (float)(pw / aN); pw *= p; }
    pw = 1.0L;
    for (int a = 0; a < m; ++a) { AT[a * n + i] = (float)pw; pw *= p; }
  }
  return WINO_OK;
}

// ------------------------------------------------------------ im2row baseline
static wino_status make_ref_geom(int N, int C, int K, int H, int W, int stride, int pad,
                                 int dtype, RefGeom* g) {
  if (dtype != WINO_F32 && dtype != WINO_I8) return WINO_E_BAD_DTYPE;
  if (N < 1 || C < 1 || K < 1 || H < 1 || W < 1) return WINO_E_BAD_SHAPE;
  if (stride != 1 && stride != 2) return WINO_E_BAD_ARG;
  if (pad != 0 && pad != 1) return WINO_E_BAD_SHAPE;
  if (H + 2 * pad < 3 || W + 2 * pad < 3) return WINO_E_BAD_SHAPE;
  g->N = N; g->C = C; g->K = K; g->H = H; g->W = W; g->stride = stride; g->pad = pad;
  g->Ho = (H + 2 * pad - 3) / stride + 1;
  g->Wo = (W + 2 * pad - 3) / stride + 1;
  g->i8 = dtype == WINO_I8;
  const long long T = (long long)N * g->Ho * g->Wo, limit = 0x7fffffffLL;
  if (T > limit - 64) return WINO_E_BAD_SHAPE;
  g->T = (int)T;
  g->Tp = round_up(g->T, 64);
  g->Cp = round_up(C, g->i8 ? 64 : 16);
  g->Kp = round_up(K, 64);
  if ((long long)g->Tp * 9 * g->Cp > limit || (long long)g->Tp * g->Kp > limit ||
      (long long)N * C * H * W > limit || (long long)g->Kp * 9 * g->Cp > limit)
    return WINO_E_BAD_SHAPE;
  return WINO_OK;
}

size_t conv2d_ref_packed_weights_bytes(int C, int K, int dtype) {
  if (C < 1 || K < 1 || (dtype != WINO_F32 && dtype != WINO_I8)) return 0;
  const int i8 = dtype == WINO_I8;
  // (int8: the tap-major rows and the copy in operand order, one after the other)
  return align256((size_t)round_up(K, 64) * 9 * round_up(C, i8 ? 64 : 16) * (i8 ? 2 : 4));
}

size_t conv2d_ref_workspace_bytes(int N, int C, int K, int H, int W, int stride, int pad,
                                  int dtype) {
  RefGeom g;
  if (make_ref_geom(N, C, K, H, W, stride, pad, dtype, &g) != WINO_OK) return 0;
  return align256((size_t)g.Tp * 9 * g.Cp * (g.i8 ? 1 : 4)) + align256((size_t)g.Tp * g.Kp * 4);
}

wino_status conv2d_ref_pack_weights(int C, int K, int dtype, const void* w_dev, void* wp_dev,
                                    void* stream) {
  if (dtype != WINO_F32 && dtype != WINO_I8) return WINO_E_BAD_DTYPE;
  if (C < 1 || K < 1) return WINO_E_BAD_SHAPE;
  if (!w_dev || !wp_dev) return WINO_E_NULL;
  if (!aligned256(wp_dev)) return WINO_E_WORKSPACE;
  const int i8 = dtype == WINO_I8;
  if ((long long)round_up(K, 64) * 9 * round_up(C, i8 ? 64 : 16) > 0x7fffffffLL)
    return WINO_E_BAD_SHAPE;
  if (launch_ref_pack_weights(C, K, round_up(C, i8 ? 64 : 16), round_up(K, 64), i8, w_dev, wp_dev,
                              (hipStream_t)stream) != hipSuccess)
    return WINO_E_HIP;
  return WINO_OK;
}

// explicit: always the three-kernel form that writes the row matrix.
static wino_status ref_conv(int N, int C, int K, int H, int W, int stride, int pad, int dtype,
                            const void* x_dev, const void* wp_dev, void* y_dev, float s_x, float s_w,
                            float s_y, int qmax, void* workspace_dev, size_t workspace_bytes,
                            void* stream, bool explicit_rows) {
  RefGeom g;
  wino_status st = make_ref_geom(N, C, K, H, W, stride, pad, dtype, &g);
  if (st != WINO_OK) return st;
  if (!x_dev || !wp_dev || !y_dev || !workspace_dev) return WINO_E_NULL;
  float r_y = 1.0f;
  if (g.i8) {
    const float s[3] = {s_x, s_w, s_y};
    for (float v : s)
      if (!isfinite(v) || !(v > 0.0f)) return WINO_E_BAD_SCALE;
    if (qmax < 1 || qmax > 127) return WINO_E_BAD_SCALE;
    volatile float sxw = s_x * s_w;
    r_y = sxw / s_y;
  }
  const size_t rows_b = align256((size_t)g.Tp * 9 * g.Cp * (g.i8 ? 1 : 4));
  if (workspace_bytes < rows_b + align256((size_t)g.Tp * g.Kp * 4) || !aligned256(workspace_dev) ||
      !aligned256(wp_dev))
    return WINO_E_WORKSPACE;
  hipStream_t hs = (hipStream_t)stream;
  if (!explicit_rows && conv_implicit_supported(g)) {
    if (launch_conv_implicit(g, x_dev, wp_dev, y_dev, r_y, (float)qmax, hs) != hipSuccess)
      return WINO_E_HIP;
    return WINO_OK;
  }
  void* rows = workspace_dev;
  void* M = (char*)workspace_dev + rows_b;
  if (launch_im2row(g, x_dev, rows, hs) != hipSuccess) return WINO_E_HIP;
  if (launch_gemm(1, g.Tp, g.Kp, 9 * g.Cp, g.i8, 0, rows, wp_dev, M, hs) != hipSuccess)
    return WINO_E_HIP;
  if (launch_ref_epilogue(g, M, y_dev, r_y, (float)qmax, hs) != hipSuccess) return WINO_E_HIP;
  return WINO_OK;
}

wino_status conv2d_ref_gpu(int N, int C, int K, int H, int W, int stride, int pad, int dtype,
                           const void* x_dev, const void* wp_dev, void* y_dev, float s_x, float s_w,
                           float s_y, int qmax, void* workspace_dev, size_t workspace_bytes,
                           void* stream) {
  return ref_conv(N, C, K, H, W, stride, pad, dtype, x_dev, wp_dev, y_dev, s_x, s_w, s_y, qmax,
                  workspace_dev, workspace_bytes, stream, false);
}

wino_status conv2d_ref_gpu_rows(int N, int C, int K, int H, int W, int stride, int pad, int dtype,
                                const void* x_dev, const void* wp_dev, void* y_dev, float s_x,
                                float s_w, float s_y, int qmax, void* workspace_dev,
                                size_t workspace_bytes, void* stream) {
  return ref_conv(N, C, K, H, W, stride, pad, dtype, x_dev, wp_dev, y_dev, s_x, s_w, s_y, qmax,
                  workspace_dev, workspace_bytes, stream, true);
}

}  // extern "C"
