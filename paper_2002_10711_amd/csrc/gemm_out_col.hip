// int8 Hadamard/GEMM stage fused with the output transform for long reductions (Eq. 1,
// Sec. 3.1; GEMM formulation of Sec. 5.3): M never reaches memory, for 64 .. 512 input
// channels and any number of output channels, with per-tensor or per-position scales.
//
// gemm_out_kernel keeps the accumulators of all n*n Winograd positions in registers, which
// confines it to short reductions.  Here the positions are visited column by column
// (j outer, i inner) and the output transform runs along with them in exactly the pinned
// order: z[a] = fma(A^T[a][i], M[i][j], z[a]) as the accumulators of column j arrive
// (ascending i), then Y[a][b] = fma(z[a], A^T[b][j], Y[a][b]) once the column is complete
// (ascending j).  A lane keeps m + m*m floats per output channel instead of n*n
// accumulators, so the whole reduction of a position can run before the next one starts.
//
// A wavefront owns 16 output channels x kTW blocks of 16 tiles; the four wavefronts of a
// workgroup share the tiles.  V reaches them through LDS (loaded once per workgroup,
// positions ahead in registers, two buffers, one barrier per position); U comes straight
// from global memory in its blocked layout through a register ring.  What bounds such a
// kernel is the number of wavefront loads its compute unit has to take in (about 44 cycles
// per 16-byte-per-lane load as measured in this kernel, first touches from beyond the L2
// included; 15 - 19 from the L2 alone), so every operand is fetched once per workgroup (V)
// or serves kTW MFMAs (U).
#include <type_traits>

#include "output_stage.h"

namespace wino {
namespace {

typedef uint32_t v4u __attribute__((ext_vector_type(4)));

// largest divisor of the steps per column that is at most 16
constexpr int ring_depth(int sj) {
  for (int d = 16; d > 1; --d)
    if (sj % d == 0) return d;
  return 1;
}

// kTwoWG (m = 6 only): held to 128 registers so that two workgroups fit a CU -- it spills a
// little, which pays when the grid would otherwise need a second, mostly empty round.
template <int M, int NCH, bool kSparse, int kTW, bool kTwoWG = false>
__global__ __launch_bounds__(256, kTwoWG ? 2 : 1) void gemm_out_col_kernel(Geom g, MatAT at,
                                                           const int8_t* __restrict__ V,
                                                           const int8_t* __restrict__ U,
                                                           int8_t* __restrict__ y, PosScale w,
                                                           float r_m, float r_y, float qmax,
                                                           int fast) {
  constexpr int n = M + 2;
  constexpr int SJ = n * NCH;                          // steps (64 channels each) per column
  // U ring, in steps (shorter where two workgroups share a CU's registers)
  constexpr int kDepth = (kTwoWG || M == 6) ? 8 : ring_depth(SJ);
  constexpr int kBlocks = NCH * kTW;                   // 1 KB operand blocks of V per position
  constexpr int kLd = (kBlocks + 3) / 4;               // 16-byte loads per thread and position
  constexpr int kPos = kLd > 1 ? 2 : (NCH >= 4 || M == 6) ? n / 2 : n;        // positions ahead
  static_assert(n % kPos == 0 && n % 2 == 0 && kPos + 1 <= n + 1, "static ring slots");
  constexpr int kBufPieces = kBlocks * 64;             // 16-byte pieces of one position
  __shared__ v4u vlds[2 * kBufPieces];
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, grp = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tb = blockIdx.x * 16 * kTW, kb = blockIdx.y * 64;
  // Addresses = uniform byte offset (position, channel step: scalar registers, recomputed
  // per load and hidden from the optimiser, which would otherwise keep one 64-bit vector
  // pointer per load site) + one 32-bit per-lane offset per tensor.
  // U (u_byte_index): block of (position, 16 channels k, 64 channels c) = 1 KB, the
  // lane's piece at lane * 16.
  const char* Ub = (const char*)U;
  const char* Vb = (const char*)V;
  const size_t ublock = (size_t)((kb + wave * 16) >> 4) * NCH * 1024;
  const size_t ustep_p = (size_t)(g.Kp >> 4) * NCH * 1024;
  const size_t vplane = (size_t)g.Tp * g.Cp;           // bytes of one position of V
  const uint32_t ulane = (uint32_t)lane * 16u;
  // V piece e = tid + 256 k of a position, in operand order [channel step][tile block]
  // [tile row][16 bytes]: e & 3 = piece of the 64-byte row, (e >> 2) & 15 = tile,
  // e >> 6 = channel step * kTW + tile block (wave + 4 k)
  const int tbk0 = wave % kTW, ch0 = wave / kTW;
  const uint32_t vthr = (uint32_t)(tb + tbk0 * 16 + ((tid >> 2) & 15)) * (uint32_t)g.Cp +
                        (uint32_t)ch0 * 64u + (uint32_t)(tid & 3) * 16u;
  constexpr int kStepK = 4 / kTW * 64;                 // bytes from load k to load k + 1

  v4i ru[kDepth];
  v4u vst[kPos][kLd];
  auto fetch = [&](int sj, int j, int slot) {
    const int p = (sj / NCH) * n + j, ch = sj % NCH;
    size_t uo = ublock + (size_t)p * ustep_p + (size_t)ch * 1024;
    asm volatile("" : "+s"(uo));
    ru[slot] = *(const v4i*)(Ub + uo + ulane);
  };
  // the workgroup's share of position (i, j) into ring slot `slot` (wavefronts beyond the
  // last operand block of a short reduction load nothing)
  auto vfetch = [&](int i, int j, int slot) {
    const int p = i * n + j;
#pragma unroll
    for (int k = 0; k < kLd; ++k) {
      if (wave + 4 * k < kBlocks) {
        size_t vo = (size_t)p * vplane + (size_t)k * kStepK;
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
  vfetch(0, 0, 0);
  vstore(0, 0);
#pragma unroll
  for (int x = 1; x <= kPos; ++x) vfetch(x % n, x / n, x % kPos);
#pragma unroll
  for (int s = 0; s < kDepth; ++s) fetch(s, 0, s);

  float z[kTW][M][4], Y[kTW][M][M][4];
#pragma unroll
  for (int tk = 0; tk < kTW; ++tk)
#pragma unroll
    for (int a = 0; a < M; ++a)
#pragma unroll
      for (int b = 0; b < M; ++b)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) Y[tk][a][b][rr] = 0.0f;

  // (one copy of the loop per setting of the Hadamard-stage quantizer: a test per
  // accumulator would cut the loop body into pieces the scheduler cannot overlap)
  // Two things a lone wavefront per SIMD needs here.  A position's operands of V are all read
  // from LDS right after the barrier, before the first MFMA (read step by step between the
  // loads of U, each read's latency was waited for in full).  And the output work of a
  // position (conversion, chains) is issued one position late, right after the next
  // position's MFMAs, and pinned there: the wavefront then has it to do while the matrix
  // cores work through that chain of dependent MFMAs (left to itself the compiler collects a
  // whole column's output work behind the column's last MFMA).
  auto columns = [&](auto mq_tag) {
    constexpr bool kMQ = decltype(mq_tag)::value;
    // position (i, j) into the chains z; i is a compile-time value at every call
    auto out_step = [&](int i, float wp, const v4i (&acc)[kTW]) {
#pragma unroll
      for (int tk = 0; tk < kTW; ++tk)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          float f = (float)acc[tk][rr] * wp;
          if constexpr (kMQ) f = quantize_f(f, r_m, qmax);
#pragma unroll
          for (int a = 0; a < M; ++a) z[tk][a][rr] = at_step<M, kSparse>(at, a, i, f, z[tk][a][rr]);
        }
    };
    // column j, complete in z, into Y
    auto y_step = [&](int j) {
#pragma unroll
      for (int b = 0; b < M; ++b) {
        const float abj = at.v[b * n + j];
#pragma unroll
        for (int tk = 0; tk < kTW; ++tk)
#pragma unroll
          for (int a = 0; a < M; ++a)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
              Y[tk][a][b][rr] = __builtin_fmaf(z[tk][a][rr], abj, Y[tk][a][b][rr]);
      }
    };
    // (Where it pays: F(4x4,3x3), and F(2x2,3x3) up to 256 channels.  F(6x6,3x3) and
    // F(2x2,3x3) at 512 channels pass 256 registers with it and lose their second resident
    // workgroup: up to 2.3 times slower on 512 -> 512 at 32 x 32 with F6.  They keep the
    // plain order: operands read step by step, output work right behind the MFMAs.)
    constexpr bool kLate = M == 4 || (M == 2 && NCH <= 4);
    v4i prev[kTW];                                     // sums of the position before this one
#pragma unroll
    for (int tk = 0; tk < kTW; ++tk) prev[tk] = v4i{0, 0, 0, 0};
#pragma unroll 1
    for (int j = 0; j < n; ++j) {
      // (columns past the last: the loads repeat valid addresses, their data is never used)
      const int jn = j + 1 < n ? j + 1 : j, jnn = j + 2 < n ? j + 2 : n - 1;
#pragma unroll
      for (int i = 0; i < n; ++i) {
        // Every wavefront has finished the previous position, whose buffer the next
        // position's operands may now overwrite; this position's buffer is complete.
        __syncthreads();
        // factor of the position whose output work follows this position's MFMAs (1 with
        // per-tensor scales: exact); a scalar load, requested here so that it is not waited
        // for there
        float wp = 1.0f;
        if constexpr (kLate)
          wp = i > 0 ? w.r[(i - 1) * n + j] : w.r[(n - 1) * n + (j > 0 ? j - 1 : 0)];
        const v4i* vops = (const v4i*)(vlds + (i & 1) * kBufPieces) + (r * 4 + grp);
        // (with two tile blocks per wavefront the 2 NCH operands up front would push the
        // F(2x2,3x3) form past 256 registers, which costs it its second resident workgroup)
        constexpr bool kHoist = kLate && kTW == 1;
        v4i vr[kHoist ? NCH : 1][kTW];
        if constexpr (kHoist) {
#pragma unroll
          for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
            for (int tk = 0; tk < kTW; ++tk) vr[ch][tk] = vops[(ch * kTW + tk) * 64];
        }
        vstore((i + 1) % kPos, (i + 1) & 1);
        constexpr int kAhead = 1 + kPos;
        vfetch((i + kAhead) % n, (i + kAhead) / n == 0 ? j : (i + kAhead) / n == 1 ? jn : jnn,
               (i + 1) % kPos);
        v4i acc[kTW];
#pragma unroll
        for (int tk = 0; tk < kTW; ++tk) acc[tk] = v4i{0, 0, 0, 0};
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
          const int sj = i * NCH + ch, slot = sj % kDepth;
          const v4i u = ru[slot];
#pragma unroll
          for (int tk = 0; tk < kTW; ++tk)
            acc[tk] = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                u, kHoist ? vr[kHoist ? ch : 0][tk] : vops[(ch * kTW + tk) * 64], acc[tk], 0, 0, 0);
          // refill the slot once its operand has been issued; the compiler-level fence
          // keeps later steps' loads behind this one, so that the ring, not the
          // scheduler, decides what is in flight
          if (sj + kDepth < SJ) fetch(sj + kDepth, j, slot);
          else fetch(sj + kDepth - SJ, jn, slot);
          asm volatile("" ::: "memory");
        }
        if constexpr (kLate) {
          __builtin_amdgcn_sched_barrier(0);
          if (i > 0) {
            out_step(i - 1, wp, prev);
          } else if (j > 0) {
            out_step(n - 1, wp, prev);
            y_step(j - 1);
          }
          // (the chains' values are claimed here, so that their instructions stay here)
#pragma unroll
          for (int tk = 0; tk < kTW; ++tk)
#pragma unroll
            for (int a = 0; a < M; ++a)
#pragma unroll
              for (int rr = 0; rr < 4; ++rr) asm volatile("" : "+v"(z[tk][a][rr]));
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int tk = 0; tk < kTW; ++tk) prev[tk] = acc[tk];
        } else {
          out_step(i, w.r[i * n + j], acc);
        }
      }
      if constexpr (!kLate) y_step(j);
    }
    if constexpr (kLate) {
      out_step(n - 1, w.r[n * n - 1], prev);
      y_step(n - 1);
    }
  };
  if (r_m > 0.0f) columns(std::true_type{});
  else columns(std::false_type{});

#pragma unroll
  for (int tk = 0; tk < kTW; ++tk) {
    const int t = tb + tk * 16 + r;
    if (t >= g.T) continue;
    const int tw = t % g.TW, th = (t / g.TW) % g.TH, img = t / (g.TW * g.TH);
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int k = kb + wave * 16 + grp * 4 + rr;
      if (k >= g.K) continue;
      int q[M][M];
#pragma unroll
      for (int a = 0; a < M; ++a)
#pragma unroll
        for (int b = 0; b < M; ++b) q[a][b] = quantize(Y[tk][a][b][rr], r_y, qmax);
      store_codes<M, int8_t>(y + ((size_t)img * g.K + k) * g.Ho * g.Wo, g, th * M, tw * M, q,
                             fast != 0);
    }
  }
}

template <int M, bool kSparse>
hipError_t launch_ms(const Geom& g, const MatAT& at, const void* V, const void* U, void* y,
                     const PosScale* w, float r_m, float r_y, float qmax, hipStream_t s,
                     bool two_blocks) {
  PosScale one;
  for (int p = 0; p < 64; ++p) one.r[p] = 1.0f;
  const PosScale& ws = w ? *w : one;
  const int8_t* Vi = (const int8_t*)V;
  const int8_t* Ui = (const int8_t*)U;
  int8_t* yo = (int8_t*)y;
  const int fast = g.Ho % M == 0 && g.Wo % M == 0 && ((uintptr_t)y & 3) == 0;
#define WINO_COL_GO(NCHV)                                                                \
  gemm_out_col_kernel<M, NCHV, kSparse, 1><<<dim3(g.Tp / 16, g.Kp / 64), 256, 0, s>>>(   \
      g, at, Vi, Ui, yo, ws, r_m, r_y, qmax, fast)
#define WINO_COL_GO2(NCHV)                                                               \
  gemm_out_col_kernel<M, NCHV, kSparse, 2><<<dim3(g.Tp / 32, g.Kp / 64), 256, 0, s>>>(   \
      g, at, Vi, Ui, yo, ws, r_m, r_y, qmax, fast)
  // Two tile blocks per wavefront halve the operand loads of U per MFMA and the number of
  // workgroups; built where it has measured faster on layers with many tiles (F2 at 256
  // channels, F4 at 512 channels).
  if (two_blocks) {
    if constexpr (M == 2) {
      if (g.Cp == 256) {
        WINO_COL_GO2(4);
        return hipGetLastError();
      }
    }
    if constexpr (M == 4) {
      if (g.Cp == 512) {
        WINO_COL_GO2(8);
        return hipGetLastError();
      }
    }
    return hipErrorInvalidValue;
  }
  if constexpr (M == 6) {
    // more workgroups than CUs, but not many more: two per CU finish in one round
    const long long wgs = (long long)(g.Tp / 16) * (g.Kp / 64);
    if (wgs > 256) {
#define WINO_COL_GO6(NCHV)                                                               \
  gemm_out_col_kernel<M, NCHV, kSparse, 1, true><<<dim3(g.Tp / 16, g.Kp / 64), 256, 0, s>>>( \
      g, at, Vi, Ui, yo, ws, r_m, r_y, qmax, fast)
      switch (g.Cp) {
        case 64: WINO_COL_GO6(1); break;
        case 128: WINO_COL_GO6(2); break;
        case 192: WINO_COL_GO6(3); break;
        case 256: WINO_COL_GO6(4); break;
        case 320: WINO_COL_GO6(5); break;
        case 384: WINO_COL_GO6(6); break;
        case 448: WINO_COL_GO6(7); break;
        default: WINO_COL_GO6(8); break;
      }
#undef WINO_COL_GO6
      return hipGetLastError();
    }
  }
  switch (g.Cp) {
    case 64: WINO_COL_GO(1); break;
    case 128: WINO_COL_GO(2); break;
    case 192: WINO_COL_GO(3); break;
    case 256: WINO_COL_GO(4); break;
    case 320: WINO_COL_GO(5); break;
    case 384: WINO_COL_GO(6); break;
    case 448: WINO_COL_GO(7); break;
    default: WINO_COL_GO(8); break;
  }
#undef WINO_COL_GO2
#undef WINO_COL_GO
  return hipGetLastError();
}

template <int M>
hipError_t launch_m(const Geom& g, const MatAT& at, const void* V, const void* U, void* y,
                    const PosScale* w, float r_m, float r_y, float qmax, hipStream_t s, bool two) {
  return sparse_at<M>(at.v)
             ? launch_ms<M, true>(g, at, V, U, y, w, r_m, r_y, qmax, s, two)
             : launch_ms<M, false>(g, at, V, U, y, w, r_m, r_y, qmax, s, two);
}

}  // namespace

bool gemm_out_col_supported(const Geom& g) {
  const bool nch_ok = g.Cp % 64 == 0 && g.Cp >= 64 && g.Cp <= 512;
  // (the per-thread part of a V address must fit 32 bits)
  return g.i8 && nch_ok && g.Kp / 64 <= 65535 && (size_t)g.Tp * g.Cp < 0xffffffffull;
}

bool gemm_out_col2_supported(const Geom& g) {
  return gemm_out_col_supported(g) && ((g.m == 2 && g.Cp == 256) || (g.m == 4 && g.Cp == 512));
}

hipError_t launch_gemm_out_col(const Geom& g, const MatAT& at, const void* V, const void* U,
                               void* y, const PosScale* w_pos, float r_m, float r_y, float qmax,
                               hipStream_t s, bool two_blocks) {
  if (!(two_blocks ? gemm_out_col2_supported(g) : gemm_out_col_supported(g)))
    return hipErrorInvalidValue;
  switch (g.m) {
    case 2: return launch_m<2>(g, at, V, U, y, w_pos, r_m, r_y, qmax, s, two_blocks);
    case 4: return launch_m<4>(g, at, V, U, y, w_pos, r_m, r_y, qmax, s, two_blocks);
    default: return launch_m<6>(g, at, V, U, y, w_pos, r_m, r_y, qmax, s, two_blocks);
  }
}

}  // namespace wino
