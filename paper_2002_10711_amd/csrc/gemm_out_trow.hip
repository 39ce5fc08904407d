// int8 Hadamard/GEMM stage fused with the output transform (Eq. 1, Sec. 3.1; GEMM
// formulation of Sec. 5.3) for F(6x6,3x3) with 64, 128 or 256 padded input channels: the
// layers where the output transform's fp32 chains (about 600 fused multiply-adds per tile
// and output channel) are the work and everything else has to stay out of their way.
//
// Same arithmetic as gemm_out_col_kernel: positions are visited column by column (j outer,
// i inner), each position's channel reduction is finished before the next one starts,
// z[a] = fma(A^T[a][i], M[i][j], z[a]) in ascending i, then
// Y[a][b] = fma(z[a], A^T[b][j], Y[a][b]) in ascending j -- the pinned order of the two-sided
// transform.  A wavefront owns 16 tiles x 16 output channels (one MFMA result per position).
//
// What differs:
//  * A workgroup is 2 x 2 wavefronts = 32 tiles x 32 output channels, and both operands go
//    through LDS in stages of four 64-channel steps (4, 2 or 1 positions), two buffers, ONE
//    barrier per stage instead of one per position: 16 bytes per thread and step, loaded a
//    stage ahead into registers.  Every operand byte is fetched once per workgroup.
//  * The MFMAs of the next position are issued before the chains of the current one, also
//    across a stage's barrier, so the chains never wait for the matrix cores.
//  * The 32 tiles are whole rows of tiles (R = 32 / TW rows; the rest of the 32 is idle):
//    a row of tiles is M consecutive rows of an output plane, i.e. one run of consecutive
//    bytes.  The codes are assembled in LDS and leave as 16-byte stores of those runs
//    instead of one 2-byte store per lane, tile row and pair of pixels (6 does not divide
//    the image sizes, so the per-lane stores of the other kernels are 2-byte stores with
//    bounds checks: a third of their memory instructions).
//  * Workgroups that share a block of tiles are neighbours on one XCD (dispatch is
//    round-robin over the eight XCDs), so V reaches each L2 once.
#include <type_traits>

#include "fastdiv.h"
#include "output_stage.h"

namespace wino {
namespace {

typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int kStepBytes = 4096;                 // one 64-channel step: 2 KB of V, 2 KB of U
constexpr int kStageBytes = 4 * kStepBytes;
constexpr int kLdsBytes = 40 * 1024;             // two stages, or the staged output codes

struct TrowPlan {
  int R;                  // rows of tiles per workgroup
  int rows_all;           // N * TH
  int nTB, nKB;           // blocks of tile rows, blocks of 32 output channels
  int pitch, plane_b;     // staged codes: bytes per row, bytes per output channel
  int ppr, ppt;           // 16-byte pieces per output row, per row of tiles
  uint32_t inv_TW, inv_TH, inv_ppt, inv_ppr, inv_nKB;
};

// Six codes (low bytes of b0 .. b5) to LDS as a dword and a pair: tile columns start at
// 6 tw, on a dword boundary for even tw and in mid-dword for odd tw.
__device__ __forceinline__ void lds_row6(char* row, bool odd, uint32_t b0, uint32_t b1, uint32_t b2,
                                         uint32_t b3, uint32_t b4, uint32_t b5) {
  const uint32_t lo4 = pack_codes(b0, b1, b2, b3);
  const uint32_t hi2 = __builtin_amdgcn_perm(b5, b4, 0x0c0c0400u);
  const uint32_t dv = odd ? __builtin_amdgcn_alignbit(hi2, lo4, 16) : lo4;
  const uint32_t sv = odd ? lo4 : hi2;
  *(uint32_t*)(row + (odd ? 2 : 0)) = dv;
  *(uint16_t*)(row + (odd ? 0 : 4)) = (uint16_t)sv;
}

template <int M, int NCH, bool kSparse>
__global__ __launch_bounds__(256, 2) void gemm_out_trow_kernel(
    Geom g, MatAT at, const int8_t* __restrict__ V, const int8_t* __restrict__ U,
    int8_t* __restrict__ y, PosScale w, float r_m, float r_y, float qmax, int plain, TrowPlan pl) {
  constexpr int n = M + 2;
  constexpr int G = 4 / NCH;                     // positions per stage
  constexpr int SC = n / G;                      // stages per column
  static_assert(M == 6, "the row stores are written for six codes per tile row");
  static_assert(NCH == 1 || NCH == 2 || NCH == 4, "a stage is four steps");
  static_assert(n % G == 0 && SC % 2 == 0, "a column is a whole, even number of stages");
  __shared__ __attribute__((aligned(16))) char lds[kLdsBytes];

  // workgroup -> (block of tile rows, block of output channels); uniform
  const uint32_t L = blockIdx.x, xcd = L & 7u, idx = L >> 3;
  const uint32_t tq = fast_div(idx, pl.inv_nKB);
  const int kbi = (int)(idx - tq * (uint32_t)pl.nKB);
  const int tbi = (int)(tq * 8u + xcd);
  if (tbi >= pl.nTB) return;

  const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, grp = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tb2 = wave & 1, kb2 = wave >> 1;     // which 16 tiles, which 16 output channels
  const int t0 = tbi * pl.R * g.TW;              // first tile of the block

  // ---- loader side: wavefronts 0, 1 fetch V, wavefronts 2, 3 fetch U ----
  // Step block in LDS: [32 tile rows x 64 bytes of V][2 x 1 KB of U in operand order].  The
  // 16-byte pieces of a row of V are stored at piece ^ (row / 4 % 4): the operand reads
  // (16 consecutive rows, one piece index) then touch every bank group once.
  const bool ldv = wave < 2;
  const char* const lbase = ldv ? (const char*)V : (const char*)U;
  const size_t pstep = ldv ? (size_t)g.Tp * g.Cp : (size_t)(g.Kp >> 4) * NCH * 1024;
  const uint32_t cstep = ldv ? 64u : 1024u;
  uint32_t loff, ldst;
  {
    const int e = (wave & 1) * 64 + lane;        // piece of the wavefront pair's 2 KB
    const int row = e >> 2, piece = e & 3;
    int tr = t0 + row;
    tr = tr < g.Tp ? tr : g.Tp - 1;              // (idle rows past the end: any valid row)
    const uint32_t voff = (uint32_t)tr * (uint32_t)g.Cp + (uint32_t)piece * 16u;
    const uint32_t vdst = (uint32_t)row * 64u + (uint32_t)(piece ^ ((row >> 2) & 3)) * 16u;
    const uint32_t uoff = (uint32_t)((kbi * 2 + (wave & 1)) * NCH) * 1024u + (uint32_t)lane * 16u;
    const uint32_t udst = 2048u + (uint32_t)e * 16u;
    loff = ldv ? voff : uoff;
    ldst = ldv ? vdst : udst;
  }
  v4u R[4];
  // the four steps of stage sc of column jj into registers
  auto load_stage = [&](int sc, int jj) {
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      const int i = sc * G + st / NCH, ch = st % NCH;
      size_t off = (size_t)(i * n + jj) * pstep + (size_t)ch * cstep;
      asm volatile("" : "+s"(off));
      R[st] = *(const v4u*)(lbase + off + loff);
    }
  };
  auto write_stage = [&](int buf) {
#pragma unroll
    for (int st = 0; st < 4; ++st) *(v4u*)(lds + buf * kStageBytes + st * kStepBytes + ldst) = R[st];
  };

  // ---- multiplying side ----
  const int vrow = tb2 * 16 + r;
  const uint32_t vrd = (uint32_t)vrow * 64u + (uint32_t)(grp ^ ((vrow >> 2) & 3)) * 16u;
  const uint32_t urd = 2048u + (uint32_t)kb2 * 1024u + (uint32_t)lane * 16u;
  // the accumulators of position q of the stage in buffer buf
  auto mfma_pos = [&](int buf, int q) {
    v4i acc = v4i{0, 0, 0, 0};
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      const char* sb = lds + buf * kStageBytes + (q * NCH + ch) * kStepBytes;
      const v4i u = *(const v4i*)(sb + urd);
      const v4i v = *(const v4i*)(sb + vrd);
      acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(u, v, acc, 0, 0, 0);
    }
    return acc;
  };

  // A lane owns, for tile vrow of the block, the output channels kb2*16 + grp*4 + rr.
  float z[M][4], Y[M][M][4];
#pragma unroll
  for (int a = 0; a < M; ++a)
#pragma unroll
    for (int b = 0; b < M; ++b)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) Y[a][b][rr] = 0.0f;

  load_stage(0, 0);
  write_stage(0);
  load_stage(1, 0);
  __syncthreads();
  v4i acc_nx = mfma_pos(0, 0);

  // (one copy of the loop without per-position factors and Hadamard-stage quantizer, one
  // with: multiplying by a factor of 1 is exact, but costs an instruction per accumulator)
  auto columns = [&](auto plain_tag) {
    constexpr bool kPlain = decltype(plain_tag)::value;
    const bool mq = r_m > 0.0f;
#pragma unroll 1
    for (int j = 0; j < n; ++j) {
#pragma unroll
      for (int i = 0; i < n; ++i) {
        const int q = i % G, sc = i / G;
        const v4i acc = acc_nx;
        if (q == G - 1) {
          // The next position opens a stage.  Its operands wait in R: into the buffer that
          // held the stage before this one (everybody passed this stage's barrier after
          // their last read of it), then the stage after it into R, then the barrier that
          // publishes the buffer.  Past the last stage the same is done with clamped
          // addresses and nobody reads the result: the loop body stays one straight line
          // (a branch here lets the compiler sink the chains behind both stages of a column).
          // The scheduler may not move a stage's memory operations up past the chains of the
          // positions before it: those chains are what the loads' latency hides behind.
          __builtin_amdgcn_sched_barrier(0);
          write_stage((sc + 1) & 1);
          const int jn = j + (sc + 2) / SC;
          load_stage((sc + 2) % SC, jn < n ? jn : n - 1);
          __syncthreads();
        }
        acc_nx = i < n - 1 ? mfma_pos(((i + 1) / G) & 1, (i + 1) % G) : mfma_pos(0, 0);
        float wp = 1.0f;
        if constexpr (!kPlain) wp = w.r[i * n + j];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          float f = (float)acc[rr];
          if constexpr (!kPlain) {
            f *= wp;
            const float fq = quantize_f(f, r_m, qmax);
            f = mq ? fq : f;
          }
#pragma unroll
          for (int a = 0; a < M; ++a) {
            if (i == 0) z[a][rr] = 0.0f;
            if (at_nonzero<M, kSparse>(a, i)) z[a][rr] = __builtin_fmaf(at.v[a * n + i], f, z[a][rr]);
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
  if (plain) columns(std::true_type{});
  else columns(std::false_type{});

  // ---- output codes: to LDS as [channel of the block][row of tiles][M rows][pitch] ----
  __syncthreads();                               // every operand read is done: LDS is free
  {
    const uint32_t trow = fast_div((uint32_t)vrow, pl.inv_TW);
    const int tw = vrow - (int)trow * g.TW;
    if ((int)trow < pl.R) {
      const float lo = kMagic - qmax, hi = kMagic + qmax;
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        char* tp = lds + (kb2 * 16 + grp * 4 + rr) * pl.plane_b + (int)trow * M * pl.pitch + tw * M;
#pragma unroll
        for (int a = 0; a < M; ++a) {
          uint32_t b[M];
#pragma unroll
          for (int c = 0; c < M; ++c) b[c] = quantize_bits(Y[a][c][rr], r_y, lo, hi);
          lds_row6(tp + a * pl.pitch, (tw & 1) != 0, b[0], b[1], b[2], b[3], b[4], b[5]);
        }
      }
    }
  }
  __syncthreads();
  // ... and out: a plane's share of the block is R runs of M * Wo consecutive bytes (fewer
  // rows at the lower image edge); slot s of a plane = (row of tiles, row, 16-byte piece).
  {
    const int slots = pl.R * pl.ppt;             // <= 72
    uint32_t src[2];
    size_t dst[2];
    bool ok[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t s = (uint32_t)(lane + 64 * h);
      const uint32_t trow = fast_div(s, pl.inv_ppt);
      const uint32_t rem = s - trow * (uint32_t)pl.ppt;
      const uint32_t yr = fast_div(rem, pl.inv_ppr), x16 = rem - yr * (uint32_t)pl.ppr;
      const uint32_t gr = (uint32_t)(tbi * pl.R) + trow;      // row of tiles in the batch
      const uint32_t img = fast_div(gr, pl.inv_TH), th = gr - img * (uint32_t)g.TH;
      const uint32_t oy = th * M + yr;
      ok[h] = (int)s < slots && (int)gr < pl.rows_all && (int)oy < g.Ho;
      src[h] = (trow * M + yr) * (uint32_t)pl.pitch + x16 * 16u;
      dst[h] = ((size_t)img * g.K * g.Ho + oy) * g.Wo + x16 * 16u;
    }
    const size_t plane = (size_t)g.Ho * g.Wo;
#pragma unroll 1
    for (int kk = wave; kk < 32; kk += 4) {
      const int k = kbi * 32 + kk;
      if (k >= g.K) break;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        if (ok[h]) {
          const uint32_t* sp = (const uint32_t*)(lds + kk * pl.plane_b + src[h]);
          *(v4u*)(y + dst[h] + (size_t)k * plane) = v4u{sp[0], sp[1], sp[2], sp[3]};
        }
      }
    }
  }
}

bool make_plan(const Geom& g, TrowPlan* pl) {
  if (!g.i8 || g.w16 || g.m != 6) return false;
  if (!(g.Cp == 64 || g.Cp == 128 || g.Cp == 256)) return false;
  if (g.TW > 32 || g.TW < 1 || g.Wo % 16 != 0) return false;
  const int M = 6;
  TrowPlan p;
  p.R = 32 / g.TW;
  const long long rows_all = (long long)g.N * g.TH;
  p.rows_all = (int)rows_all;
  p.nTB = (int)((rows_all + p.R - 1) / p.R);
  p.nKB = g.Kp / 32;
  p.pitch = round_up(g.TW * M, 4);
  p.plane_b = p.R * M * p.pitch;
  p.ppr = g.Wo / 16;
  p.ppt = M * p.ppr;
  if (32 * p.plane_b > kLdsBytes || p.R * p.ppt > 128) return false;
  // 32-bit per-lane offsets, exact reciprocal divisions, 1-D grid
  if ((size_t)g.Tp * g.Cp >= 0xffffffffull || (size_t)g.Kp * g.Cp >= 0xffffffffull) return false;
  if (rows_all >= (1ll << 24) || g.TH > 255 || p.nKB > 256 ||
      (long long)(p.nTB + 7) / 8 * 8 * p.nKB >= (1ll << 24))
    return false;
  p.inv_TW = make_inv((uint32_t)g.TW);
  p.inv_TH = make_inv((uint32_t)g.TH);
  p.inv_ppt = make_inv((uint32_t)p.ppt);
  p.inv_ppr = make_inv((uint32_t)p.ppr);
  p.inv_nKB = make_inv((uint32_t)p.nKB);
  *pl = p;
  return true;
}

template <int NCH, bool kSparse>
hipError_t go(const Geom& g, const MatAT& at, const void* V, const void* U, void* y,
              const PosScale* w, float r_m, float r_y, float qmax, const TrowPlan& pl,
              hipStream_t s) {
  PosScale one;
  for (int p = 0; p < 64; ++p) one.r[p] = 1.0f;
  const int plain = !w && !(r_m > 0.0f);
  const unsigned grid = (unsigned)((pl.nTB + 7) / 8 * 8 * pl.nKB);
  gemm_out_trow_kernel<6, NCH, kSparse><<<dim3(grid), 256, 0, s>>>(
      g, at, (const int8_t*)V, (const int8_t*)U, (int8_t*)y, w ? *w : one, r_m, r_y, qmax, plain, pl);
  return hipGetLastError();
}

}  // namespace

bool gemm_out_trow_supported(const Geom& g) {
  TrowPlan pl;
  return make_plan(g, &pl);
}

hipError_t launch_gemm_out_trow(const Geom& g, const MatAT& at, const void* V, const void* U,
                                void* y, const PosScale* w_pos, float r_m, float r_y, float qmax,
                                hipStream_t s) {
  TrowPlan pl;
  if (!make_plan(g, &pl) || ((uintptr_t)y & 15) != 0) return hipErrorInvalidValue;
  const bool sparse = fits_mask(at.v, g.m * g.n, CookToomMask<6>::at);
#define WINO_TROW_GO(NCHV)                                                               \
  (sparse ? go<NCHV, true>(g, at, V, U, y, w_pos, r_m, r_y, qmax, pl, s)                 \
          : go<NCHV, false>(g, at, V, U, y, w_pos, r_m, r_y, qmax, pl, s))
  switch (g.Cp) {
    case 64: return WINO_TROW_GO(1);
    case 128: return WINO_TROW_GO(2);
    default: return WINO_TROW_GO(4);
  }
#undef WINO_TROW_GO
}

}  // namespace wino
