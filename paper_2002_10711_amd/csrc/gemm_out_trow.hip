// int8 Hadamard/GEMM stage fused with the output transform (Eq. 1, Sec. 3.1; GEMM
// formulation of Sec. 5.3) for F(6x6,3x3) with 64, 128 or 256 padded input channels: the
// layers where the output transform's fp32 chains (about 600 fused multiply-adds per tile
// and output channel) are the work and everything else has to stay out of their way.
//
// Same arithmetic as gemm_out_col_kernel: positions are visited column by column (j outer,
// i inner), each position's channel reduction is finished before the next one starts,
// z[a] = fma(A^T[a][i], M[i][j], z[a]) in ascending i, then
// Y[a][b] = fma(z[a], A^T[b][j], Y[a][b]) in ascending j -- the pinned order of the two-sided
// transform.
//
// What differs:
//  * A workgroup is 32 tiles x 32 output channels, and both operands go through LDS in
//    stages of four 64-channel steps (4, 2 or 1 positions), two buffers, ONE barrier per
//    stage instead of one per position; every operand byte is fetched once per workgroup,
//    16 bytes per thread and step, a stage ahead in registers.
//  * Each 16 x 16 MFMA result is shared by TWO wavefronts: a lane of an MFMA result holds
//    four output channels of a tile, and each wavefront transforms two of them (both issue
//    the MFMA; it costs a fiftieth of the chains).  That halves the transform state per lane
//    (84 floats), so four wavefronts fit a SIMD instead of two, and halves the time a
//    wavefront lives: a grid that does not fill the chip evenly ends with a shorter tail.
//    The second wavefront reads the rows of U in an order that puts its two channels where
//    the first one's are, so both run the same code.
//  * A position's operand reads are issued two positions ahead and its MFMAs one position
//    ahead of the chains that consume them, also across a stage's barrier, so the chains
//    wait neither for LDS nor for the matrix cores.
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
// 6 tw, on a dword boundary for even tw and in mid-dword for odd tw.  (Three pairs would
// save the selects and measured 7 % slower on the whole kernel: what the LDS charges for
// is the number of sub-dword writes.)
__device__ __forceinline__ void lds_row6(char* row, bool odd, uint32_t b0, uint32_t b1, uint32_t b2,
                                         uint32_t b3, uint32_t b4, uint32_t b5) {
  const uint32_t lo4 = pack_codes(b0, b1, b2, b3);
  const uint32_t hi2 = __builtin_amdgcn_perm(b5, b4, 0x0c0c0400u);
  const uint32_t dv = odd ? __builtin_amdgcn_alignbit(hi2, lo4, 16) : lo4;
  const uint32_t sv = odd ? lo4 : hi2;
  *(uint32_t*)(row + (odd ? 2 : 0)) = dv;
  *(uint16_t*)(row + (odd ? 0 : 4)) = (uint16_t)sv;
}

// kHalf: two wavefronts per MFMA result (eight wavefronts, two channels per lane, four
// wavefronts per SIMD at 128 registers) -- for 64 input channels, and for 128 while the grid
// gives a compute unit at most one workgroup; otherwise a wavefront keeps all four channels
// of its lanes (four wavefronts, two per SIMD): with longer reductions the operand
// registers of a position press on the 128, and at 256 channels they no longer fit.
// (second launch bound: wavefronts per SIMD)
template <int M, int NCH, bool kSparse, bool kHalf>
__global__ __launch_bounds__(kHalf ? 512 : 256, kHalf ? 4 : 2) void gemm_out_trow_kernel(
    Geom g, MatAT at, const int8_t* __restrict__ V, const int8_t* __restrict__ U,
    int8_t* __restrict__ y, PosScale w, float r_m, float r_y, float qmax, int plain, TrowPlan pl) {
  constexpr int n = M + 2;
  constexpr int G = 4 / NCH;                     // positions per stage
  constexpr int SC = n / G;                      // stages per column
  constexpr int RR = kHalf ? 2 : 4;              // output channels per lane
  constexpr int LPS = kHalf ? 2 : 4;             // 16-byte loads per thread and stage
  constexpr int NW = kHalf ? 8 : 4;              // wavefronts
  // operand reads two positions ahead of their use (else next to their MFMAs, one ahead)
  constexpr bool kDeep = kHalf && NCH <= 2;
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
  // which 16 tiles, which 16 output channels, which two of a lane's four channels
  const int tb2 = wave & 1, kb2 = (wave >> 1) & 1, hf = kHalf ? wave >> 2 : 0;
  const int t0 = tbi * pl.R * g.TW;              // first tile of the block

  // ---- loader side: of every four wavefronts, two fetch V and two fetch U; wavefronts
  // 0 .. 3 take steps 0 and 2 of a stage, wavefronts 4 .. 7 steps 1 and 3 ----
  // Step block in LDS: [32 tile rows x 64 bytes of V][2 x 1 KB of U in operand order].  The
  // 16-byte pieces of a row of V are stored at piece ^ (row / 4 % 4): the operand reads
  // (16 consecutive rows, one piece index) then touch every bank group once.
  const int wl = wave & 3, sp = kHalf ? wave >> 2 : 0;
  const bool ldv = wl < 2;
  const char* const lbase = ldv ? (const char*)V : (const char*)U;
  const size_t pstep = ldv ? (size_t)g.Tp * g.Cp : (size_t)(g.Kp >> 4) * NCH * 1024;
  const uint32_t cstep = ldv ? 64u : 1024u;
  uint32_t loff, ldst;
  {
    const int e = (wl & 1) * 64 + lane;          // piece of the wavefront pair's 2 KB
    const int row = e >> 2, piece = e & 3;
    int tr = t0 + row;
    tr = tr < g.Tp ? tr : g.Tp - 1;              // (idle rows past the end: any valid row)
    const uint32_t voff = (uint32_t)tr * (uint32_t)g.Cp + (uint32_t)piece * 16u;
    const uint32_t vdst = (uint32_t)row * 64u + (uint32_t)(piece ^ ((row >> 2) & 3)) * 16u;
    const uint32_t uoff = (uint32_t)((kbi * 2 + (wl & 1)) * NCH) * 1024u + (uint32_t)lane * 16u;
    const uint32_t udst = 2048u + (uint32_t)e * 16u;
    loff = ldv ? voff : uoff;
    ldst = (ldv ? vdst : udst) + (uint32_t)sp * kStepBytes;
  }
  v4u R[LPS];
  // this wavefront's steps of stage sc of column jj into registers
  auto load_stage = [&](int sc, int jj) {
#pragma unroll
    for (int h = 0; h < LPS; ++h) {
      // step st of the stage: position st / NCH, channel step st % NCH (uniform)
      const int st = kHalf ? 2 * h + sp : h;
      const int i = sc * G + st / NCH, ch = st % NCH;
      size_t off = (size_t)(i * n + jj) * pstep + (size_t)ch * cstep;
      asm volatile("" : "+s"(off));
      R[h] = *(const v4u*)(lbase + off + loff);
    }
  };
  auto write_stage = [&](int buf) {
#pragma unroll
    for (int h = 0; h < LPS; ++h)
      *(v4u*)(lds + buf * kStageBytes + (kHalf ? 2 : 1) * h * kStepBytes + ldst) = R[h];
  };

  // ---- multiplying side ----
  const int vrow = tb2 * 16 + r;
  const uint32_t vrd = (uint32_t)vrow * 64u + (uint32_t)(grp ^ ((vrow >> 2) & 3)) * 16u;
  // (wavefronts with hf = 1 take row r ^ 2 of U as row r of the MFMA: the lane's components
  // 0 and 1 of the result are then the channels the others find in components 2 and 3)
  const uint32_t urd = 2048u + (uint32_t)kb2 * 1024u + (uint32_t)(grp * 16 + (r ^ (hf << 1))) * 16u;
  // The operands of position q of the stage in buffer buf, and their product.  The reads of
  // a position are issued two positions before its accumulators are needed and its MFMAs
  // one position before: a wavefront that has its SIMD to itself (a small layer, the tail
  // of a grid) then waits for neither.
  struct Ops {
    v4i u[NCH], v[NCH];
  };
  auto read_ops = [&](Ops& o, int buf, int q) {
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      const char* sb = lds + buf * kStageBytes + (q * NCH + ch) * kStepBytes;
      o.u[ch] = *(const v4i*)(sb + urd);
      o.v[ch] = *(const v4i*)(sb + vrd);
    }
  };
  auto mfma_ops = [&](const Ops& o) {
    v4i acc = v4i{0, 0, 0, 0};
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch)
      acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(o.u[ch], o.v[ch], acc, 0, 0, 0);
    return acc;
  };
  // The operands of position i2 (0 .. 2 n - 1: positions past n - 1 belong to the next
  // column) of column j.  A position that opens a stage first publishes it: the stage waits
  // in R; it goes into the buffer that held the stage before the current one (everybody
  // passed the current stage's barrier after their last read of it), the stage after it
  // into R, then the barrier.  Past the last stage the same is done with clamped addresses
  // and nobody uses the result: the loop body stays one straight line (a branch here lets
  // the compiler sink the chains behind both stages of a column).
  Ops ops;
  auto fetch_ops = [&](int i2, int j) {
    const int ii = i2 % n, jj = j + i2 / n;
    const int sc = ii / G, q = ii % G;
    if (q == 0) {
      // (nothing of the stage may move up past the chains before it: they are what the
      // loads' latency hides behind)
      if (!kDeep) __builtin_amdgcn_sched_barrier(0);
      write_stage(sc & 1);
      const int jn = jj + (sc + 1) / SC;
      load_stage((sc + 1) % SC, jn < n ? jn : n - 1);
      __syncthreads();
    }
    read_ops(ops, sc & 1, q);
  };

  // A lane owns, for tile vrow of the block, the output channels kb2*16 + grp*4 + 2 hf + rr.
  float z[M][RR], Y[M][M][RR];
#pragma unroll
  for (int a = 0; a < M; ++a)
#pragma unroll
    for (int b = 0; b < M; ++b)
#pragma unroll
      for (int rr = 0; rr < RR; ++rr) Y[a][b][rr] = 0.0f;

  // (one copy of the loop without per-position factors and Hadamard-stage quantizer, one
  // with: multiplying by a factor of 1 is exact, but costs an instruction per accumulator)
  auto columns = [&](auto plain_tag) {
    constexpr bool kPlain = decltype(plain_tag)::value;
    const bool mq = r_m > 0.0f;
    // (the first stage is loaded inside each copy: a value that lives across the branch
    // between the copies is spilled at 128 registers, and a spill here is 64 lanes x 4 bytes
    // per wavefront of memory traffic -- as much as the layer's output for a few registers)
    load_stage(0, 0);
    write_stage(0);
    load_stage(1 % SC, 1 / SC);
    __syncthreads();
    read_ops(ops, 0, 0);
    v4i acc_cur = mfma_ops(ops);
    if (kDeep) fetch_ops(1, 0);
    // One column of positions.  The first and the last column are compiled with j known:
    // A^T has a single nonzero entry there (Cook-Toom pattern), and 5 of the 6 row updates
    // of the second product drop out; the columns between run as a loop.
    auto column = [&](auto jt) {
      constexpr bool kStaticJ = !std::is_same<decltype(jt), int>::value;
      const int j = jt;
#pragma unroll
      for (int i = 0; i < n; ++i) {
        // position i + 1 to the matrix cores, the operands of position i + 2 on their way,
        // then the chains of position i.  (The scheduler may not move anything across the
        // end of this step: it would undo the distance between issue and use.)
        if (!kDeep) fetch_ops(i + 1, j);
        const v4i acc_nx = mfma_ops(ops);
        if (kDeep) fetch_ops(i + 2, j);
        const v4i acc = acc_cur;
        float wp = 1.0f;
        if constexpr (!kPlain) wp = w.r[i * n + j];
#pragma unroll
        for (int rr = 0; rr < RR; ++rr) {
          float f = (float)acc[rr];
          if constexpr (!kPlain) {
            f *= wp;
            const float fq = quantize_f(f, r_m, qmax);
            f = mq ? fq : f;
          }
#pragma unroll
          for (int a = 0; a < M; ++a) {
            z[a][rr] = at_step<M, kSparse>(at, a, i, f, z[a][rr]);
          }
        }
        acc_cur = acc_nx;
        if (kDeep) __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int b = 0; b < M; ++b) {
        if constexpr (kStaticJ) {
          if (!at_nonzero<M, kSparse>(b, decltype(jt)::value)) continue;
        }
        const float abj = at.v[b * n + j];
#pragma unroll
        for (int a = 0; a < M; ++a)
#pragma unroll
          for (int rr = 0; rr < RR; ++rr) Y[a][b][rr] = __builtin_fmaf(z[a][rr], abj, Y[a][b][rr]);
      }
    };
    column(std::integral_constant<int, 0>{});
#pragma unroll 1
    for (int j = 1; j < n - 1; ++j) column(j);
    column(std::integral_constant<int, n - 1>{});
  };
  if (plain) columns(std::true_type{});
  else columns(std::false_type{});

  // ---- output codes: to LDS as [channel of the block][row of tiles][M rows][pitch] ----
  __syncthreads();                               // every operand read is done: LDS is free
  // (the lane's coordinates are derived again from the thread id, hidden from the
  // optimiser: kept alive through the loop they would be spilled, see above)
  int tid_e = threadIdx.x;
  asm volatile("" : "+v"(tid_e));
  const int lane_e = tid_e & 63, r_e = lane_e & 15, grp_e = lane_e >> 4;
  const int vrow_e = tb2 * 16 + r_e;
  {
    const uint32_t trow = fast_div((uint32_t)vrow_e, pl.inv_TW);
    const int tw = vrow_e - (int)trow * g.TW;
    if ((int)trow < pl.R) {
      const float lo = kMagic - qmax, hi = kMagic + qmax;
#pragma unroll
      for (int rr = 0; rr < RR; ++rr) {
        char* tp = lds + (kb2 * 16 + grp_e * 4 + 2 * hf + rr) * pl.plane_b +
                   (int)trow * M * pl.pitch + tw * M;
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
      const uint32_t s = (uint32_t)(lane_e + 64 * h);
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
    for (int kk = wave; kk < 32; kk += NW) {
      const int k = kbi * 32 + kk;
      if (k >= g.K) break;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        if (ok[h]) {
          const uint32_t* sp4 = (const uint32_t*)(lds + kk * pl.plane_b + src[h]);
          *(v4u*)(y + dst[h] + (size_t)k * plane) = v4u{sp4[0], sp4[1], sp4[2], sp4[3]};
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
  // (whole rows of tiles must fill at least three quarters of the 32 MFMA rows: 19 tiles per
  // row -- 112 pixels -- would leave 13 idle, and the column-wise kernel is faster there)
  if (p.R * g.TW < 24) return false;
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

template <int NCH, bool kSparse, bool kHalf>
hipError_t go(const Geom& g, const MatAT& at, const void* V, const void* U, void* y,
              const PosScale* w, float r_m, float r_y, float qmax, const TrowPlan& pl,
              hipStream_t s) {
  PosScale one;
  for (int p = 0; p < 64; ++p) one.r[p] = 1.0f;
  const int plain = !w && !(r_m > 0.0f);
  const unsigned grid = (unsigned)((pl.nTB + 7) / 8 * 8 * pl.nKB);
  gemm_out_trow_kernel<6, NCH, kSparse, kHalf><<<dim3(grid), kHalf ? 512 : 256, 0, s>>>(
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
  const bool sparse = sparse_at<6>(at.v);
#define WINO_TROW_GO(NCHV, HALF)                                                         \
  (sparse ? go<NCHV, true, HALF>(g, at, V, U, y, w_pos, r_m, r_y, qmax, pl, s)           \
          : go<NCHV, false, HALF>(g, at, V, U, y, w_pos, r_m, r_y, qmax, pl, s))
  switch (g.Cp) {
    case 64: return WINO_TROW_GO(1, true);
    case 128:
      // (measured on 128 -> 128 at 16 x 16 and 32 x 32: with at most one workgroup per
      // compute unit the eight-wavefront form is 2 us faster -- two wavefronts per SIMD
      // instead of one --, with more the four-wavefront form is 1 us faster)
      return pl.nTB * pl.nKB <= 256 ? WINO_TROW_GO(2, true) : WINO_TROW_GO(2, false);
    default: return WINO_TROW_GO(4, false);
  }
#undef WINO_TROW_GO
}

}  // namespace wino
