// int8 Hadamard/GEMM stage fused with the output transform (Eq. 1, Sec. 3.1; GEMM
// formulation of Sec. 5.3) for F(2x2,3x3) layers with 512 input channels and many tiles:
// 32x32x32 MFMAs, workgroup tiles of 32 tiles x 64 output channels.
//
// What bounds this stage on such layers is the number of 1 KB wavefront loads a compute
// unit's L1 has to serve (about 22 cycles each here, whatever the address pattern): a
// workgroup that owns TB tiles x KB output channels loads P * Cp * (TB + KB) bytes.
// gemm_out_col_kernel's 16 x 64 tile makes that 1.3 MB per compute unit for 1 k tiles x 512
// channels; 32 x 64 (the squarest tile that still gives each of the 256 compute units a
// workgroup) makes it 0.79 MB, and every byte is loaded exactly once per workgroup.
//
// The output transform is the column-by-column form of gemm_out_col_kernel: positions are
// visited j outer, i inner, each position's channel reduction is finished before the next
// starts, z[a] = fma(A^T[a][i], M[i][j], z[a]) in ascending i, then
// Y[a][b] = fma(z[a], A^T[b][j], Y[a][b]) in ascending j -- the pinned order of the
// two-sided transform.  The reduction itself is split four ways over the input channels;
// the parts are int32 sums, so the order in which they are added cannot matter.  Output
// codes leave through LDS in NCHW order where a workgroup covers whole images (16-byte
// stores of consecutive planes instead of one 2-byte store per lane, tile row and channel).
//
// Workgroups are numbered so that the ones an XCD receives (dispatch is round-robin over
// the eight XCDs) share a sub-rectangle of the (tile block, channel block) grid: an XCD's
// L2 then fetches only that rectangle's rows of V and U instead of all of one operand.
#include <type_traits>

#include "lds_dma.h"
#include "output_stage.h"

namespace wino {
namespace {

typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Which (tile block, channel block) a workgroup takes: XCD x = blockIdx % 8 owns the
// sub-rectangle (x % XT, x / XT) of ST x SK blocks.
struct XcdMap {
  int XT, ST, SK, nTB, nKB;
};

constexpr int kTB = 32, kKB = 64;              // workgroup tile: tiles x output channels

// NCH = Cp / 64, CH = 64-channel steps per chunk (2 or 4: a row of V contributes CH * 64
// consecutive bytes to a chunk), S = ring slots of V in LDS, D = chunks of U in flight in
// each multiplying wavefront's registers.
//
// Nine wavefronts.  0 .. 7 multiply: (kh, cq) = half of the output channels x quarter of a
// chunk's input channels, 32 tiles x 32 output channels each.  Every byte of U is needed by
// exactly one of them, so U goes straight from global memory into that wavefront's MFMA
// operand registers (its stored order is the operand order: four runs of 256 bytes per
// load).  V (32 rows, needed by both kh) goes through LDS, loaded by wavefront 8, which does
// nothing else.  (With the loads' address arithmetic and waits in the multiplying
// wavefronts, the rate at which a lone wavefront issues instructions was the bound; with
// both operands in LDS, the LDS itself: loads into LDS occupy it at the rate their data
// returns.)  Eight multiplying wavefronts rather than four: each keeps D chunks of its U
// stream in flight in few registers, and owns 4 instead of 8 outputs per lane, which is
// what lets the F(4x4,3x3) output state fit.
template <int M, int NCH, int CH, bool kSparse, int S, int D>
__global__ __launch_bounds__(576, 1) void gemm_out_lds_kernel(
    Geom g, MatAT at, const int8_t* __restrict__ V, const int8_t* __restrict__ U,
    int8_t* __restrict__ y, PosScale w, float r_m, float r_y, float qmax, int fast, int staged,
    XcdMap xm) {
  constexpr int n = M + 2;
  constexpr int NQ = NCH / CH;                 // chunks per position
  constexpr int QC = n * NQ;                   // chunks per column of positions
  constexpr int TOTAL = n * QC;                // chunks in all
  constexpr int VI = kTB * CH / 16;            // 1 KB loads of V per chunk
  constexpr int SLOT = VI * 1024;
  constexpr int NP = 4 * CH;                   // 16-byte pieces of a row per chunk
  constexpr int RPI = 16 / CH;                 // rows of V per 1 KB load
  constexpr int SPW = CH / 2;                  // 32-channel steps per wavefront and chunk
  // exchange area [buffer][kh][owner][source] x 1 KB; one buffer is enough when two barriers
  // lie between the ends of consecutive positions
  constexpr int XBUF = NQ >= 2 ? 1 : 2;
  constexpr int XBYTES = XBUF * 2 * 4 * 3 * 1024;
  static_assert(NCH % CH == 0 && (CH == 2 || CH == 4), "shape");
  static_assert((S - 2) * VI < 64 && S >= 3 && S <= TOTAL && S * SLOT + XBYTES <= 160 * 1024,
                "ring");
  static_assert(QC % 2 == 0 && QC % D == 0, "register sets rotate consistently across columns");
  static_assert(2048 * M * M <= S * SLOT + XBYTES, "the output staging reuses the ring");
  __shared__ __attribute__((aligned(1024))) char lds[S * SLOT + XBYTES];

  // workgroup -> blocks (uniform)
  const int L = blockIdx.x, xcd = L & 7, sidx = L >> 3;
  const int tbi = (xcd % xm.XT) * xm.ST + sidx % xm.ST;
  const int kbi = (xcd / xm.XT) * xm.SK + sidx / xm.ST;
  if (tbi >= xm.nTB || kbi >= xm.nKB) return;

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  char* const xch = lds + S * SLOT;
  // (The compiler sees no store into the ring -- the loads into LDS write it behind its
  // back -- but the exchange area and the output staging are written the ordinary way, so
  // `lds` is ordinary shared memory to it.)

  // Barrier b (b = 0 .. TOTAL - 1) says: chunk b of V has landed in LDS (the loader waited
  // for its loads first), and the multiplying wavefronts hold the operands of chunk b - 1 in
  // registers -- so slot (b - 1) % S is free for chunk b + S - 1.
  if (wave == 8) {
    // ---- loader of V ----
    // A chunk is VI pieces of 1 KB, piece e = rows e*RPI .. of the tile block, each row
    // CH*64 bytes whose 16-byte pieces are stored at piece ^ swz(row): the MFMA operand
    // reads (consecutive rows, one piece index) then hit different bank groups.  Which
    // piece is folded into the per-lane offsets: all loads of a chunk share one base.
    const uint32_t lds0 =
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    uint32_t vlane[VI];
#pragma unroll
    for (int e = 0; e < VI; ++e) {
      const int row = e * RPI + lane / NP;
      const int swe = CH == 4 ? (row & 15) : (row & 7);
      vlane[e] = (uint32_t)(tbi * kTB + row) * (uint32_t)g.Cp + (uint32_t)((lane % NP) ^ swe) * 16u;
    }
    const size_t vplane = (size_t)g.Tp * g.Cp;
    const char* Vb = (const char*)V;
    int ii = 0, ij = 0, icq = 0, islot = 0;    // next chunk to issue: (row, column, channel chunk)
    auto issue_next = [&]() {
      const char* vb = Vb + (size_t)(ii * n + ij) * vplane + (size_t)icq * (CH * 64);
      const uint32_t sl = lds0 + (uint32_t)islot * SLOT;
#pragma unroll
      for (int e = 0; e < VI; ++e) dma_1k(sl + (uint32_t)e * 1024u, vb, vlane[e]);
      if (++icq == NQ) {
        icq = 0;
        if (++ii == n) {
          ii = 0;
          ++ij;
        }
      }
      islot = islot + 1 == S ? 0 : islot + 1;
    };
#pragma unroll 1
    for (int c = 0; c < S - 1; ++c) issue_next();
#pragma unroll 1
    for (int b = 0; b < TOTAL; ++b) {
      // chunk b landed: loads are issued up to chunk min(b + S - 2, TOTAL - 1)
      if (b + S - 2 <= TOTAL - 1) wait_vm<(S - 2) * VI>();
      else wait_vm_chunks<VI, S - 2>(TOTAL - 1 - b);
      lds_barrier();
      if (b + S - 1 < TOTAL) issue_next();
    }
    lds_barrier();                             // barrier TOTAL
    lds_barrier();                             // the last exchange of partial sums
  } else {
    // ---- multiplying wavefronts ----
    const int kh = wave & 1, cq4 = wave >> 1;  // half of the channels out, quarter of a chunk's in
    // V from LDS: row l32 of the tile block, piece 2 * step + half of the chunk's row, for
    // this wavefront's SPW steps of 32 channels (steps cq4*SPW .. of the chunk's 2 CH).
    const int sw = CH == 4 ? (l32 & 15) : (l32 & 7);
    uint32_t vrd[SPW];
#pragma unroll
    for (int s = 0; s < SPW; ++s)
      vrd[s] = (uint32_t)(l32 / RPI) * 1024u + (uint32_t)(l32 % RPI) * (CH * 64) +
               (uint32_t)(((cq4 * SPW + s) * 2 + half) ^ sw) * 16u;
    // U from global memory: output channel k = kh*32 + l32 of the block; the 32-channel
    // step t of a chunk is half (t % 2) of the 64-byte step t / 2, of which this lane
    // takes piece 2 * (t % 2) + half: stored at ((2 (t % 2) + half) * 16 + k % 16) * 16 in
    // the 1 KB block of (16 output channels, 64-byte step).
    const int t0 = cq4 * SPW;
    const uint32_t ulane = (uint32_t)((kh * 2 + (l32 >> 4)) * NCH) * 1024u +
                           (uint32_t)(half * 16 + (l32 & 15)) * 16u;
    const size_t ustep_p = (size_t)(g.Kp >> 4) * NCH * 1024;
    const char* Ub = (const char*)U + (size_t)(kbi * (kKB / 16)) * NCH * 1024 +
                     (size_t)(t0 / 2) * 1024 + (size_t)(t0 % 2) * 512;
    struct UOps {
      v4i u[SPW];
    };
    auto load_u = [&](UOps& o, int i, int j, int cq) {
      size_t off = (size_t)(i * n + j) * ustep_p + (size_t)cq * (CH * 1024);
      asm volatile("" : "+s"(off));
      const char* b = Ub + off + ulane;
#pragma unroll
      for (int s = 0; s < SPW; ++s) o.u[s] = *(const v4i*)(b + s * 512);   // (SPW = 2: t0 even)
      asm volatile("" ::: "memory");
    };
    struct VOps {
      v4i v[SPW];
    };
    auto read_v = [&](VOps& o, int slot) {
      const char* sl = lds + slot * SLOT;
#pragma unroll
      for (int s = 0; s < SPW; ++s) o.v[s] = *(const v4i*)(sl + vrd[s]);
    };

    // A lane ends up owning, for tile l32, the 4 output channels
    // kh*32 + 8 cq4 + 4 half + e (e = 0 .. 3) of the channel block.
    float z[4][M], Y[4][M][M];
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int a = 0; a < M; ++a)
#pragma unroll
        for (int b = 0; b < M; ++b) Y[e][a][b] = 0.0f;

    // End of a position: the four quarters of the reduction meet.  Accumulator group gq
    // (registers 4 gq .. 4 gq + 3: output channels 8 gq + 4 half + rr) belongs to wavefront
    // cq4 = gq; every wavefront sends the three groups it does not own and keeps one.
    v4i own;
    auto swap_out = [&](const v16i& acc, int buf) {
      // (source slot of wavefront c at owner o: (c - o - 1) & 3, one of 0 .. 2)
      char* x = xch + ((buf % XBUF) * 2 + kh) * (12 * 1024) + lane * 16;
      auto send = [&](auto me) {
        constexpr int me_v = decltype(me)::value;
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const v4i grp = v4i{acc[4 * gq], acc[4 * gq + 1], acc[4 * gq + 2], acc[4 * gq + 3]};
          if (gq == me_v) own = grp;
          else *(v4i*)(x + (gq * 3 + ((me_v - gq - 1) & 3)) * 1024) = grp;
        }
      };
      switch (cq4) {
        case 0: send(std::integral_constant<int, 0>{}); break;
        case 1: send(std::integral_constant<int, 1>{}); break;
        case 2: send(std::integral_constant<int, 2>{}); break;
        default: send(std::integral_constant<int, 3>{}); break;
      }
    };
    auto finish_position = [&](auto mq_tag, int i, int j, int buf) {
      constexpr bool kMQ = decltype(mq_tag)::value;
      const char* x = xch + ((buf % XBUF) * 2 + kh) * (12 * 1024) + cq4 * (3 * 1024) + lane * 16;
      v4i sum = own;
#pragma unroll
      for (int d = 1; d < 4; ++d) sum += *(const v4i*)(x + (d - 1) * 1024);
      const float wp = w.r[i * n + j];                 // 1 with per-tensor scales: exact
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float f = (float)sum[e] * wp;
        if constexpr (kMQ) f = quantize_f(f, r_m, qmax);
#pragma unroll
        for (int a = 0; a < M; ++a) {
          z[e][a] = at_step<M, kSparse>(at, a, i, f, z[e][a]);
        }
      }
      if (i == n - 1) {
#pragma unroll
        for (int b = 0; b < M; ++b) {
          const float abj = at.v[b * n + j];
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int a = 0; a < M; ++a) Y[e][a][b] = __builtin_fmaf(z[e][a], abj, Y[e][a][b]);
        }
      }
    };

    // Software pipeline over the chunk sequence c = 0, 1, ... (column j outer, row i, then
    // channel chunk cq): U of chunk c + D is requested while chunk c is multiplied; V of
    // chunk c + 1 arrives from LDS in one register set while chunk c is multiplied out of
    // the other.
    UOps uo[D];
    VOps vo[2];
#pragma unroll
    for (int c = 0; c < D; ++c) load_u(uo[c], (c / NQ) % n, c / QC, c % NQ);
    lds_barrier();                                      // barrier 0
    read_v(vo[0], 0);
    auto columns = [&](auto mq_tag) {
      int slot = 0;                                     // ring slot of the current chunk
#pragma unroll 1
      for (int j = 0; j < n; ++j) {
#pragma unroll
        for (int i = 0; i < n; ++i) {
          v16i acc;
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[e] = 0;
#pragma unroll
          for (int cq = 0; cq < NQ; ++cq) {
            const int idx = i * NQ + cq;                // place in the column
            const int cur = idx & 1, ucur = idx % D;
            slot = slot + 1 == S ? 0 : slot + 1;
            // barrier c + 1 (after the last chunk it only publishes the swapped sums)
            lds_barrier();
            if ((i < n - 1 || cq < NQ - 1 || j < n - 1))
              read_v(vo[cur ^ 1], slot);
            // the position before this one, whose parts were swapped before the barrier
            if (cq == 0 && (i > 0 || j > 0)) {
              if (i > 0) finish_position(mq_tag, i - 1, j, (i - 1) & 1);
              else finish_position(mq_tag, n - 1, j - 1, (n - 1) & 1);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < SPW; ++s)
              acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(uo[ucur].u[s], vo[cur].v[s], acc, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            {
              // U of the chunk D ahead into the registers just used (past the last column
              // the loads repeat the last column's addresses; their data is never used)
              const int nidx = idx + D;
              int jj = j + nidx / QC;
              jj = jj < n ? jj : n - 1;
              load_u(uo[ucur], (nidx % QC) / NQ, jj, nidx % NQ);
            }
          }
          swap_out(acc, i & 1);
        }
      }
      lds_barrier();
      finish_position(mq_tag, n - 1, n - 1, (n - 1) & 1);
    };
    if (r_m > 0.0f) columns(std::true_type{});
    else columns(std::false_type{});

    // Output codes.  All loads into LDS were consumed before the last barrier: the ring is free.
    if (staged) {
      // whole images per workgroup: codes to LDS as [image][channel of the block][Ho][Wo]
      // (the staging may reach into the exchange area: everybody is past its last read of it)
      lds_barrier();
      const int tpi = g.TH * g.TW, pb = g.Ho * g.Wo;    // tiles, bytes per image plane
      const int il = l32 / tpi, trem = l32 - il * tpi, tth = trem / g.TW, ttw = trem - tth * g.TW;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int kl = kh * 32 + cq4 * 8 + half * 4 + e;
        char* plane = lds + (il * kKB + kl) * pb + (tth * M) * g.Wo + ttw * M;
#pragma unroll
        for (int a = 0; a < M; ++a) {
          uint32_t bits = 0;
#pragma unroll
          for (int b = 0; b < M; ++b)
            bits |= ((uint32_t)quantize(Y[e][a][b], r_y, qmax) & 0xffu) << (8 * b);
          if constexpr (M == 2) *(uint16_t*)(plane + a * g.Wo) = (uint16_t)bits;
          else *(uint32_t*)(plane + a * g.Wo) = bits;
        }
      }
    } else if (tbi * kTB + l32 < g.T) {
      const int t = tbi * kTB + l32;
      const int k0 = kbi * kKB + kh * 32 + cq4 * 8 + half * 4;
      const int tw = t % g.TW, tth = (t / g.TW) % g.TH, img = t / (g.TW * g.TH);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int k = k0 + e;
        if (k >= g.K) continue;
        int q[M][M];
#pragma unroll
        for (int a = 0; a < M; ++a)
#pragma unroll
          for (int b = 0; b < M; ++b) q[a][b] = quantize(Y[e][a][b], r_y, qmax);
        store_codes<M, int8_t>(y + ((size_t)img * g.K + k) * g.Ho * g.Wo, g, tth * M, tw * M, q,
                               fast != 0);
      }
    }
  }
  if (staged) {
    // ... then, by all wavefronts, 16-byte pieces of each image's 64 consecutive planes to
    // global memory
    if (wave == 8) lds_barrier();
    lds_barrier();
    const int tpi = g.TH * g.TW, pb = g.Ho * g.Wo;
    const int run = kKB * pb;                           // bytes per image: 64 planes in a row
    const int pieces = (kTB / tpi) * run / 16;
    for (int e = tid; e < pieces; e += 576) {
      const int img_l = e * 16 / run, off = e * 16 - img_l * run;
      const int img = tbi * (kTB / tpi) + img_l;
      if (img < g.N)
        *(v4u*)(y + ((size_t)img * g.K + (size_t)kbi * kKB) * pb + off) =
            *(const v4u*)(lds + e * 16);
    }
  }
}

// Splits the nTB x nKB block grid into 8 sub-rectangles, one per XCD, XT along the tile
// blocks: the split with the least operand bytes per XCD (its rows of V plus its rows of
// U), ties to fewer idle workgroup slots.
XcdMap make_xcd_map(int nTB, int nKB) {
  XcdMap best{1, nTB, (nKB + 7) / 8, nTB, nKB};
  long long best_cost = -1;
  for (int XT = 1; XT <= 8; XT *= 2) {
    const int XK = 8 / XT;
    const int ST = (nTB + XT - 1) / XT, SK = (nKB + XK - 1) / XK;
    // (rows of V + rows of U per XCD, then padding as a small penalty)
    const long long cost = ((long long)ST * kTB + (long long)SK * kKB) * 1024 +
                           ((long long)ST * SK * 8 - (long long)nTB * nKB);
    if (best_cost < 0 || cost < best_cost) {
      best_cost = cost;
      best = XcdMap{XT, ST, SK, nTB, nKB};
    }
  }
  return best;
}

template <int M, int NCH, int CH, bool kSparse, int S, int D>
hipError_t go(const Geom& g, const MatAT& at, const void* V, const void* U, void* y,
              const PosScale* w, float r_m, float r_y, float qmax, hipStream_t s) {
  PosScale one;
  for (int p = 0; p < 64; ++p) one.r[p] = 1.0f;
  const PosScale& ws = w ? *w : one;
  const int whole = g.Ho % M == 0 && g.Wo % M == 0;
  const int fast = whole && ((uintptr_t)y & 3) == 0;
  // (staged stores: whole images per workgroup, every channel of the block real, 16-byte
  // aligned runs)
  const int tpi = g.TH * g.TW;
  const int staged = whole && kTB % tpi == 0 && g.K % kKB == 0 && ((uintptr_t)y & 15) == 0 &&
                     (g.Ho * g.Wo) % 16 == 0 && g.T % kTB == 0;
  const XcdMap xm = make_xcd_map(g.Tp / kTB, g.Kp / kKB);
  gemm_out_lds_kernel<M, NCH, CH, kSparse, S, D><<<dim3(8 * xm.ST * xm.SK), 576, 0, s>>>(
      g, at, (const int8_t*)V, (const int8_t*)U, (int8_t*)y, ws, r_m, r_y, qmax, fast, staged, xm);
  return hipGetLastError();
}

}  // namespace

bool gemm_out_lds_supported(const Geom& g) {
  // (the per-lane part of a V address must fit 32 bits; 1-D grid of 8 * blocks per XCD)
  return g.i8 && g.m == 2 && g.Cp == 512 && (size_t)g.Tp * g.Cp < 0xffffffffull &&
         (long long)(g.Tp / kTB) * (g.Kp / kKB) < (1ll << 27);
}

hipError_t launch_gemm_out_lds(const Geom& g, const MatAT& at, const void* V, const void* U,
                               void* y, const PosScale* w_pos, float r_m, float r_y, float qmax,
                               hipStream_t s) {
  if (!gemm_out_lds_supported(g)) return hipErrorInvalidValue;
  // 256 input channels per chunk, a ring of 6 chunks of V in LDS, 2 chunks of U in flight
  return sparse_at<2>(at.v)
             ? go<2, 8, 4, true, 6, 2>(g, at, V, U, y, w_pos, r_m, r_y, qmax, s)
             : go<2, 8, 4, false, 6, 2>(g, at, V, U, y, w_pos, r_m, r_y, qmax, s);
}

}  // namespace wino
