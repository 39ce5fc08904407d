// The im2row baseline (Sec. 5.3, Table 3) with the row matrix never written out: the
// same product rows x packed weights, but every workgroup gathers the rows of its own
// output pixels from an input patch it keeps in LDS, and requantizes and stores its
// results itself.  One kernel instead of gather + GEMM + epilogue; int8 only.
//
// Workgroup = 64 output pixels x KW*64 output channels.  The 64 pixels are a block of
// CB columns x RB rows of one image, or NI whole images when an image has fewer than
// 64 output pixels.  Per chunk of 64 input channels the patch of input pixels those
// outputs read ((RB-1)*stride+3 rows x (CB-1)*stride+3 columns per image, zero outside
// the image) is transposed from NCHW into LDS with the channels of a pixel contiguous;
// tap (r, s) of the 3x3 filter then reads, for every output pixel, the 64 bytes at a fixed
// offset from the pixel's corner: one v_mfma_i32_16x16x64_i8 operand per 16 pixels.
// A wavefront owns 16*KW output channels and takes its weight operands straight from the
// packed weights' second copy (1 KB blocks in operand order, [k/16][c/64][tap], written by
// ref_pack_weights_operand_kernel): one contiguous kilobyte per load.  (From the tap-major
// rows a load touched 16 half cache lines: 256 -> 256 channels at 8 x 8, batch 256, took
// 29.7 us instead of 20.8.)
#include <type_traits>

#include "fastdiv.h"
#include "transform_math.h"

namespace wino {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

// Bytes between two pixels of the LDS patch: 64 channels + 16, so that the 16-byte reads
// of 8 consecutive pixels fall into 8 different groups of four banks.
constexpr int kCS = 80;

struct Tiling {
  int CB, RB, NI;        // output columns, rows, images of a workgroup
  int IR, PW;            // input rows / columns of the patch, per image
  int nCB, nRB, nIG;     // grid extents: column blocks, row blocks, image groups
  int PIX;               // NI * RB * CB <= 64
  uint32_t inv_CB, inv_RBCB, inv_IR;   // make_inv of CB, RB * CB, IR
};

// The four dwords d[j] = (byte i of channel j) turned into e[i] = (byte j of column i).
__device__ __forceinline__ void transpose4x4(const uint32_t (&d)[4], uint32_t (&e)[4]) {
  const uint32_t a0 = __builtin_amdgcn_perm(d[1], d[0], 0x05010400u);   // d0.0 d1.0 d0.1 d1.1
  const uint32_t a1 = __builtin_amdgcn_perm(d[1], d[0], 0x07030602u);   // d0.2 d1.2 d0.3 d1.3
  const uint32_t b0 = __builtin_amdgcn_perm(d[3], d[2], 0x05010400u);
  const uint32_t b1 = __builtin_amdgcn_perm(d[3], d[2], 0x07030602u);
  e[0] = __builtin_amdgcn_perm(b0, a0, 0x05040100u);
  e[1] = __builtin_amdgcn_perm(b0, a0, 0x07060302u);
  e[2] = __builtin_amdgcn_perm(b1, a1, 0x05040100u);
  e[3] = __builtin_amdgcn_perm(b1, a1, 0x07060302u);
}

// Pixel p of the workgroup -> image in the group, row and column in the block.
struct PixelAt { int il, row, col; };
__device__ __forceinline__ PixelAt pixel_at(const Tiling& tl, int p) {
  PixelAt a;
  a.il = (int)fast_div((uint32_t)p, tl.inv_RBCB);
  const int rem = p - a.il * (tl.RB * tl.CB);
  a.row = (int)fast_div((uint32_t)rem, tl.inv_CB);
  a.col = rem - a.row * tl.CB;
  return a;
}

// (kLd: how the patch is gathered, see below; a template parameter so that every form gets
// its own register allocation -- as a run-time switch the widest form cost the others a
// wavefront per SIMD)
// kAhead: the pixel operands of the next tap are read from LDS before this tap's MFMAs (see
// below); 34 registers more with KW = 2, i.e. three wavefronts per SIMD instead of four.
template <int KW, int kLd, bool kAhead>
__global__ __launch_bounds__(256) void conv_implicit_i8_kernel(RefGeom g, Tiling tl,
                                                               const int8_t* __restrict__ x,
                                                               const int8_t* __restrict__ wp,
                                                               int8_t* __restrict__ y, float r_y,
                                                               float qmax, int fast_st) {
  constexpr int fast_ld = kLd;
  extern __shared__ __attribute__((aligned(16))) unsigned char Xs[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r16 = lane & 15, grp = lane >> 4;
  int bx = blockIdx.x;
  const int cb = bx % tl.nCB; bx /= tl.nCB;
  const int rb = bx % tl.nRB;
  const int ig = bx / tl.nRB;
  const int k0 = blockIdx.y * (64 * KW) + wave * (16 * KW);
  const int h0 = rb * tl.RB * g.stride - g.pad, w0 = cb * tl.CB * g.stride - g.pad;
  // aligned groups of four input columns that cover the patch's columns w0 .. w0 + PW - 1
  const int qlo = (w0 >= 0 ? w0 : w0 - 3) / 4;
  const int NQ = (w0 + tl.PW - 1) / 4 - qlo + 1;
  const int ntasks = tl.NI * tl.IR * NQ * 16;
  const uint32_t inv_NQ = make_inv((uint32_t)NQ), plane = (uint32_t)(g.H * g.W);

  // LDS offset of the corner (tap 0,0) of the pixel this lane supplies to MFMA row block mt
  int corner[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    int p = mt * 16 + r16;
    if (p >= tl.PIX) p = 0;
    const PixelAt a = pixel_at(tl, p);
    corner[mt] = ((a.il * tl.IR + a.row * g.stride) * tl.PW + a.col * g.stride) * kCS + grp * 16;
  }

  v4i acc[4][KW];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int j = 0; j < KW; ++j) acc[mt][j] = v4i{0, 0, 0, 0};

  const int8_t* wo = wp + ref_operand_weights_offset(g.Cp, g.Kp);
  const int nch = g.Cp >> 6;
  if constexpr (fast_ld == 3) {
    // the whole-plane form below writes the pixels inside the image only: the zero border of
    // the patch is written once, here
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    const int nbytes = tl.NI * tl.IR * tl.PW * kCS;               // a multiple of 16
    for (int i = tid * 16; i < nbytes; i += 256 * 16) *(v4u*)(Xs + i) = v4u{0u, 0u, 0u, 0u};
    __syncthreads();
  }
  for (int ch = 0; ch < nch; ++ch) {
    // this chunk's weight operands: the first kEarly taps are issued before the staging and
    // arrive during it; the rest is issued right after it and arrives while the first taps
    // are multiplied.  (All nine up front keep 72 registers alive through the staging, which
    // holds the kernel with 128 output channels per workgroup to three wavefronts per SIMD;
    // this way it fits four.)
    constexpr int kEarly = KW == 2 ? 4 : 9;
    v4i b[9][KW];
    auto load_b = [&](int tap) {
#pragma unroll
      for (int j = 0; j < KW; ++j)
        b[tap][j] = *(const v4i*)(wo + (((size_t)((k0 >> 4) + j) * nch + ch) * 9 + tap) * 1024 +
                                  lane * 16);
    };
#pragma unroll
    for (int tap = 0; tap < kEarly; ++tap) load_b(tap);
    if (ch) __syncthreads();                           // the previous chunk has been read
    // Transpose the chunk's patch into LDS.  A task: four channels x four input columns
    // of one patch row; 16 consecutive lanes take the 16 channel groups of one place.
    // (fast_ld == 2: four channels x SIXTEEN columns per task, one 16-byte load per channel
    // row -- the 4-byte loads of the other form fetch a 32-byte sector each for four bytes,
    // which made the gather, not the matrix cores, the bound of this kernel)
    if constexpr (fast_ld == 3) {
      // Whole images of 4 or 8 columns: a task is four channels x 16 consecutive bytes of
      // their planes (two or four image rows), so a lane's load is 16 bytes of one cache line
      // and 16 lanes cover a whole 8 x 8 plane -- with 4-byte loads along the rows every lane
      // touched a cache line of its own for four bytes, and the L1's one line per clock, not
      // the matrix cores, set the pace of these layers.
      typedef uint32_t v4u __attribute__((ext_vector_type(4)));
      const int ppp = (int)plane >> 4;                              // 16-byte pieces per plane
      const uint32_t inv_ppp = make_inv((uint32_t)ppp);
      const int wsh = g.W == 8 ? 3 : 2;
      const int ntasks3 = tl.NI * ppp * 16;
      for (int task = tid; task < ntasks3; task += 256) {
        const int cg = task & 15, v = task >> 4;
        const int il = (int)fast_div((uint32_t)v, inv_ppp), q = v - il * ppp;
        const int img = ig * tl.NI + il, c0 = ch * 64 + 4 * cg;
        const uint32_t pbase = ((uint32_t)img * g.C + c0) * plane + 16 * q;
        v4u d4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool ok = img < g.N && c0 + j < g.C;
          const v4u t = *(const v4u*)(x + (ok ? pbase + j * plane : 0u));
          d4[j] = ok ? t : v4u{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int sq = 0; sq < 4; ++sq) {
          uint32_t d[4], e[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) d[j] = d4[j][sq];
          transpose4x4(d, e);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int l = 16 * q + 4 * sq + i;
            const int hr = (l >> wsh) - h0, col = (l & (g.W - 1)) - w0;
            if (hr >= 0 && hr < tl.IR && col >= 0 && col < tl.PW)
              *(uint32_t*)(Xs + ((il * tl.IR + hr) * tl.PW + col) * kCS + 4 * cg) = e[i];
          }
        }
      }
    } else if constexpr (fast_ld == 2) {
      typedef uint32_t v4u __attribute__((ext_vector_type(4)));
      const int qlo16 = w0 < 0 ? -1 : w0 / 16;
      const int NQ16 = (w0 + tl.PW - 1) / 16 - qlo16 + 1;
      const int ntasks16 = tl.NI * tl.IR * NQ16 * 16;
      const uint32_t inv_NQ16 = make_inv((uint32_t)NQ16);
      for (int task = tid; task < ntasks16; task += 256) {
        const int cg = task & 15, v = task >> 4;
        const int prow = (int)fast_div((uint32_t)v, inv_NQ16), q = v - prow * NQ16;
        const int il = (int)fast_div((uint32_t)prow, tl.inv_IR), hr = prow - il * tl.IR;
        const int img = ig * tl.NI + il, h = h0 + hr, wb = 16 * (qlo16 + q);
        const int c0 = ch * 64 + 4 * cg;
        // an aligned group of sixteen columns is inside the image or outside it as a whole
        const bool in = img < g.N && h >= 0 && h < g.H && wb >= 0 && wb < g.W;
        const uint32_t rbase = (((uint32_t)img * g.C + c0) * g.H + h) * g.W;
        v4u d4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool ok = in && c0 + j < g.C;
          const v4u t = *(const v4u*)(x + (ok ? rbase + j * plane + wb : 0u));
          d4[j] = ok ? t : v4u{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int sq = 0; sq < 4; ++sq) {
          uint32_t d[4], e[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) d[j] = d4[j][sq];
          transpose4x4(d, e);
          unsigned char* dst = Xs + (prow * tl.PW + (wb + 4 * sq - w0)) * kCS + 4 * cg;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int col = wb + 4 * sq + i - w0;
            if (col >= 0 && col < tl.PW) *(uint32_t*)(dst + i * kCS) = e[i];
          }
        }
      }
    } else
    for (int task = tid; task < ntasks; task += 256) {
      const int cg = task & 15, v = task >> 4;
      const int prow = (int)fast_div((uint32_t)v, inv_NQ), q = v - prow * NQ;
      const int il = (int)fast_div((uint32_t)prow, tl.inv_IR), hr = prow - il * tl.IR;
      const int img = ig * tl.NI + il, h = h0 + hr, wb = 4 * (qlo + q);
      const int c0 = ch * 64 + 4 * cg;
      const bool rowok = img < g.N && h >= 0 && h < g.H;
      // (every index of x fits 31 bits: the host checks N C H W)
      const uint32_t rbase = (((uint32_t)img * g.C + c0) * g.H + h) * g.W;
      uint32_t d[4], e[4];
      if (fast_ld) {
        // an aligned group of four columns is inside the image or outside it as a whole;
        // loads from clamped addresses, selected afterwards: all four are in flight at once
        const bool in = rowok && wb >= 0 && wb < g.W;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool ok = in && c0 + j < g.C;
          const uint32_t t = *(const uint32_t*)(x + (ok ? rbase + j * plane + wb : 0u));
          d[j] = ok ? t : 0u;
        }
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool ok = rowok && c0 + j < g.C;
          uint32_t t = 0;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int w = wb + i;
            const bool okw = ok && w >= 0 && w < g.W;
            const uint32_t b1 = (uint8_t)x[okw ? rbase + j * plane + w : 0u];
            t |= (okw ? b1 : 0u) << (8 * i);
          }
          d[j] = t;
        }
      }
      transpose4x4(d, e);
      unsigned char* dst = Xs + (prow * tl.PW + (wb - w0)) * kCS + 4 * cg;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int col = wb + i - w0;
        if (col >= 0 && col < tl.PW) *(uint32_t*)(dst + i * kCS) = e[i];
      }
    }
    __syncthreads();
#pragma unroll
    for (int tap = kEarly; tap < 9; ++tap) load_b(tap);
    // kAhead: the pixel operands of tap t + 1 are read from LDS before the MFMAs of tap t are
    // issued, and held there (left to itself the compiler reads two operands, waits for them,
    // and multiplies: some twenty LDS round trips per chunk, which a workgroup that has its
    // compute unit to itself or shares it with one other sits out; with four workgroups per
    // compute unit the others fill the gaps and the registers this takes cost more: 128 -> 128
    // at 16 x 16, batch 256: 20.4 -> 24.5 us with it, 256 -> 256 at 8 x 8: 20.1 -> 19.2).
    // All four row blocks always: a block beyond PIX multiplies pixel 0 again and is dropped
    // at the end, which costs less than branches around the MFMAs.
    if constexpr (kAhead) {
      v4i a[2][4];
      auto read_a = [&](int tap, int buf) {
        const int toff = ((tap / 3) * tl.PW + tap % 3) * kCS;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) a[buf][mt] = *(const v4i*)(Xs + corner[mt] + toff);
      };
      read_a(0, 0);
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        if (tap + 1 < 9) read_a(tap + 1, (tap + 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int j = 0; j < KW; ++j)
            acc[mt][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[tap & 1][mt], b[tap][j],
                                                               acc[mt][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        const int toff = ((tap / 3) * tl.PW + tap % 3) * kCS;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          const v4i a = *(const v4i*)(Xs + corner[mt] + toff);
#pragma unroll
          for (int j = 0; j < KW; ++j)
            acc[mt][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b[tap][j], acc[mt][j], 0, 0, 0);
        }
      }
    }
  }

  // A lane holds, for output channel k0 + 16 j + r16, the pixels 16 mt + 4 grp + 0..3.
  const int hw = g.Ho * g.Wo;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
    for (int j = 0; j < KW; ++j) {
      const int k = k0 + 16 * j + r16;
      const int pb = mt * 16 + grp * 4;
      uint32_t bits[4];
#pragma unroll
      for (int e = 0; e < 4; ++e)
        bits[e] = quantize_bits((float)acc[mt][j][e], r_y, kMagic - qmax, kMagic + qmax);
      if (k >= g.K) continue;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (fast_st && e) break;
        const int p = pb + e;
        if (p >= tl.PIX) break;
        const PixelAt a = pixel_at(tl, p);
        const int img = ig * tl.NI + a.il, ho = rb * tl.RB + a.row, wo = cb * tl.CB + a.col;
        if (img >= g.N || ho >= g.Ho || wo >= g.Wo) continue;
        int8_t* o = y + ((size_t)img * g.K + k) * hw + (size_t)ho * g.Wo + wo;
        if (fast_st)
          *(uint32_t*)o = pack_codes(bits[0], bits[1], bits[2], bits[3]);
        else
          *o = (int8_t)(int)(bits[e] - kMagicBits);
      }
    }
  }
}

Tiling make_tiling(const RefGeom& g) {
  Tiling t;
  t.CB = g.Wo < 64 ? g.Wo : 64;
  t.RB = 64 / t.CB;
  if (t.RB > g.Ho) t.RB = g.Ho;
  t.NI = (t.RB == g.Ho && t.CB == g.Wo) ? 64 / (g.Ho * g.Wo) : 1;
  if (t.NI < 1) t.NI = 1;
  if (t.NI > g.N) t.NI = g.N;
  t.IR = (t.RB - 1) * g.stride + 3;
  t.PW = (t.CB - 1) * g.stride + 3;
  t.nCB = (g.Wo + t.CB - 1) / t.CB;
  t.nRB = (g.Ho + t.RB - 1) / t.RB;
  t.nIG = (g.N + t.NI - 1) / t.NI;
  t.PIX = t.NI * t.RB * t.CB;
  t.inv_CB = make_inv((uint32_t)t.CB);
  t.inv_RBCB = make_inv((uint32_t)(t.RB * t.CB));
  t.inv_IR = make_inv((uint32_t)t.IR);
  return t;
}

}  // namespace

bool conv_implicit_supported(const RefGeom& g) {
  if (!g.i8) return false;
  const Tiling t = make_tiling(g);
  return (long long)t.nCB * t.nRB * t.nIG <= 0x7fffffffLL && g.Kp / 64 <= 65535 &&
         (size_t)t.NI * t.IR * t.PW * kCS <= 65536;
}

hipError_t launch_conv_implicit(const RefGeom& g, const void* x, const void* wp, void* y, float r_y,
                                float qmax, hipStream_t s) {
  if (!conv_implicit_supported(g)) return hipErrorInvalidValue;
  const Tiling t = make_tiling(g);
  const size_t lds = (size_t)t.NI * t.IR * t.PW * kCS;
  // dword loads along the image rows / dword stores of four pixels: every row start and
  // every group of four must be 4-byte aligned
  // whole images per workgroup, 4 or 8 columns, planes that are multiples of 16 bytes
  const bool planes = ((uintptr_t)x & 15) == 0 && (g.W == 4 || g.W == 8) && (g.H * g.W) % 16 == 0 &&
                      t.CB == g.Wo && t.RB == g.Ho;
  const int fast_ld = planes                                        ? 3
                      : (((uintptr_t)x & 15) == 0 && g.W % 16 == 0) ? 2
                      : (((uintptr_t)x & 3) == 0 && g.W % 4 == 0) ? 1
                                                                   : 0;
  const int fast_st = ((uintptr_t)y & 3) == 0 && g.Wo % 4 == 0 && t.CB % 4 == 0;
  const bool two = g.Kp % 128 == 0;
  dim3 grid((unsigned)(t.nCB * t.nRB * t.nIG), (unsigned)(g.Kp / (two ? 128 : 64)));
  // (operands read a tap ahead: 64 output channels per workgroup, or at most two workgroups
  // per compute unit)
  const bool ahead = !two || (long long)grid.x * grid.y <= 512;
  auto go = [&](auto kw, auto ld) {
    if (ahead)
      conv_implicit_i8_kernel<decltype(kw)::value, decltype(ld)::value, true>
          <<<grid, 256, lds, s>>>(g, t, (const int8_t*)x, (const int8_t*)wp, (int8_t*)y, r_y, qmax,
                                  fast_st);
    else
      conv_implicit_i8_kernel<decltype(kw)::value, decltype(ld)::value, false>
          <<<grid, 256, lds, s>>>(g, t, (const int8_t*)x, (const int8_t*)wp, (int8_t*)y, r_y, qmax,
                                  fast_st);
  };
  auto with_ld = [&](auto kw) {
    switch (fast_ld) {
      case 3: go(kw, std::integral_constant<int, 3>{}); break;
      case 2: go(kw, std::integral_constant<int, 2>{}); break;
      case 1: go(kw, std::integral_constant<int, 1>{}); break;
      default: go(kw, std::integral_constant<int, 0>{}); break;
    }
  };
  if (two) with_ld(std::integral_constant<int, 2>{});
  else with_ld(std::integral_constant<int, 1>{});
  return hipGetLastError();
}

}  // namespace wino
