// Which kernel sequence the int8 forward takes (Sec. 5.3 of the paper picks the algorithm
// per layer shape from measured latencies; the same idea one level down, for the kernel
// sequences of one algorithm).  dispatch_table.h holds, for every point of a measured grid
// of (tile size, padded input channels, output-channel class, tiles), the sequences that
// can run there ordered by their measured time; a problem takes the first sequence of the
// nearest point's list that supports it.
#include <math.h>

#include "wino_internal.h"

namespace wino {

struct DispatchRow {
  int m, Cp, kclass, hw, T;      // kclass: Kp <= 64: 0, <= 128: 1, more: 2; hw: image height
  unsigned char rank[kSeqCount];  // sequence ids, fastest first, 0-terminated
};

#include "dispatch_table.h"

namespace {

int kclass_of(int Kp) { return Kp <= 64 ? 0 : Kp <= 128 ? 1 : 2; }

// The heuristics the table replaced, used only if the table has no row for a tile size.
void fallback_rank(const Geom& g, unsigned char* rank) {
  int n = 0;
  if (g.Kp <= 128 && (g.m == 2 || g.Cp <= 192) && (g.Cp <= 128 || g.T >= 2048)) rank[n++] = kSeqFused;
  if (g.T >= 1024) rank[n++] = kSeqLds;
  if (g.T >= 1024) rank[n++] = kSeqTrow;
  if (g.m == 2 || (g.m == 4 && (g.Cp <= 128 || (g.Cp <= 256 ? g.T >= 128 : g.T >= 512))) ||
      (g.m == 6 && g.Cp >= 128 && g.T >= 1024))
    rank[n++] = kSeqCol;
  if (g.Cp <= (g.m == 6 ? 64 : 128)) rank[n++] = kSeqRegs;
  rank[n++] = kSeqStaged;
  rank[n] = 0;
}

}  // namespace

bool fwd_sequence_supported(const Geom& g, const MatBT* bt, int seq) {
  if (!g.i8) return false;
  switch (seq) {
    case kSeqFused:
      return fused_fwd_supported(g) &&
             ((bt && fused_fwd_exact_supported(g, *bt)) || fused_fwd_generic_preferred(g));
    case kSeqCol: return gemm_out_col_supported(g);
    case kSeqCol2: return gemm_out_col2_supported(g);
    case kSeqLds: return gemm_out_lds_supported(g);
    case kSeqTrow: return gemm_out_trow_supported(g);
    case kSeqRegs:
      // (32-bit per-lane offsets; reductions beyond 256 channels are not worth 64
      // accumulator sets waiting for them)
      return g.Cp <= 256 && g.Kp / 64 <= 65535 && (size_t)g.Tp * g.Cp < 0xffffffffull &&
             (size_t)g.Kp * g.Cp < 0xffffffffull;
    case kSeqStaged: return true;
    default: return false;
  }
}

int fwd_sequence_auto(const Geom& g, const MatBT* bt, bool allow_fused) {
  if (!g.i8) return kSeqStaged;
  // learned (inexact) B^T: the one-kernel forward with the vector-ALU transform wherever it
  // is built (measured against two kernels when those kernels were written)
  const bool exact = bt && fused_fwd_exact_supported(g, *bt);
  if (allow_fused && !exact && fused_fwd_supported(g) && fused_fwd_generic_preferred(g))
    return kSeqFused;
  const DispatchRow* best = nullptr;
  float best_d = 0.0f;
  const float lc = log2f((float)g.Cp), lt = log2f((float)g.T), lh = log2f((float)g.H);
  const int kc = kclass_of(g.Kp);
  for (size_t i = 0; i < sizeof(kDispatch) / sizeof(kDispatch[0]); ++i) {
    const DispatchRow& r = kDispatch[i];
    if (r.m != g.m) continue;
    const float d = 8.0f * fabsf(lc - log2f((float)r.Cp)) + 3.0f * fabsf((float)(kc - r.kclass)) +
                    fabsf(lt - log2f((float)r.T)) + 0.25f * fabsf(lh - log2f((float)r.hw));
    if (!best || d < best_d) {
      best = &r;
      best_d = d;
    }
  }
  unsigned char fb[kSeqCount];
  const unsigned char* rank = best ? best->rank : fb;
  if (!best) fallback_rank(g, fb);
  for (int i = 0; i < kSeqCount && rank[i]; ++i) {
    if (rank[i] == kSeqFused && !allow_fused) continue;
    if (fwd_sequence_supported(g, bt, rank[i])) return rank[i];
  }
  return kSeqStaged;
}

}  // namespace wino
