// The matrix-core input transform and the one-kernel int8 forward built on it
// (fused_fwd_exact_impl.h), instantiated for F(2x2,3x3); also defines the host-side shape
// predicates.  One translation unit per tile size keeps the build parallel.
#define WINO_EXACT_M 2
#include "fused_fwd_exact_impl.h"
