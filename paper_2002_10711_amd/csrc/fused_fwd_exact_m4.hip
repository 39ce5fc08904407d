// The matrix-core input transform and the one-kernel int8 forward built on it
// (fused_fwd_exact_impl.h), instantiated for F(4x4,3x3); also defines the entry points that
// dispatch on the tile size.
#define WINO_EXACT_M 4
#include "fused_fwd_exact_impl.h"
