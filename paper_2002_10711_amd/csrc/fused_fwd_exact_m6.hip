// The matrix-core input transform (fused_fwd_exact_impl.h) instantiated for F(6x6,3x3): the
// input stage alone, with the Kronecker matrix in two int8 digits.
#define WINO_EXACT_M 6
#include "fused_fwd_exact_impl.h"
