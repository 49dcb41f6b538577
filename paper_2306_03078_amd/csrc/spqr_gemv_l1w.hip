// Instance of the fused decode + matvec kernel for tiles of 8 x 64 codes (beta1 = 8, beta2 = 64: the size-matched
// setting of Sec. 5), bilevel layout, one activation vector per launch.
#include "spqr_gemv_inst.h"

namespace spqr {
SPQR_DEFINE_GEMV_UNIT(l1w, 1, SPQR_GEMV_WIDE_SHAPES, SPQR_NB_1)
}  // namespace spqr
