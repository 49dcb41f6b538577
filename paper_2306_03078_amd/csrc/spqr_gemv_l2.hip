// Instances of the fused decode + matvec kernel for the integer zero-point layout (Sec. 5, ablations): one activation vector per launch.
#include "spqr_gemv_inst.h"

namespace spqr {
SPQR_DEFINE_GEMV_UNIT(l2, 2, SPQR_GEMV_SHAPES, SPQR_NB_1)
}  // namespace spqr
