// Instances of the fused decode + matvec kernel for the layout with 16-bit statistics (Sec. 5, ablations): one activation vector per launch.
#include "spqr_gemv_inst.h"

namespace spqr {
SPQR_DEFINE_GEMV_UNIT(l3, 3, SPQR_GEMV_SHAPES, SPQR_NB_1)
}  // namespace spqr
