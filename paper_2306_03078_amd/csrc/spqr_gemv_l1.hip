// Instances of the fused decode + matvec kernel for the bilevel layout (Sec. 4.2): 1, 2 and 4 activation vectors per launch.
#include "spqr_gemv_inst.h"

namespace spqr {
SPQR_DEFINE_GEMV_UNIT(l1, 1, SPQR_GEMV_SHAPES, SPQR_NB_124)
}  // namespace spqr
