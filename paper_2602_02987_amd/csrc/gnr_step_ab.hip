// Step kernel instantiations: abandonment, solo-first router.
#include "gnr_step.h"

namespace gnr {
GNR_STEP_VARIANT(step_kernel_ab, true, false, false, false)
}
