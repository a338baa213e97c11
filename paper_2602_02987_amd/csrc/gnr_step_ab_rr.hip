// Step kernel instantiations: abandonment, randomized router.
#include "gnr_step.h"

namespace gnr {
GNR_STEP_VARIANT(step_kernel_ab_rr, true, true, false, false)
}
