// Step kernel instantiations: randomized router.
#include "gnr_step.h"

namespace gnr {
GNR_STEP_VARIANT(step_kernel_rr, false, true, false, false)
}
