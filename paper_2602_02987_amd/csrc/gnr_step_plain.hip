// Step kernel instantiations: solo-first router, no abandonment.
#include "gnr_step.h"

namespace gnr {
GNR_STEP_VARIANT(step_kernel_plain, false, false, false, false)
}
