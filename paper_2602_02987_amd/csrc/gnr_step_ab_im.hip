// Step kernel instantiations: abandonment, immediate decode.
#include "gnr_step.h"

namespace gnr {
GNR_STEP_VARIANT(step_kernel_ab_im, true, false, true, false)
}
