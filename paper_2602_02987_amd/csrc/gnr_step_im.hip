// Step kernel instantiations: immediate same-slot decode.
#include "gnr_step.h"

namespace gnr {
GNR_STEP_VARIANT(step_kernel_im, false, false, true, false)
}
