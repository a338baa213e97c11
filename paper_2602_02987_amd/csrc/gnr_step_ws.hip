// Step kernel instantiations: weighted router (deadline rings, randomized split, class draws).
#include "gnr_step.h"

namespace gnr {
GNR_STEP_VARIANT(step_kernel_ws, true, true, false, true)
}
