// Process-wide services of the library (runtime.hip).
#pragma once
#include "../../include/chebykan.h"

namespace chebykan {

// Makes the current device usable: checks that it is a gfx950 part and, the first time on each
// device, raises the dynamic-LDS limit of every registered kernel.  Thread-safe; cheap after the
// first call.  CHEBYKAN_ERR_DEVICE for another architecture or no device, CHEBYKAN_ERR_LAUNCH if
// HIP refuses an attribute.
chebykan_status prepare_device();

// Kernel-family override (chebykan_set_kernel_family): 0 automatic, 1 any-degree, 2 matrix-core.
int kernel_family();

}  // namespace chebykan
