// Specialised kernels of degree 15: explicit instantiation of the per-degree entry points.
#include "degree_impl.h"

namespace chebykan {
template void degree_forward<15>(const float*, const float*, float*, int, int, int, void*, hipStream_t);
template void degree_backward<15>(const float*, const float*, const float*, float*, float*, int, int, int, void*,
                                  hipStream_t);
}  // namespace chebykan
