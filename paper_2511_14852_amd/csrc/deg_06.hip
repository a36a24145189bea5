// Specialised kernels of degree 6: explicit instantiation of the per-degree entry points.
#include "degree_impl.h"

namespace chebykan {
template void degree_forward<6>(const float*, const float*, float*, int, int, int, void*, hipStream_t);
template void degree_backward<6>(const float*, const float*, const float*, float*, float*, int, int, int, void*,
                                  hipStream_t);
}  // namespace chebykan
