// Specialised kernels of degree 24: explicit instantiation of the per-degree entry points.
#include "degree_impl.h"

namespace chebykan {
template void degree_forward<24, ExactBasis>(const float*, const float*, float*, int, int, int, void*,
                                            const ExactBasis::Args&, hipStream_t);
template void degree_backward<24, ExactBasis>(const float*, const float*, const float*, float*, float*, int, int, int,
                                             void*, const ExactBasis::Args&, hipStream_t);
template void degree_stack_combine<24>(CombineArgs&, hipStream_t);
template void degree_pair_backward<24>(const PairArgs&, CombineJob*, hipStream_t);
}  // namespace chebykan
