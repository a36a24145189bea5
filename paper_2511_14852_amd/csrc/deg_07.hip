// Specialised kernels of degree 7: explicit instantiation of the per-degree entry points.
#include "degree_impl.h"

namespace chebykan {
template void degree_forward<7, ExactBasis>(const float*, const float*, float*, int, int, int, void*,
                                            const ExactBasis::Args&, hipStream_t);
template void degree_backward<7, ExactBasis>(const float*, const float*, const float*, float*, float*, int, int, int,
                                             void*, const ExactBasis::Args&, hipStream_t);
// the table-interpolated variant (paper Sec. 4.2) of the same kernels
template void degree_forward<7, TableBasis>(const float*, const float*, float*, int, int, int, void*,
                                            const TableBasis::Args&, hipStream_t);
template void degree_backward<7, TableBasis>(const float*, const float*, const float*, float*, float*, int, int, int,
                                             void*, const TableBasis::Args&, hipStream_t);
// the same with the auxiliary derivative table (backward only: forward is that of the table variant)
template void degree_backward<7, DerivTableBasis>(const float*, const float*, const float*, float*, float*, int, int, int,
                                                  void*, const DerivTableBasis::Args&, hipStream_t);
template void degree_stack_combine<7>(CombineArgs&, hipStream_t);
template void degree_pair_backward<7>(const PairArgs&, CombineJob*, hipStream_t);
}  // namespace chebykan
