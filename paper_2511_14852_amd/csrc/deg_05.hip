// Specialised kernels of degree 5: explicit instantiation of the per-degree entry points.
#include "degree_impl.h"

namespace chebykan {
template void degree_forward<5, ExactBasis>(const float*, const float*, float*, int, int, int, void*,
                                            const ExactBasis::Args&, hipStream_t);
template void degree_backward<5, ExactBasis>(const float*, const float*, const float*, float*, float*, int, int, int,
                                             void*, const ExactBasis::Args&, hipStream_t);
// the table-interpolated variant (paper Sec. 4.2) of the same kernels
template void degree_forward<5, TableBasis>(const float*, const float*, float*, int, int, int, void*,
                                            const TableBasis::Args&, hipStream_t);
template void degree_backward<5, TableBasis>(const float*, const float*, const float*, float*, float*, int, int, int,
                                             void*, const TableBasis::Args&, hipStream_t);
// the same with the auxiliary derivative table (backward only: forward is that of the table variant)
template void degree_backward<5, DerivTableBasis>(const float*, const float*, const float*, float*, float*, int, int, int,
                                                  void*, const DerivTableBasis::Args&, hipStream_t);
// other bases on the same kernels (paper Sec. 2.3)
template void degree_forward<5, LegendreBasis>(const float*, const float*, float*, int, int, int, void*,
                                            const LegendreBasis::Args&, hipStream_t);
template void degree_backward<5, LegendreBasis>(const float*, const float*, const float*, float*, float*, int, int, int,
                                             void*, const LegendreBasis::Args&, hipStream_t);
template void degree_forward<5, HermiteBasis>(const float*, const float*, float*, int, int, int, void*,
                                            const HermiteBasis::Args&, hipStream_t);
template void degree_backward<5, HermiteBasis>(const float*, const float*, const float*, float*, float*, int, int, int,
                                             void*, const HermiteBasis::Args&, hipStream_t);
// forward of a narrow stack in one launch
template void degree_chain_forward<5>(const ChainArgs&, int, hipStream_t);
template void degree_stack_combine<5>(CombineArgs&, hipStream_t);
template void degree_pair_backward<5>(const PairArgs&, CombineJob*, hipStream_t);
}  // namespace chebykan
