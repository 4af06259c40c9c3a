// Kernel instantiations of one group of element types (see ttc_kernels.h).
#include "ttc_kernels.h"

namespace ttc {

hipError_t launch_mixed_real(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s)
{
    if (P.dtype == TTC_F32_F64) return launch_mode<float, double, 4, 2>(P, c, A, B, s);
    return launch_mode<double, float, 2, 4>(P, c, A, B, s);
}

}  // namespace ttc
