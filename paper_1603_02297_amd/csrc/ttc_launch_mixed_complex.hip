// Kernel instantiations of one group of element types (see ttc_kernels.h).
#include "ttc_kernels.h"

namespace ttc {

hipError_t launch_mixed_complex(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s)
{
    if (P.dtype == TTC_C64_C128) return launch_mode<cfloat, cdouble, 2, 1>(P, c, A, B, s);
    return launch_mode<cdouble, cfloat, 1, 2>(P, c, A, B, s);
}

}  // namespace ttc
