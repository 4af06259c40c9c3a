// Kernel instantiations of one group of element types (see ttc_kernels.h).
#include "ttc_kernels.h"

namespace ttc {

hipError_t launch_f32(const Problem& P, const Candidate& c, const void* A, void* B, hipStream_t s)
{
    return launch_mode<float, float, 4, 4>(P, c, A, B, s);
}

}  // namespace ttc
