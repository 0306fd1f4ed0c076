// placeholder until the backward kernels land
#include "gsa_launch.h"
namespace gsa {
hipError_t launch_bwd(const Plan &, const Work &, const void *, const void *, const void *, const float *,
                      const float *, const float *, const float *, const void *, const float *, const float *, void *,
                      void *, void *, float *, float *, float *, hipStream_t)
{
    return hipErrorNotSupported;
}
}  // namespace gsa
