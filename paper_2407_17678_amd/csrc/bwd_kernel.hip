// placeholder until the backward kernels land
#include "kernels.h"
namespace s2 {
hipError_t launch_bwd(const AttnParams&, bool, hipStream_t) { return hipErrorNotSupported; }
}
