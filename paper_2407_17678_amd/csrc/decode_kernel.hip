#include "kernels.h"
namespace s2 {
hipError_t launch_decode(const DecodeParams&, hipStream_t) { return hipErrorNotSupported; }
}
