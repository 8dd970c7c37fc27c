#include "common.hpp"
#include "kernels.hpp"
namespace burst {
hipError_t launch_step_bwd(const BwdParams& p, hipStream_t stream) { return hipErrorNotSupported; }
}
