#include "sp_common.hpp"
#include "sp_launch.hpp"
namespace sp {
hipError_t launch_bwd_bf16(const Problem& p, hipStream_t s) { return hipErrorNotSupported; }
}
