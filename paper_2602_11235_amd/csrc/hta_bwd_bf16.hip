#include "hta_common.h"
namespace hta {
hipError_t launch_bwd_bf16(const Params& p, hipStream_t s) { return hipErrorNotSupported; }
}  // namespace hta
