// The dK/dV pass at head_dim 128 (one workgroup per compute unit with the whole register file), softmax weights, no
// real-time tokens: the instantiation of hta_bwd_dkdv.h that is compiled with the scheduling strategy favouring
// instruction-level parallelism (build.py); its real-time and pointwise variants spill under that strategy and stay with
// the default one in hta_bwd_bf16.hip.
#include "hta_bwd_dkdv.h"

namespace hta {

hipError_t launch_bwd_dkdv128_bf16(const Params& p, hipStream_t s) { return launch_dkdv_as<128, 4, false>(p, s); }

}  // namespace hta
