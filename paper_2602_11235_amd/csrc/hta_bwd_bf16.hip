// bf16 backward of Hybrid Target Attention for gfx950: the call's two launches.
//
// Gradient of A = softmax_visible(scale Q K^T) V (the two attention equations of Section 3.2.2)
// with the probabilities recomputed from the saved logsumexp:
//   P = exp(scale S - lse),  dP = dO V^T,  dS = P o (dP - delta),  delta_i = <dO_i, O_i>
//   dV = P^T dO,  dK = scale dS^T Q  (both summed over the query heads of the kv group),  dQ = scale dS K
//
// Three pieces of work in two launches, no atomics, no float32 staging of any gradient:
//   1. bwd_self and 2. bwd_dq (hta_bwd_dq_bf16.hip): the self-key terms of the target rows' keys, and dQ,
//      row-stationary; the first launch also leaves -delta and -lse/scale of every row in the workspace.
//   3. bwd_dkdv (hta_bwd_dkdv.h): key-stationary, dk/dv of history (and real-time) keys, written once.
// S and dP are thus computed twice (7 matrix products instead of 5); in exchange neither dQ nor
// dK/dV ever crosses a workgroup, which removes a float32 accumulator three times the size of q, its
// zero-fill and conversion passes, and an atomic traffic of several GB per call.
// Only history keys are ever visited: target x target and history-row x target-key tiles do not exist
// under the hybrid mask.  Every transposed operand (K^T, Q^T, dO^T) is produced by the LDS transpose
// read from a row-major tile; nothing is transposed when staged.
#include "../../include/mtfm_hta_timing.h"
#include "hta_bwd_dkdv.h"

namespace hta {

hipError_t launch_bwd_bf16(const Params& p, hipStream_t s) {
    timing_begin(MTFM_HTA_KERNEL_BWD_DQ, s);
    hipError_t e = launch_bwd_dq_bf16(p, s);
    timing_end(MTFM_HTA_KERNEL_BWD_DQ, s);
    if (e != hipSuccess) return e;
    timing_begin(MTFM_HTA_KERNEL_BWD_DKDV, s);
    switch (p.d) {
        case 32: e = launch_dkdv<32, 4>(p, s); break;
        case 64: e = launch_dkdv<64, 4>(p, s); break;
        default:  // 128: the softmax kernel for samples without real-time tokens is built in a unit of its own
            if (p.pointwise) e = p.rt_len ? launch_dkdv_as<128, 4, true, true>(p, s) : launch_dkdv_as<128, 4, false, true>(p, s);
            else if (p.rt_len) e = launch_dkdv_as<128, 4, true>(p, s);
            else e = launch_bwd_dkdv128_bf16(p, s);
            break;
    }
    timing_end(MTFM_HTA_KERNEL_BWD_DKDV, s);
    return e;
}

}  // namespace hta
