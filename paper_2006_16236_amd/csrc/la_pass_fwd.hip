// Forward passes: causal (eq. 9-12), global read-out (eq. 5-6) and the K,V segment totals.
#include "la_launch.h"

namespace la {

hipError_t launch_pass_fwd(bool global, int D, int M, int dtype, const PassArgs &a, int nblocks,
                           hipStream_t s) {
    LA_DISPATCH_DM(D, M, {
        if (global) {
            if (dtype == 0) causal_pass_kernel<kGlobal, kD, kM, float><<<nblocks, kWave, 0, s>>>(a);
            else causal_pass_kernel<kGlobal, kD, kM, bf16_t><<<nblocks, kWave, 0, s>>>(a);
        } else {
            if (dtype == 0) causal_pass_kernel<kFwd, kD, kM, float><<<nblocks, kWave, 0, s>>>(a);
            else causal_pass_kernel<kFwd, kD, kM, bf16_t><<<nblocks, kWave, 0, s>>>(a);
        }
    });
    return hipGetLastError();
}

hipError_t launch_segment_state(int D, int M, int dtype, const SegArgs &a, int nblocks,
                                hipStream_t s) {
    LA_DISPATCH_DM(D, M, {
        if (dtype == 0) segment_state_kernel<kD, kM, float><<<nblocks, kWave, 0, s>>>(a);
        else segment_state_kernel<kD, kM, bf16_t><<<nblocks, kWave, 0, s>>>(a);
    });
    return hipGetLastError();
}

}  // namespace la
