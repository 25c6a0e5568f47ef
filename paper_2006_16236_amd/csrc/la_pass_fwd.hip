// Forward passes: causal (eq. 9-12), global read-out (eq. 5-6) and the K,V segment totals.
#include "la_launch.h"

namespace la {

hipError_t launch_pass_fwd(bool global, int D, int M, int dtype, const PassArgs &a, int nblocks,
                           hipStream_t s) {
    LA_DISPATCH(D, M, dtype, {
        if (a.tok_heads > 1) {
            if (global) causal_pass_kernel<kGlobal, kD, kM, TT, true><<<nblocks, kWave, 0, s>>>(a);
            else causal_pass_kernel<kFwd, kD, kM, TT, true><<<nblocks, kWave, 0, s>>>(a);
        } else {
            if (global) causal_pass_kernel<kGlobal, kD, kM, TT><<<nblocks, kWave, 0, s>>>(a);
            else causal_pass_kernel<kFwd, kD, kM, TT><<<nblocks, kWave, 0, s>>>(a);
        }
    });
    return hipGetLastError();
}

hipError_t launch_segment_state(int D, int M, int dtype, const SegArgs &a, int nblocks,
                                hipStream_t s) {
    LA_DISPATCH(D, M, dtype, {
        if (a.tok_heads > 1) segment_state_kernel<kD, kM, TT, true><<<nblocks, kWave, 0, s>>>(a);
        else segment_state_kernel<kD, kM, TT><<<nblocks, kWave, 0, s>>>(a);
    });
    return hipGetLastError();
}

}  // namespace la
