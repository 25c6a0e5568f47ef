// Forward-direction half of the backward: dQ (eq. 13), causal and non-causal (see la_passes.h).
#include "la_launch.h"

namespace la {

hipError_t launch_pass_dq(bool causal, int D, int M, int dtype, const PassArgs &a, int nblocks,
                          hipStream_t s) {
    LA_DISPATCH(D, M, dtype, {
        if (a.tok_heads > 1) {
            if (!causal) dq_pass_kernel<kD, kM, TT, true><<<nblocks, 2 * kWave, 0, s>>>(a);
            else dq_causal_kernel<kD, kM, TT, true><<<nblocks, 2 * kWave, 0, s>>>(a);
        } else {
            if (!causal) dq_pass_kernel<kD, kM, TT><<<nblocks, 2 * kWave, 0, s>>>(a);
            else dq_causal_kernel<kD, kM, TT><<<nblocks, 2 * kWave, 0, s>>>(a);
        }
    });
    return hipGetLastError();
}

}  // namespace la
