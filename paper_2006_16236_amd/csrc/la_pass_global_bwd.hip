// Gradients of the non-causal form (eq. 4-6) for V and K: read-outs against the grand totals
// (see la_passes.h for the operand table).
#include "la_launch.h"

namespace la {

hipError_t launch_pass_global_bwd(int which, int D, int M, int dtype, const PassArgs &a,
                                  int nblocks, hipStream_t s) {
    LA_DISPATCH_DM(D, M, {
        if (which == 1) {
            if (dtype == 0) causal_pass_kernel<kGlobalDv, kD, kM, float><<<nblocks, kWave, 0, s>>>(a);
            else causal_pass_kernel<kGlobalDv, kD, kM, bf16_t><<<nblocks, kWave, 0, s>>>(a);
        } else {
            if (dtype == 0) causal_pass_kernel<kGlobalDk, kD, kM, float><<<nblocks, kWave, 0, s>>>(a);
            else causal_pass_kernel<kGlobalDk, kD, kM, bf16_t><<<nblocks, kWave, 0, s>>>(a);
        }
    });
    return hipGetLastError();
}

}  // namespace la
