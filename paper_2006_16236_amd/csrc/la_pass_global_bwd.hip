// Gradients of the non-causal form (eq. 4-6) for V and K: read-outs against the grand totals
// (see la_passes.h for the operand table).
#include "la_launch.h"

namespace la {

hipError_t launch_pass_global_bwd(int which, int D, int M, int dtype, const PassArgs &a,
                                  int nblocks, hipStream_t s) {
    LA_DISPATCH(D, M, dtype, {
        if (a.tok_heads > 1) {
            if (which == 1) causal_pass_kernel<kGlobalDv, kD, kM, TT, true><<<nblocks, kWave, 0, s>>>(a);
            else causal_pass_kernel<kGlobalDk, kD, kM, TT, true><<<nblocks, kWave, 0, s>>>(a);
        } else {
            if (which == 1) causal_pass_kernel<kGlobalDv, kD, kM, TT><<<nblocks, kWave, 0, s>>>(a);
            else causal_pass_kernel<kGlobalDk, kD, kM, TT><<<nblocks, kWave, 0, s>>>(a);
        }
    });
    return hipGetLastError();
}

}  // namespace la
