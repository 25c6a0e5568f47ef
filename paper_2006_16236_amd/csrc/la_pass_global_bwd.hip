// Gradients of the non-causal form (eq. 4-6) for V and K: read-outs against the grand totals,
// both in one kernel (see la_passes.h for the operand table).
#include "la_launch.h"

namespace la {

hipError_t launch_global_dkdv(int D, int M, int dtype, const PassArgs &a, int nblocks, hipStream_t s) {
    LA_DISPATCH(D, M, dtype, {
        if (a.tok_heads > 1) global_dkdv_kernel<kD, kM, TT, true><<<nblocks, 2 * kWave, 0, s>>>(a);
        else global_dkdv_kernel<kD, kM, TT><<<nblocks, 2 * kWave, 0, s>>>(a);
    });
    return hipGetLastError();
}

}  // namespace la
