// Reverse-direction half of the backward: dV (eq. 15) and dK (eq. 14) in one kernel, two
// waves per workgroup sharing one fetch of Q, K, V and dO (see la_passes.h).
#include "la_launch.h"

namespace la {

hipError_t launch_pass_reverse(int D, int M, int dtype, const PassArgs &a, int nblocks,
                               hipStream_t s) {
    LA_DISPATCH(D, M, dtype, {
        if (a.tok_heads > 1) reverse_pass_kernel<kD, kM, TT, true><<<nblocks, 2 * kWave, 0, s>>>(a);
        else reverse_pass_kernel<kD, kM, TT><<<nblocks, 2 * kWave, 0, s>>>(a);
    });
    return hipGetLastError();
}

}  // namespace la
