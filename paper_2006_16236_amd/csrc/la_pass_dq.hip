// Backward pass kDq of Algorithm 1 (see la_passes.h for the operand table).
#include "la_launch.h"

namespace la {

hipError_t launch_pass_dq(int D, int M, int dtype, const PassArgs &a, int nblocks, hipStream_t s) {
    LA_DISPATCH_DM(D, M, {
        if (dtype == 0) dq_pass_kernel<kD, kM, float><<<nblocks, 2 * kWave, 0, s>>>(a);
        else dq_pass_kernel<kD, kM, bf16_t><<<nblocks, 2 * kWave, 0, s>>>(a);
    });
    return hipGetLastError();
}

}  // namespace la
