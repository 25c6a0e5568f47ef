// Host-side launchers of the kernels, one per translation unit, used by the C ABI shell.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>

#include "la_passes.h"

namespace la {

// dtype: the la_dtype of the public header (0 fp32, 1 bf16, 2 / 3 the same with Q, K holding
// feature values already, 4 fp32 with the degree-2 polynomial map: D is then the FEATURE width
// 64, Q and K hold 8 raw values per token)
hipError_t launch_pass_fwd(bool global, int D, int M, int dtype, const PassArgs &a, int nblocks,
                           hipStream_t s);
// dQ, 1/den, delta and (a.totals) the per-segment Q, dO sums; causal or against the global sums
hipError_t launch_pass_dq(bool causal, int D, int M, int dtype, const PassArgs &a, int nblocks,
                          hipStream_t s);
// both reverse passes (dV into a.out, dK into a.out2) on one fetch of the inputs
hipError_t launch_pass_reverse(int D, int M, int dtype, const PassArgs &a, int nblocks,
                               hipStream_t s);
// read-out-only gradients of the non-causal form: dV into a.out, dK into a.out2
hipError_t launch_global_dkdv(int D, int M, int dtype, const PassArgs &a, int nblocks, hipStream_t s);
hipError_t launch_segment_state(int D, int M, int dtype, const SegArgs &a, int nblocks,
                                hipStream_t s);

enum ScanMode { kScanForward = 0, kScanReverse = 1, kScanTotal = 2 };
// In-place scan over the nseg slots of every sequence: exclusive prefix, exclusive
// suffix, or the grand total written to slot 0.
// init_S [BH, DM] / init_z [BH, stride - DM]: optional starting value of the prefix or suffix.
hipError_t launch_scan(float *state, int BH, int nseg, int stride, int mode, hipStream_t s,
                       const float *init_S = nullptr, const float *init_z = nullptr, int DM = 0);

hipError_t launch_recurrent_step(const void *q, const void *k, const void *v, float *S, float *z,
                                 void *out, int BH, int D, int M, float eps, int dtype,
                                 hipStream_t s);

// T steps in one launch; q, k [T, BH, D], v, out [T, BH, M]
hipError_t launch_recurrent_steps(const void *q, const void *k, const void *v, float *S, float *z,
                                  void *out, int steps, int BH, int D, int M, float eps, int dtype,
                                  hipStream_t s);

#define LA_DISPATCH_T(dtype, ...)                                              \
    do {                                                                       \
        if ((dtype) == 0) { using TT = float; __VA_ARGS__; }                   \
        else if ((dtype) == 1) { using TT = bf16_t; __VA_ARGS__; }             \
        else if ((dtype) == 2) { using TT = feat_f32; __VA_ARGS__; }           \
        else if ((dtype) == 3) { using TT = feat_bf16; __VA_ARGS__; }          \
        else return hipErrorInvalidValue;                                      \
    } while (0)

#define LA_DISPATCH_DM(D, M, ...)                                              \
    do {                                                                       \
        if ((D) == 32 && (M) == 32) { constexpr int kD = 32, kM = 32; __VA_ARGS__; }  \
        else if ((D) == 32 && (M) == 64) { constexpr int kD = 32, kM = 64; __VA_ARGS__; } \
        else if ((D) == 64 && (M) == 32) { constexpr int kD = 64, kM = 32; __VA_ARGS__; } \
        else if ((D) == 64 && (M) == 64) { constexpr int kD = 64, kM = 64; __VA_ARGS__; } \
        else return hipErrorInvalidValue;                                      \
    } while (0)

// every supported (D, M, element type): the four head sizes for the first four types; the
// degree-2 polynomial map has 64 features (D = 64 here) and either M
#define LA_DISPATCH(D, M, dtype, ...)                                          \
    do {                                                                       \
        if ((dtype) == 4) {                                                    \
            using TT = poly2_f32;                                              \
            if ((D) == 64 && (M) == 32) { constexpr int kD = 64, kM = 32; __VA_ARGS__; }      \
            else if ((D) == 64 && (M) == 64) { constexpr int kD = 64, kM = 64; __VA_ARGS__; } \
            else return hipErrorInvalidValue;                                  \
        } else {                                                               \
            LA_DISPATCH_DM(D, M, LA_DISPATCH_T(dtype, __VA_ARGS__));           \
        }                                                                      \
    } while (0)

}  // namespace la
