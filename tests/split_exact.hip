// GPU check of the operand split of the kernels (la::split3 / la::split2 in la_device.h):
// every fp32 value must equal the sum of its three bf16 parts exactly, the parts must shrink by
// 2^-8 each, and the two-part split must be good to 2^-16.  Runs the library's own device
// functions on 4M values (random bit patterns, values whose roundings carry, tiny and huge
// magnitudes) and compares on the host in double precision.  Exit code 0 = all exact.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../paper_2006_16236_amd/csrc/la_device.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(2); } } while (0)

__global__ void split_kernel(const float *x, unsigned *h, unsigned *m, unsigned *l, unsigned *h2,
                             unsigned *m2, int nquads) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nquads) return;
    const float q[4] = {x[4 * i], x[4 * i + 1], x[4 * i + 2], x[4 * i + 3]};
    const la::Split3 s = la::split3(q);
    const la::Split2 t = la::split2(q);
    for (int j = 0; j < 2; ++j) {
        h[2 * i + j] = s.h[j]; m[2 * i + j] = s.m[j]; l[2 * i + j] = s.l[j];
        h2[2 * i + j] = t.h[j]; m2[2 * i + j] = t.m[j];
    }
}

static double bf(uint16_t b) {
    const uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

int main() {
    const int n = 1 << 22;
    std::vector<float> x(n);
    srand(1);
    for (int i = 0; i < n; ++i) {
        const uint32_t u = ((uint32_t)rand() << 16) ^ (uint32_t)rand() ^ ((uint32_t)rand() << 31);
        float f;
        switch (i % 4) {
            case 0:          // any bit pattern of a finite value of ordinary size
                memcpy(&f, &u, 4);
                if (!isfinite(f) || fabsf(f) > 1e37f || (f != 0 && fabsf(f) < 1e-30f)) f = 1.0f + (u & 0x7fffff) * 1.1920929e-7f;
                break;
            case 1:          // full 24-bit mantissas over 32 binades, both signs
                f = ldexpf((float)(u & 0xffffff) / 16777216.0f + 1.0f, (int)((u >> 24) & 31) - 16) * ((u >> 30) & 1 ? -1.f : 1.f);
                break;
            case 2: {        // long runs of ones: every rounding carries
                uint32_t v = 0x3f800000u | (u & 0x7fffff) | 0x7fff;
                if (u & 0x800000) v &= ~0x8000u;
                memcpy(&f, &v, 4);
                break;
            }
            default: {       // exact ties of the first rounding
                const uint32_t v = 0x3f000000u | ((u & 1) ? 0x7fffffu : 0x7f8000u);
                memcpy(&f, &v, 4);
                f *= (float)((u >> 8) & 255);
            }
        }
        x[i] = f;
    }
    x[0] = 0.f; x[1] = -0.f; x[2] = 1.f; x[3] = 8.5e37f; x[4] = 1e-30f; x[5] = -1e-30f;
    float *dx;
    unsigned *d[5];
    CK(hipMalloc(&dx, (size_t)n * 4));
    for (int k = 0; k < 5; ++k) CK(hipMalloc(&d[k], (size_t)n * 2));
    CK(hipMemcpy(dx, x.data(), (size_t)n * 4, hipMemcpyHostToDevice));
    split_kernel<<<(n / 4 + 255) / 256, 256>>>(dx, d[0], d[1], d[2], d[3], d[4], n / 4);
    CK(hipGetLastError());
    CK(hipDeviceSynchronize());
    std::vector<uint16_t> p[5];
    for (int k = 0; k < 5; ++k) {
        p[k].resize(n);
        CK(hipMemcpy(p[k].data(), d[k], (size_t)n * 2, hipMemcpyDeviceToHost));
    }
    long bad = 0;
    for (int i = 0; i < n; ++i) {
        const double xi = (double)x[i];
        const double h = bf(p[0][i]), m = bf(p[1][i]), l = bf(p[2][i]);
        const bool exact = h + m + l == xi;
        const bool shrink = fabs(m) <= fabs(h) * 0x1p-8 && fabs(l) <= fabs(h) * 0x1p-16;
        const double two = bf(p[3][i]) + bf(p[4][i]);
        const bool close = fabs(two - xi) <= fabs(xi) * 0x1p-16;
        if (!(exact && shrink && close)) {
            if (bad < 10) printf("x=%a: h=%a m=%a l=%a (sum %a), two-part sum %a\n", xi, h, m, l, h + m + l, two);
            ++bad;
        }
    }
    printf("split3 / split2 on %d values: %ld wrong\n", n, bad);
    return bad != 0;
}
