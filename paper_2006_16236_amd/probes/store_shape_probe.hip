// Probe: does the shape of the stores matter?  Copy of 16x64 fp32 tiles with three store patterns.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e_), __LINE__); exit(1);} } while (0)
typedef float f4 __attribute__((ext_vector_type(4)));
template <int MODE, bool NT>
__global__ __launch_bounds__(64) void tilecopy(const float *src, float *dst, size_t tiles_per_wg) {
    const int lane = threadIdx.x, c = lane & 15, g = lane >> 4;
    const float *s = src + (size_t)blockIdx.x * tiles_per_wg * 1024;
    float *d = dst + (size_t)blockIdx.x * tiles_per_wg * 1024;
    f4 cur[4];
    for (int i = 0; i < 4; ++i) cur[i] = *reinterpret_cast<const f4 *>(s + 4 * (lane + 64 * i));
    for (size_t t = 0; t < tiles_per_wg; ++t) {
        f4 nxt[4];
        const size_t tn = t + 1 < tiles_per_wg ? t + 1 : t;
        for (int i = 0; i < 4; ++i) nxt[i] = *reinterpret_cast<const f4 *>(s + tn * 1024 + 4 * (lane + 64 * i));
        float *o = d + t * 1024;
        if (MODE == 0) {
            for (int i = 0; i < 4; ++i) {
                f4 *q = reinterpret_cast<f4 *>(o + 4 * (lane + 64 * i));
                if (NT) __builtin_nontemporal_store(cur[i], q); else *q = cur[i];
            }
        } else if (MODE == 1) {
            for (int r = 0; r < 4; ++r)
                for (int zt = 0; zt < 4; ++zt) {
                    float *q = o + (4 * g + r) * 64 + 16 * zt + c;
                    if (NT) __builtin_nontemporal_store(cur[zt][r], q); else *q = cur[zt][r];
                }
        } else {
            for (int zt = 0; zt < 4; ++zt) {
                f4 *q = reinterpret_cast<f4 *>(o + c * 64 + 16 * zt + 4 * g);
                if (NT) __builtin_nontemporal_store(cur[zt], q); else *q = cur[zt];
            }
        }
        for (int i = 0; i < 4; ++i) cur[i] = nxt[i];
    }
}
int main() {
    const size_t bytes = (size_t)512 << 20;
    float *a, *b; CK(hipMalloc(&a, bytes)); CK(hipMalloc(&b, bytes));
    CK(hipMemset(a, 0, bytes)); CK(hipMemset(b, 0, bytes));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int nwg = 2048; const size_t tpw = bytes / 4096 / nwg;
    auto timeit = [&](auto launch, const char *name) {
        for (int i = 0; i < 10; ++i) launch();
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0));
        for (int i = 0; i < 20; ++i) launch();
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= 20;
        printf("%-44s %.3f ms  %.0f GB/s (read+write)\n", name, ms, 2.0 * bytes / ms / 1e6); fflush(stdout);
    };
    timeit([&] { tilecopy<0, false><<<nwg, 64>>>(a, b, tpw); }, "16 B/lane, 1 KiB contiguous per instr");
    timeit([&] { tilecopy<1, false><<<nwg, 64>>>(a, b, tpw); }, "4 B/lane, 4 rows x 64 B per instr (x16)");
    timeit([&] { tilecopy<2, false><<<nwg, 64>>>(a, b, tpw); }, "16 B/lane, 16 rows x 64 B per instr (x4)");
    timeit([&] { tilecopy<0, true><<<nwg, 64>>>(a, b, tpw); }, "nt: 16 B/lane, 1 KiB contiguous per instr");
    timeit([&] { tilecopy<1, true><<<nwg, 64>>>(a, b, tpw); }, "nt: 4 B/lane, 4 rows x 64 B per instr (x16)");
    timeit([&] { tilecopy<2, true><<<nwg, 64>>>(a, b, tpw); }, "nt: 16 B/lane, 16 rows x 64 B per instr (x4)");
    return 0;
}
