// Probe of the memory-side cache: how fast is a second read of a buffer that a kernel has just
// read, in the same or in the opposite walking direction, and a read right after a copy wrote it?
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <vector>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e_), __LINE__); exit(1);} } while (0)
typedef float f4 __attribute__((ext_vector_type(4)));
// each workgroup (64 threads) walks its own contiguous slice in 4 KiB steps (4 loads of 1 KiB per wave in flight)
__global__ __launch_bounds__(64) void walk(const f4 *p, size_t slice_f4, int dir, float *sink) {
    const f4 *base = p + (size_t)blockIdx.x * slice_f4;
    const size_t steps = slice_f4 / 256;     // 256 f4 = 4 KiB per step
    f4 acc = {0, 0, 0, 0};
    for (size_t s = 0; s < steps; ++s) {
        const size_t st = dir > 0 ? s : steps - 1 - s;
        const f4 *q = base + st * 256 + threadIdx.x;
        f4 a = q[0], b = q[64], c = q[128], d = q[192];
        acc += a + b + c + d;
    }
    if (acc[0] + acc[1] + acc[2] + acc[3] == 12345.678f) sink[blockIdx.x] = acc[0];
}
__global__ __launch_bounds__(64) void walk_copy(const f4 *p, f4 *o, size_t slice_f4) {
    const f4 *base = p + (size_t)blockIdx.x * slice_f4;
    f4 *ob = o + (size_t)blockIdx.x * slice_f4;
    const size_t steps = slice_f4 / 256;
    for (size_t s = 0; s < steps; ++s) {
        const f4 *q = base + s * 256 + threadIdx.x;
        f4 a = q[0], b = q[64], c = q[128], d = q[192];
        f4 *w = ob + s * 256 + threadIdx.x;
        w[0] = a; w[64] = b; w[128] = c; w[192] = d;
    }
}
int main() {
    const size_t GiB = (size_t)1 << 30;
    f4 *buf, *other; float *sink;
    CK(hipMalloc(&buf, GiB)); CK(hipMalloc(&other, GiB)); CK(hipMalloc(&sink, 1 << 20));
    CK(hipMemset(buf, 1, GiB)); CK(hipMemset(other, 1, GiB));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int nwg = 2048;
    auto run = [&](const f4 *p, size_t bytes, int dir) {
        size_t slice = bytes / 16 / nwg;
        CK(hipEventRecord(e0));
        walk<<<nwg, 64>>>(p, slice, dir, sink);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1)); return ms;
    };
    // warm up clocks
    for (int i = 0; i < 20; ++i) run(other, GiB, 1);
    printf("size_MB cold_GBs warm_same_dir_GBs warm_opposite_dir_GBs\n");
    size_t sizes[] = {32, 64, 96, 128, 160, 192, 224, 256, 320, 384, 512, 768, 1024};
    for (size_t mb : sizes) {
        size_t bytes = mb << 20;
        float cold = 0, warm = 0, opp = 0; const int reps = 5;
        for (int r = 0; r < reps; ++r) {
            run(other, GiB, 1);                 // evict
            cold += run(buf, bytes, 1);
            warm += run(buf, bytes, 1);
            run(other, GiB, 1);
            run(buf, bytes, 1);
            opp += run(buf, bytes, -1);
        }
        printf("%6zu %8.0f %8.0f %8.0f\n", mb, bytes / (cold / reps) / 1e6, bytes / (warm / reps) / 1e6, bytes / (opp / reps) / 1e6);
        fflush(stdout);
    }
    // read after write: copy 'other'->buf region then read buf
    for (size_t mb : {64, 128, 192, 256, 512}) {
        size_t bytes = mb << 20; size_t slice = bytes / 16 / nwg; float t = 0, tc = 0;
        for (int r = 0; r < 5; ++r) {
            run(other + (GiB / 32), GiB / 2, 1);
            CK(hipEventRecord(e0));
            walk_copy<<<nwg, 64>>>(other, buf, slice);
            CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
            float ms; CK(hipEventElapsedTime(&ms, e0, e1)); tc += ms;
            t += run(buf, bytes, 1);
        }
        printf("copy %zu MB: copy %.0f GB/s (r+w), read-after-write %.0f GB/s\n", mb, 2.0 * bytes / (tc / 5) / 1e6, bytes / (t / 5) / 1e6);
        fflush(stdout);
    }
    return 0;
}
