// A torch-free client of the C ABI: device memory from hipMalloc, inputs from a small
// generator, one causal forward + backward through include/la.h, compared on the host with
// the fp64 oracle (linked as a C library).  Built by __graft_entry__.build(), run by
// tests/test_gpu_c_client.py.  Prints the four relative errors; exit status 0 iff all <= tol.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "la.h"

extern "C" {
void la_oracle_causal_fwd_prefix(const double *Q, const double *K, const double *V, double *O,
                                 double *den, int BH, int N, int D, int M, double eps);
void la_oracle_causal_bwd_linear(const double *Q, const double *K, const double *V, const double *G,
                                 double *dQ, double *dK, double *dV, int BH, int N, int D, int M,
                                 double eps);
}

#define HIP_OK(call)                                                                   \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess) {                                                        \
            std::fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));            \
            return 2;                                                                  \
        }                                                                              \
    } while (0)

// uniform in [-2, 2) from a 64-bit LCG (values exactly representable in fp32)
static float next_value(unsigned long long &s) {
    s = s * 6364136223846793005ULL + 1442695040888963407ULL;
    return (float)((long long)(s >> 40) - (1LL << 23)) / (float)(1 << 22);
}

static double max_abs(const std::vector<double> &x) {
    double m = 0.0;
    for (double v : x) m = std::fmax(m, std::fabs(v));
    return m;
}

// max|got - ref| / max(max|ref|, floor)
static double rel_err(const std::vector<float> &got, const std::vector<double> &ref, double floor) {
    double num = 0.0;
    for (size_t i = 0; i < ref.size(); ++i) num = std::fmax(num, std::fabs((double)got[i] - ref[i]));
    return num / std::fmax(std::fmax(max_abs(ref), floor), 1e-300);
}

int main(int argc, char **argv) {
    const int B = 2, H = 3, N = argc > 1 ? std::atoi(argv[1]) : 1234, D = 64, M = 64;
    const float eps = 1e-6f;
    const size_t rows = (size_t)B * H * N;
    unsigned long long seed = 20061623ULL;
    std::vector<float> hQ(rows * D), hK(rows * D), hV(rows * M), hG(rows * M);
    for (auto *v : {&hQ, &hK, &hV, &hG})
        for (float &x : *v) x = next_value(seed);

    float *Q, *K, *V, *G, *O, *den, *dQ, *dK, *dV;
    void *wsf = nullptr, *wsb = nullptr;
    const size_t nf = la_causal_fwd_workspace(B, H, N, D, M, LA_F32);
    const size_t nb = la_causal_bwd_workspace(B, H, N, D, M, LA_F32);
    HIP_OK(hipMalloc((void **)&Q, rows * D * 4)); HIP_OK(hipMalloc((void **)&K, rows * D * 4));
    HIP_OK(hipMalloc((void **)&V, rows * M * 4)); HIP_OK(hipMalloc((void **)&G, rows * M * 4));
    HIP_OK(hipMalloc((void **)&O, rows * M * 4)); HIP_OK(hipMalloc((void **)&den, rows * 4));
    HIP_OK(hipMalloc((void **)&dQ, rows * D * 4)); HIP_OK(hipMalloc((void **)&dK, rows * D * 4));
    HIP_OK(hipMalloc((void **)&dV, rows * M * 4));
    if (nf) HIP_OK(hipMalloc(&wsf, nf));
    HIP_OK(hipMalloc(&wsb, nb));
    HIP_OK(hipMemcpy(Q, hQ.data(), rows * D * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(K, hK.data(), rows * D * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(V, hV.data(), rows * M * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(G, hG.data(), rows * M * 4, hipMemcpyHostToDevice));

    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    int st = la_causal_fwd(Q, K, V, O, den, B, H, N, D, M, eps, LA_F32, wsf, nf, stream);
    if (st == LA_OK)
        st = la_causal_bwd(Q, K, V, nullptr, den, wsf, G, dQ, dK, dV, B, H, N, D, M, eps, LA_F32,
                           wsb, nb, stream);
    if (st != LA_OK) {
        std::fprintf(stderr, "library call failed: %s\n", la_status_string(st));
        return 3;
    }
    HIP_OK(hipStreamSynchronize(stream));
    std::vector<float> gO(rows * M), gdQ(rows * D), gdK(rows * D), gdV(rows * M);
    HIP_OK(hipMemcpy(gO.data(), O, rows * M * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gdQ.data(), dQ, rows * D * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gdK.data(), dK, rows * D * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gdV.data(), dV, rows * M * 4, hipMemcpyDeviceToHost));

    std::vector<double> q(hQ.begin(), hQ.end()), k(hK.begin(), hK.end()), v(hV.begin(), hV.end()),
        g(hG.begin(), hG.end());
    std::vector<double> rO(rows * M), rden(rows), rdQ(rows * D), rdK(rows * D), rdV(rows * M);
    la_oracle_causal_fwd_prefix(q.data(), k.data(), v.data(), rO.data(), rden.data(), B * H, N, D, M, eps);
    la_oracle_causal_bwd_linear(q.data(), k.data(), v.data(), g.data(), rdQ.data(), rdK.data(),
                                rdV.data(), B * H, N, D, M, eps);
    // each gradient is scaled by its own largest entry, but by no less than 1e-3 of the largest
    // of the three (dQ, dK vanish by cancellation for very short sequences)
    const double gfloor = 1e-3 * std::fmax(max_abs(rdQ), std::fmax(max_abs(rdK), max_abs(rdV)));
    const double e[4] = {rel_err(gO, rO, 0.0), rel_err(gdQ, rdQ, gfloor), rel_err(gdK, rdK, gfloor),
                         rel_err(gdV, rdV, gfloor)};
    std::printf("O %.3e dQ %.3e dK %.3e dV %.3e\n", e[0], e[1], e[2], e[3]);
    const double tol = N <= 4096 ? 1e-4 : 1e-3;
    for (double x : e)
        if (!(x <= tol)) return 1;
    return 0;
}
