// Small bandwidth-bound kernels: the scan over segment states and the recurrent
// decode step (eq. 16-20).
#include "la_launch.h"

namespace la {

// ---- scan over the segment states of each sequence ------------------------------------------
// state: [BH, nseg, stride], stride a multiple of 4.  A thread owns four consecutive elements
// (16-byte loads and stores); a workgroup takes 4 * 256 / PARTS consecutive elements of one
// sequence, and its PARTS groups of threads split the nseg slots into PARTS consecutive runs.
// Each group first sums its run (all loads independent), the run totals are exchanged through
// LDS, then the group walks its run again (now from cache) and writes the exclusive prefix.
// Slots are visited in scan order: ascending for the prefix, descending for the suffix.
// Fixed order: deterministic.  PARTS grows with nseg (1 for a handful of slots: every thread
// then has elements of its own and no thread idles).
template <int PARTS>
__global__ __launch_bounds__(256) void scan_states_kernel(float *state, int nseg, int stride,
                                                          int mode, const float *init_S,
                                                          const float *init_z, int DM) {
    constexpr int EPW = 256 / PARTS;          // threads (quads of elements) per run
    __shared__ f32x4 part_total[PARTS][EPW];
    const int el = threadIdx.x % EPW, part = threadIdx.x / EPW;
    const int e = 4 * (blockIdx.x * EPW + el);
    const bool live = e < stride;
    float *p = state + (size_t)blockIdx.y * nseg * stride + (live ? e : 0);
    const bool reverse = mode == kScanReverse;
    const int per = (nseg + PARTS - 1) / PARTS;
    const int k0 = min(part * per, nseg), k1 = min(k0 + per, nseg);
    // the last slot in scan order holds no total (nobody reads past it): never read it
    const int klast = mode == kScanTotal ? nseg : nseg - 1;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    auto slot = [&](const int k) { return reinterpret_cast<f32x4 *>(p + (size_t)(reverse ? nseg - 1 - k : k) * stride); };

    // eight independent loads in flight per thread (a plain loop waits for each in turn)
    constexpr int kBlock = 8;
    const int kread = min(k1, klast);
    f32x4 total = zero4;
    for (int kb = k0; kb < kread; kb += kBlock) {
        f32x4 t[kBlock];
#pragma unroll
        for (int j = 0; j < kBlock; ++j) t[j] = *slot(min(kb + j, kread - 1));
#pragma unroll
        for (int j = 0; j < kBlock; ++j) total += kb + j < kread ? t[j] : zero4;
    }
    // the scan starts from the caller's initial state when there is one (forward prefix only)
    f32x4 acc = zero4;
    if (init_S != nullptr && live)
        acc = e < DM ? *reinterpret_cast<const f32x4 *>(init_S + (size_t)blockIdx.y * DM + e)
                     : *reinterpret_cast<const f32x4 *>(init_z + (size_t)blockIdx.y * (stride - DM) + (e - DM));
    if constexpr (PARTS > 1) {
        part_total[part][el] = total;
        __syncthreads();
        for (int q = 0; q < part; ++q) acc += part_total[q][el];
    }
    if (mode == kScanTotal) {
        if (part == PARTS - 1 && live) *reinterpret_cast<f32x4 *>(p) = acc + total;
        return;
    }
    for (int kb = k0; kb < k1; kb += kBlock) {
        f32x4 t[kBlock];
#pragma unroll
        for (int j = 0; j < kBlock; ++j) {
            const int k = min(kb + j, k1 - 1);
            t[j] = k < klast ? *slot(k) : zero4;
        }
#pragma unroll
        for (int j = 0; j < kBlock; ++j) {
            const int k = kb + j;
            if (k < k1) {
                if (live) *slot(k) = acc;
                acc += t[j];
            }
        }
    }
}

hipError_t launch_scan(float *state, int BH, int nseg, int stride, int mode, hipStream_t s,
                       const float *init_S, const float *init_z, int DM) {
    const int quads = (stride + 3) / 4;
    if (nseg <= 4) {
        dim3 grid((quads + 255) / 256, BH);
        scan_states_kernel<1><<<grid, 256, 0, s>>>(state, nseg, stride, mode, init_S, init_z, DM);
    } else if (nseg <= 16) {
        dim3 grid((quads + 127) / 128, BH);
        scan_states_kernel<2><<<grid, 256, 0, s>>>(state, nseg, stride, mode, init_S, init_z, DM);
    } else if (nseg <= 32) {
        dim3 grid((quads + 63) / 64, BH);
        scan_states_kernel<4><<<grid, 256, 0, s>>>(state, nseg, stride, mode, init_S, init_z, DM);
    } else {
        dim3 grid((quads + 31) / 32, BH);
        scan_states_kernel<8><<<grid, 256, 0, s>>>(state, nseg, stride, mode, init_S, init_z, DM);
    }
    return hipGetLastError();
}

// feature d of one token's q or k: eq. 7 of element d, the element itself when the caller has
// applied the map, or x_i x_j with 8i + j = d for the degree-2 polynomial map (section 3.2)
template <typename T> __device__ __forceinline__ float feature_of(const T *row, int d) {
    if constexpr (is_poly<T>) return to_f32(row[d >> 3]) * to_f32(row[d & 7]);
    else return feature<T>(to_f32(row[d]));
}

// ---- recurrent decode step (eq. 16-20) -------------------------------------------------------
// One workgroup of four waves per head.  Every lane owns four adjacent columns of
// S; M/4 lanes cover a row, a wave covers 256/M rows per iteration.  The rank-1
// update, the z update and the read-out run in one sweep over S (read once,
// written once); the column sums are combined by wave shuffles, then across the
// four waves through LDS.  Fixed order everywhere: bit-identical run to run.
template <int D, int M, typename T>
__global__ __launch_bounds__(256) void recurrent_step_kernel(const T *q, const T *k, const T *v,
                                                             float *S, float *z, T *out,
                                                             float eps) {
    constexpr int LPR = M / 4;            // lanes per row of S
    constexpr int RPW = kWave / LPR;      // rows per wave per iteration
    constexpr int RPI = 4 * RPW;          // rows per workgroup per iteration
    static_assert(D % RPI == 0, "D must be a multiple of the rows swept per iteration");
    __shared__ float red[4][M];
    __shared__ float dred[4];

    const int bh = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col4 = (lane % LPR) * 4, rsub = lane / LPR;
    constexpr int W = qk_width<T>(D);          // elements per token of q and k
    const T *qh = q + (size_t)bh * W, *kh = k + (size_t)bh * W;
    float *Sh = S + (size_t)bh * D * M, *zh = z + (size_t)bh * D;

    const f32x4 v4 = load4(v + (size_t)bh * M + col4);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float dpart = 0.f;
#pragma unroll
    for (int it = 0; it < D / RPI; ++it) {
        const int d = it * RPI + wave * RPW + rsub;
        const float kd = feature_of<T>(kh, d);
        const float qd = feature_of<T>(qh, d);
        f32x4 s4 = *reinterpret_cast<f32x4 *>(Sh + (size_t)d * M + col4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            s4[e] = fmaf(kd, v4[e], s4[e]);          // eq. 18
            acc[e] = fmaf(qd, s4[e], acc[e]);
        }
        *reinterpret_cast<f32x4 *>(Sh + (size_t)d * M + col4) = s4;
        if (col4 == 0) {
            const float zn = zh[d] + kd;             // eq. 19
            zh[d] = zn;
            dpart = fmaf(qd, zn, dpart);
        }
    }
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += __shfl_xor(acc[e], off);
    }
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) dpart += __shfl_xor(dpart, off);
    if (rsub == 0) {
#pragma unroll
        for (int e = 0; e < 4; ++e) red[wave][col4 + e] = acc[e];
    }
    if (lane == 0) dred[wave] = dpart;
    __syncthreads();
    if (tid < M) {
        const float num = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
        const float den = ((dred[0] + dred[1]) + (dred[2] + dred[3])) + eps;
        store_elem(out + (size_t)bh * M + tid, num / den);     // eq. 20 (the fraction)
    }
}

// T consecutive decode steps in one launch, for callers that already hold the q, k, v of
// all T tokens (scoring, teacher forcing): the state stays in registers between steps, the
// next token's q, k, v are fetched while the current one is processed.  The arithmetic of a
// step, lane for lane, is that of recurrent_step_kernel: T steps here and T launches of
// the single step give bit-identical outputs and states.
template <int D, int M, typename T>
__global__ __launch_bounds__(256) void recurrent_steps_kernel(const T *q, const T *k, const T *v,
                                                              float *S, float *z, T *out,
                                                              float eps, int steps, size_t BH) {
    constexpr int LPR = M / 4, RPW = kWave / LPR, RPI = 4 * RPW, NIT = D / RPI;
    __shared__ float red[2][4][M];
    __shared__ float dred[2][4];

    const int bh = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col4 = (lane % LPR) * 4, rsub = lane / LPR;
    float *Sh = S + (size_t)bh * D * M, *zh = z + (size_t)bh * D;

    f32x4 s4[NIT];
    float zr[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int d = it * RPI + wave * RPW + rsub;
        s4[it] = *reinterpret_cast<const f32x4 *>(Sh + (size_t)d * M + col4);
        zr[it] = zh[d];
    }
    constexpr int W = qk_width<T>(D);          // elements per token of q and k
    // The wave sweeps NR rows of S per step, and every lane of a row needs that row's feature of
    // k and of q.  The feature map is evaluated once per row and wave, not once per lane: lane
    // j < NR fetches and maps k's element of row j of the sweep, lane NR + j the same of q (the
    // lanes above 2 NR repeat them, unused), and the lanes of a row pick the values up with a
    // shuffle.  The values are those every lane computed for itself before, bit for bit.
    constexpr int NR = NIT * RPW;
    static_assert(2 * NR <= kWave, "one lane per row and operand");
    const int j = lane % NR;
    const bool mine_is_q = ((lane / NR) & 1) != 0;
    const int dj = (j / RPW) * RPI + wave * RPW + (j % RPW);
    auto fetch = [&](int t, float &x, f32x4 &v4) {
        const T *row = (mine_is_q ? q : k) + ((size_t)t * BH + bh) * W;
        if constexpr (is_poly<T>) x = feature_of<T>(row, dj);   // the feature itself (x_i x_j): nothing is left to map
        else x = to_f32(row[dj]);
        v4 = load4(v + ((size_t)t * BH + bh) * M + col4);
    };
    float x_next;
    f32x4 v_next;
    fetch(0, x_next, v_next);
    for (int t = 0; t < steps; ++t) {
        const float f = feature<T>(x_next);
        const f32x4 v4 = v_next;
        if (t + 1 < steps) fetch(t + 1, x_next, v_next);

        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        float dpart = 0.f;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const float kd = __shfl(f, it * RPW + rsub);
            const float qd = __shfl(f, NR + it * RPW + rsub);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                s4[it][e] = fmaf(kd, v4[e], s4[it][e]);
                acc[e] = fmaf(qd, s4[it][e], acc[e]);
            }
            if (col4 == 0) {
                zr[it] += kd;
                dpart = fmaf(qd, zr[it], dpart);
            }
        }
#pragma unroll
        for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] += __shfl_xor(acc[e], off);
        }
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) dpart += __shfl_xor(dpart, off);
        const int buf = t & 1;            // two LDS buffers: one barrier per step suffices
        if (rsub == 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) red[buf][wave][col4 + e] = acc[e];
        }
        if (lane == 0) dred[buf][wave] = dpart;
        __syncthreads();
        if (tid < M) {
            const float num = (red[buf][0][tid] + red[buf][1][tid]) + (red[buf][2][tid] + red[buf][3][tid]);
            const float den = ((dred[buf][0] + dred[buf][1]) + (dred[buf][2] + dred[buf][3])) + eps;
            store_elem(out + ((size_t)t * BH + bh) * M + tid, num / den);
        }
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int d = it * RPI + wave * RPW + rsub;
        *reinterpret_cast<f32x4 *>(Sh + (size_t)d * M + col4) = s4[it];
        if (col4 == 0) zh[d] = zr[it];
    }
}

hipError_t launch_recurrent_steps(const void *q, const void *k, const void *v, float *S, float *z,
                                  void *out, int steps, int BH, int D, int M, float eps, int dtype,
                                  hipStream_t s) {
    LA_DISPATCH(D, M, dtype, {
        recurrent_steps_kernel<kD, kM, TT><<<BH, 256, 0, s>>>((const TT *)q, (const TT *)k,
                                                             (const TT *)v, S, z, (TT *)out, eps,
                                                             steps, (size_t)BH);
    });
    return hipGetLastError();
}

hipError_t launch_recurrent_step(const void *q, const void *k, const void *v, float *S, float *z,
                                 void *out, int BH, int D, int M, float eps, int dtype,
                                 hipStream_t s) {
    LA_DISPATCH(D, M, dtype, {
        recurrent_step_kernel<kD, kM, TT><<<BH, 256, 0, s>>>((const TT *)q, (const TT *)k,
                                                            (const TT *)v, S, z, (TT *)out, eps);
    });
    return hipGetLastError();
}

}  // namespace la
