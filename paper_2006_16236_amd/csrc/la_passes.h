// Chunked causal products on fp32 MFMA, one wavefront per (sequence, segment).
//
// The causal forward (paper eq. 9-12) and the three gradients of Algorithm 1
// (eq. 13-15) are all the same operation on different operands,
//
//     out_a = sum_{b <= a} (X_a . Y_b) Z_b            (b >= a for the reverse passes)
//           = mask(X Y^T) Z  restricted to the chunk  +  X_a U,
//     U     = sum over the tokens before (after) the chunk of Y_b^T Z_b,
//
// with 16-token chunks: the masked 16x16 block of X Y^T is a dense contraction
// and so is the product with the carried state U, which stays in accumulator
// registers for the whole segment (it is the S_i of eq. 10, or the reverse sum
// of eq. 14-15, sampled at chunk borders).
//
//   pass      X            Y            Z            U (rows x cols)      direction
//   kFwd      phi(Q)       phi(K)       V            S      D x M         forward
//   kDq       dO/den       V            phi(K)       S^T    M x D         forward
//   kDv       phi(K)       phi(Q)       dO/den       R      D x M         reverse
//   kDk       V            dO/den       phi(Q)       R^T    M x D         reverse
//   kGlobal   phi(Q)       -            -            total  D x M         (read-out only, eq. 5-6)
//
// The denominator of eq. 12 rides along as the "ones column" of the values:
//   kFwd  also carries z = sum phi(K_b) and forms den_a = rowsum(mask(XY^T)) + X_a.z + eps;
//   kDq   adds delta_a to every kept entry of X Y^T and delta_a * z to the state term,
//         delta_a = -(dO_a . O_a)/den_a being the gradient that reaches den_a;
//   kDk   adds delta_b to every kept entry and carries rho = sum delta_b phi(Q_b).
// kDq and kDk finish with the chain rule through phi (times phi'(Q), phi'(K)).
#pragma once

#include "la_device.h"

namespace la {

enum Pass { kFwd = 0, kDq = 1, kDv = 2, kDk = 3, kGlobal = 4 };

// floats per carried state in the workspace: the D x M matrix (row-major [D][M])
// followed by the D-vector that belongs to the ones column (z or rho).
__host__ __device__ constexpr int state_stride(int D, int M) { return D * M + D; }

struct PassArgs {
    const void *Q, *K, *V, *G;   // raw tensors, [BH, N, D] / [BH, N, M]
    const float *rden;           // [BH, N] 1/den_i             (backward passes)
    const float *delta;          // [BH, N] -(dO_i.O_i)/den_i   (backward passes)
    void *out;                   // [BH, N, DZ]
    float *den;                  // [BH, N] or null             (kFwd)
    const float *state;          // [BH, nseg, state_stride] exclusive states; null = zero state
    int N, nseg, chunks_per_seg;
    float eps;
};

template <int PASS, int D, int M, typename T>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(2))) void causal_pass_kernel(const PassArgs a) {
    constexpr bool kXisD = (PASS == kFwd || PASS == kDv || PASS == kGlobal);
    constexpr int DX = kXisD ? D : M;     // contraction width of X . Y and of X . U
    constexpr int DZ = kXisD ? M : D;     // width of Z, of the output and of U's columns
    constexpr int XT = DX / 16, ZT = DZ / 16;
    constexpr bool kReverse = (PASS == kDv || PASS == kDk);

    const int lane = threadIdx.x, c = lane & 15, g = lane >> 4;
    const int seg = blockIdx.x % a.nseg, bh = blockIdx.x / a.nseg;
    const int nchunks = (a.N + kChunk - 1) / kChunk;
    const int ch_begin = seg * a.chunks_per_seg;
    const int ch_end = min(ch_begin + a.chunks_per_seg, nchunks);

    const size_t rowbase = (size_t)bh * a.N;
    const T *Qs = static_cast<const T *>(a.Q) + rowbase * D;
    const T *Ks = static_cast<const T *>(a.K) + rowbase * D;
    const T *Vs = static_cast<const T *>(a.V) + rowbase * M;
    const T *Gs = static_cast<const T *>(a.G) + rowbase * M;
    const float *rden = a.rden + rowbase;
    const float *delta = a.delta + rowbase;
    T *outs = static_cast<T *>(a.out) + rowbase * DZ;

    // ---- carried state --------------------------------------------------------------------
    f32x4 U[XT][ZT];
    float zg[XT][4];   // kFwd/kGlobal: z[16xt + 4g + r]  (lines up with the token-lane X)
    float ec[ZT];      // kDq: z[16zt + c];  kDk: rho[16zt + c]  (lines up with the output)
#pragma unroll
    for (int xt = 0; xt < XT; ++xt) {
#pragma unroll
        for (int zt = 0; zt < ZT; ++zt) U[xt][zt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) zg[xt][r] = 0.f;
    }
#pragma unroll
    for (int zt = 0; zt < ZT; ++zt) ec[zt] = 0.f;

    if (a.state != nullptr) {
        const float *st = a.state +
                          ((size_t)bh * a.nseg + (PASS == kGlobal ? 0 : seg)) * state_stride(D, M);
#pragma unroll
        for (int xt = 0; xt < XT; ++xt)
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt) {
                if constexpr (kXisD) {        // U[d][m], d = 16xt + 4g + r, m = 16zt + c
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        U[xt][zt][r] = st[(16 * xt + 4 * g + r) * M + 16 * zt + c];
                } else {                      // U[m][d] = S[d][m], m = 16xt + 4g + r, d = 16zt + c
                    U[xt][zt] = load4(st + (16 * zt + c) * M + 16 * xt + 4 * g);
                }
            }
        if constexpr (PASS == kFwd || PASS == kGlobal) {
#pragma unroll
            for (int xt = 0; xt < XT; ++xt) {
                const f32x4 v = load4(st + D * M + 16 * xt + 4 * g);
#pragma unroll
                for (int r = 0; r < 4; ++r) zg[xt][r] = v[r];
            }
        }
        if constexpr (PASS == kDq || PASS == kDk) {
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt) ec[zt] = st[D * M + 16 * zt + c];
        }
    }

    for (int it = 0; it < ch_end - ch_begin; ++it) {
        const int ch = kReverse ? ch_end - 1 - it : ch_begin + it;
        const int t0 = ch * kChunk;
        const int nvalid = min(kChunk, a.N - t0);
        const bool tok_ok = c < nvalid;

        float xa[XT][4];                 // X, token-lane
        float ya[XT][4];                 // Y, token-lane
        float yf[XT][4];                 // Y, feature-lane
        float zf[ZT][4];                 // Z, feature-lane
        float raw[ZT][4];                // raw Q or K under the output, for phi'
        float sc1 = 0.f, dl1 = 0.f;      // per-token scalars of token c
        float sc4[4] = {0.f, 0.f, 0.f, 0.f}, dl4[4] = {0.f, 0.f, 0.f, 0.f};   // of tokens 4g + s

        // ---- fetch and prepare the chunk's operands ---------------------------------------
        if constexpr (PASS == kFwd || PASS == kGlobal) {
            load_token_lane<D>(Qs + (size_t)t0 * D, nvalid, c, g, xa);
#pragma unroll
            for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                for (int r = 0; r < 4; ++r) xa[xt][r] = tok_ok ? phi(xa[xt][r]) : 0.f;
        }
        if constexpr (PASS == kFwd) {
            load_token_lane<D>(Ks + (size_t)t0 * D, nvalid, c, g, ya);
            load_feature_lane<D>(Ks + (size_t)t0 * D, nvalid, c, g, yf);
            load_feature_lane<M>(Vs + (size_t)t0 * M, nvalid, c, g, zf);
#pragma unroll
            for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    ya[xt][r] = tok_ok ? phi(ya[xt][r]) : 0.f;
                    yf[xt][r] = (4 * g + r) < nvalid ? phi(yf[xt][r]) : 0.f;
                }
        }
        if constexpr (PASS == kDq) {
            sc1 = tok_ok ? rden[t0 + c] : 0.f;
            dl1 = tok_ok ? delta[t0 + c] : 0.f;
            load_rows4(delta + t0, nvalid, g, dl4);
            load_token_lane<M>(Gs + (size_t)t0 * M, nvalid, c, g, xa);
            load_token_lane<M>(Vs + (size_t)t0 * M, nvalid, c, g, ya);
            load_feature_lane<M>(Vs + (size_t)t0 * M, nvalid, c, g, yf);
            load_feature_lane<D>(Ks + (size_t)t0 * D, nvalid, c, g, zf);
            load_feature_lane<D>(Qs + (size_t)t0 * D, nvalid, c, g, raw);
#pragma unroll
            for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                for (int r = 0; r < 4; ++r) xa[xt][r] *= sc1;
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt)
#pragma unroll
                for (int s = 0; s < 4; ++s) zf[zt][s] = (4 * g + s) < nvalid ? phi(zf[zt][s]) : 0.f;
        }
        if constexpr (PASS == kDv) {
            load_rows4(rden + t0, nvalid, g, sc4);
            load_token_lane<D>(Ks + (size_t)t0 * D, nvalid, c, g, xa);
            load_token_lane<D>(Qs + (size_t)t0 * D, nvalid, c, g, ya);
            load_feature_lane<D>(Qs + (size_t)t0 * D, nvalid, c, g, yf);
            load_feature_lane<M>(Gs + (size_t)t0 * M, nvalid, c, g, zf);
#pragma unroll
            for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    xa[xt][r] = tok_ok ? phi(xa[xt][r]) : 0.f;
                    ya[xt][r] = tok_ok ? phi(ya[xt][r]) : 0.f;
                    yf[xt][r] = (4 * g + r) < nvalid ? phi(yf[xt][r]) : 0.f;
                }
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt)
#pragma unroll
                for (int s = 0; s < 4; ++s) zf[zt][s] *= sc4[s];
        }
        if constexpr (PASS == kDk) {
            sc1 = tok_ok ? rden[t0 + c] : 0.f;
            load_rows4(rden + t0, nvalid, g, sc4);
            load_rows4(delta + t0, nvalid, g, dl4);
            load_token_lane<M>(Vs + (size_t)t0 * M, nvalid, c, g, xa);
            load_token_lane<M>(Gs + (size_t)t0 * M, nvalid, c, g, ya);
            load_feature_lane<M>(Gs + (size_t)t0 * M, nvalid, c, g, yf);
            load_feature_lane<D>(Qs + (size_t)t0 * D, nvalid, c, g, zf);
            load_feature_lane<D>(Ks + (size_t)t0 * D, nvalid, c, g, raw);
#pragma unroll
            for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    ya[xt][r] *= sc1;
                    yf[xt][r] *= sc4[r];
                }
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt)
#pragma unroll
                for (int s = 0; s < 4; ++s) zf[zt][s] = (4 * g + s) < nvalid ? phi(zf[zt][s]) : 0.f;
        }

        // ---- state term: out = X U  (lane (c, g), register r: token 4g + r, column 16zt + c)
        f32x4 out[ZT];
#pragma unroll
        for (int zt = 0; zt < ZT; ++zt) out[zt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int xt = 0; xt < XT; ++xt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt) out[zt] = mfma16(xa[xt][r], U[xt][zt][r], out[zt]);

        float den_a = 1.0f;              // kFwd / kGlobal: denominator of token c
        if constexpr (PASS == kGlobal) {
            float p = 0.f;
#pragma unroll
            for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                for (int r = 0; r < 4; ++r) p = fmaf(xa[xt][r], zg[xt][r], p);
            den_a = sum_over_groups(p) + a.eps;
        } else {
            // ---- W[a][b] = X_a . Y_b, lane (c = a, g), register r: b = 4g + r --------------
            f32x4 w0 = {0.f, 0.f, 0.f, 0.f}, w1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int xt = 0; xt < XT; xt += 2)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    w0 = mfma16(ya[xt][r], xa[xt][r], w0);
                    w1 = mfma16(ya[xt + 1][r], xa[xt + 1][r], w1);
                }
            f32x4 w;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = w0[r] + w1[r];
                if constexpr (PASS == kDq) v += dl1;
                if constexpr (PASS == kDk) v += dl4[r];
                const bool keep = kReverse ? (4 * g + r) >= c : (4 * g + r) <= c;
                w[r] = keep ? v : 0.f;               // select, never multiply: no NaN leaks
            }
            if constexpr (PASS == kFwd) {
                float p = (w[0] + w[1]) + (w[2] + w[3]);
#pragma unroll
                for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) p = fmaf(xa[xt][r], zg[xt][r], p);
                den_a = sum_over_groups(p) + a.eps;
            }
            // ---- in-chunk term: out += W Z -------------------------------------------------
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt) out[zt] = mfma16(w[s], zf[zt][s], out[zt]);
        }

        // ---- finish and store ---------------------------------------------------------------
        if constexpr (PASS == kFwd || PASS == kGlobal) {
            const float rinv = tok_ok ? 1.0f / den_a : 0.f;
            if constexpr (PASS == kFwd) {
                if (a.den != nullptr && g == 0 && tok_ok) a.den[rowbase + t0 + c] = den_a;
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float ri = __shfl(rinv, 4 * g + r);
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt) out[zt][r] *= ri;
            }
        }
        if constexpr (PASS == kDq) {
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    out[zt][r] = fmaf(dl4[r], ec[zt], out[zt][r]) * dphi(raw[zt][r]);
        }
        if constexpr (PASS == kDk) {
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt)
#pragma unroll
                for (int r = 0; r < 4; ++r) out[zt][r] = (out[zt][r] + ec[zt]) * dphi(raw[zt][r]);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 4 * g + r;
            if (row < nvalid) {
                T *p = outs + (size_t)(t0 + row) * DZ + c;
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt) store_elem(p + 16 * zt, out[zt][r]);
            }
        }

        // ---- carry: U += Y^T Z, and the ones-column vector --------------------------------
        if constexpr (PASS != kGlobal) {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                    for (int zt = 0; zt < ZT; ++zt)
                        U[xt][zt] = mfma16(yf[xt][s], zf[zt][s], U[xt][zt]);
        }
        if constexpr (PASS == kFwd) {
#pragma unroll
            for (int xt = 0; xt < XT; ++xt) {
                const float zc = sum_over_groups((yf[xt][0] + yf[xt][1]) + (yf[xt][2] + yf[xt][3]));
#pragma unroll
                for (int r = 0; r < 4; ++r) zg[xt][r] += __shfl(zc, 4 * g + r);
            }
        }
        if constexpr (PASS == kDq) {
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt)
                ec[zt] += sum_over_groups((zf[zt][0] + zf[zt][1]) + (zf[zt][2] + zf[zt][3]));
        }
        if constexpr (PASS == kDk) {
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt) {
                float p = dl4[0] * zf[zt][0];
#pragma unroll
                for (int s = 1; s < 4; ++s) p = fmaf(dl4[s], zf[zt][s], p);
                ec[zt] += sum_over_groups(p);
            }
        }
    }
}

// ---- per-segment totals (first phase of the segment scan) ---------------------------------
// KIND 0: S = sum phi(K_b)^T V_b,      z   = sum phi(K_b)            (eq. 10-11 over a segment)
// KIND 1: R = sum phi(Q_b)^T dO_b/den, rho = sum delta_b phi(Q_b)    (eq. 14-15 over a segment)
// Written as [D][M] row-major followed by the D-vector.
struct SegArgs {
    const void *Y;        // K or Q  [BH, N, D]
    const void *Z;        // V or dO [BH, N, M]
    const float *rden;    // KIND 1
    const float *delta;   // KIND 1
    float *state;         // [BH, nseg, state_stride]
    int N, nseg, chunks_per_seg;
    int skip_seg;         // segment whose total nobody reads (-1: none)
};

template <int KIND, int D, int M, typename T>
__global__ __launch_bounds__(kWave) void segment_state_kernel(const SegArgs a) {
    constexpr int XT = D / 16, ZT = M / 16;
    const int lane = threadIdx.x, c = lane & 15, g = lane >> 4;
    const int seg = blockIdx.x % a.nseg, bh = blockIdx.x / a.nseg;
    if (seg == a.skip_seg) return;
    const int nchunks = (a.N + kChunk - 1) / kChunk;
    const int ch_begin = seg * a.chunks_per_seg;
    const int ch_end = min(ch_begin + a.chunks_per_seg, nchunks);
    const size_t rowbase = (size_t)bh * a.N;
    const T *Ys = static_cast<const T *>(a.Y) + rowbase * D;
    const T *Zs = static_cast<const T *>(a.Z) + rowbase * M;

    f32x4 U[XT][ZT];
    float ec[XT];
#pragma unroll
    for (int xt = 0; xt < XT; ++xt) {
        ec[xt] = 0.f;
#pragma unroll
        for (int zt = 0; zt < ZT; ++zt) U[xt][zt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    for (int ch = ch_begin; ch < ch_end; ++ch) {
        const int t0 = ch * kChunk;
        const int nvalid = min(kChunk, a.N - t0);
        float yf[XT][4], zf[ZT][4];
        float w4[4] = {1.f, 1.f, 1.f, 1.f};
        load_feature_lane<D>(Ys + (size_t)t0 * D, nvalid, c, g, yf);
        load_feature_lane<M>(Zs + (size_t)t0 * M, nvalid, c, g, zf);
#pragma unroll
        for (int xt = 0; xt < XT; ++xt)
#pragma unroll
            for (int s = 0; s < 4; ++s) yf[xt][s] = (4 * g + s) < nvalid ? phi(yf[xt][s]) : 0.f;
        if constexpr (KIND == 1) {
            float sc4[4];
            load_rows4(a.rden + rowbase + t0, nvalid, g, sc4);
            load_rows4(a.delta + rowbase + t0, nvalid, g, w4);
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt)
#pragma unroll
                for (int s = 0; s < 4; ++s) zf[zt][s] *= sc4[s];
        }
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt) U[xt][zt] = mfma16(yf[xt][s], zf[zt][s], U[xt][zt]);
#pragma unroll
        for (int xt = 0; xt < XT; ++xt)
#pragma unroll
            for (int s = 0; s < 4; ++s) ec[xt] = fmaf(w4[s], yf[xt][s], ec[xt]);
    }
    float *st = a.state + ((size_t)bh * a.nseg + seg) * state_stride(D, M);
#pragma unroll
    for (int xt = 0; xt < XT; ++xt) {
#pragma unroll
        for (int zt = 0; zt < ZT; ++zt)
#pragma unroll
            for (int r = 0; r < 4; ++r) st[(16 * xt + 4 * g + r) * M + 16 * zt + c] = U[xt][zt][r];
        const float e = sum_over_groups(ec[xt]);
        if (g == 0) st[D * M + 16 * xt + c] = e;
    }
}

}  // namespace la
