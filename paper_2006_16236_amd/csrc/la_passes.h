// Chunked causal products on the matrix units.  For fp32 tensors the products run on the fp32
// MFMA or, where one operand quad feeds several products, on the bf16 MFMA with exactly split
// operands (split3 in la_device.h).  For bf16 tensors the forward passes use plain bf16 products
// and the backward passes (and the segment sums they start from) 16-bit operands in two parts.
// The forward runs one wavefront per (sequence, segment); the two kernels of the backward run
// two wavefronts per (sequence, segment) that share one fetch of the inputs.
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
// Without the causal mask (eq. 4-6) both sums run over the whole sequence, so the gradients
// are read-outs against the two grand totals, with no in-chunk part and no carried update:
//   kGlobalDq dO/den       -            -            total S^T            delta as in kDq, then times phi'(Q)
//   kGlobalDv phi(K)       -            -            total R
//   kGlobalDk V            -            -            total R^T            plus rho, then times phi'(K)
//
// The denominator of eq. 12 rides along as the "ones column" of the values:
//   kFwd  also carries z = sum phi(K_b) and forms den_a = rowsum(mask(XY^T)) + X_a.z + eps;
//   kDq   needs delta_a = -(dO_a . O_a)/den_a, the gradient that reaches den_a.  It does not
//         read O for it: with A_a = S_a dO_a/den_a (its own result before the ones column is
//         added) dO_a . O_a = phi(Q_a) . A_a, so delta_a = -(phi(Q_a) . A_a)/den_a.  Then
//         dphi(Q)_a = A_a + delta_a z_a with z_a = z + the in-chunk running sum of phi(K)
//         (one more product against the constant lower-triangular mask).  delta and 1/den
//         are written out for the reverse passes;
//   kDk   adds delta_b to every kept entry and carries rho = sum delta_b phi(Q_b).
// kDq and kDk finish with the chain rule through phi (times phi'(Q), phi'(K)).
//
// Data movement per chunk: every input tile (16 tokens x 32|64 features) is fetched
// once with fully coalesced 16-byte loads into staging registers while the previous
// chunk is being computed, then mapped (phi, phi', 1/den scaling, zero fill of rows past
// the end of the sequence) and parked in LDS as fp32, from where the MFMA operands are read in
// whichever of the two layouts of la_device.h each product needs.
#pragma once

#include <type_traits>

#include "la_device.h"

#ifndef LA_SPLIT_SUMS
#define LA_SPLIT_SUMS 1          // 0: every fp32 product on the fp32 MFMA (for comparison)
#endif
#ifndef LA_GLOBAL_DEPTH
#define LA_GLOBAL_DEPTH(T) 1     // chunks in flight per wave in the non-causal passes (1 or 2)
#endif
// Issue priority (s_setprio, 0..3) of the two waves of the two-wave kernels.  Measured: in the
// reverse kernel the dK wave, which borrows the state through LDS every chunk, is the one the
// chunk waits for; letting it issue first takes 3.5 % off the kernel timed between events
// (0.358 -> 0.346 ms) and 0.5-1 % off the whole step (1.016 -> 1.011 ms, a second box 1.040 ->
// 1.027 ms, wall clock over back-to-back steps).  In the
// dQ kernel neither choice helps (state wave first: 0.328 against 0.323 ms), nor in the two-wave
// kernels of the non-causal backward and of bf16 tensors (tried, within noise; not kept).
#ifndef LA_PRIO_DQ_CHUNK_WAVE
#define LA_PRIO_DQ_CHUNK_WAVE 0
#endif
#ifndef LA_PRIO_DQ_STATE_WAVE
#define LA_PRIO_DQ_STATE_WAVE 0
#endif
#ifndef LA_PRIO_REV_DV_WAVE
#define LA_PRIO_REV_DV_WAVE 0
#endif
#ifndef LA_PRIO_REV_DK_WAVE
#define LA_PRIO_REV_DK_WAVE 3
#endif
#ifndef LA_SLEEP_AFTER_FETCH
#define LA_SLEEP_AFTER_FETCH 1   // in units of 64 clocks
#endif

namespace la {

enum Pass { kFwd = 0, kDq = 1, kDv = 2, kDk = 3, kGlobal = 4, kGlobalDq = 5, kGlobalDv = 6, kGlobalDk = 7 };

// the causal pass whose operand roles a read-out-only pass shares
__host__ __device__ constexpr int base_pass(int p) {
    return p == kGlobal ? kFwd : p == kGlobalDq ? kDq : p == kGlobalDv ? kDv : p == kGlobalDk ? kDk : p;
}

// floats per carried state in the workspace: the D x M matrix (row-major [D][M])
// followed by the D-vector that belongs to the ones column (z or rho).
__host__ __device__ constexpr int state_stride(int D, int M) { return D * M + D; }

struct PassArgs {
    const void *Q, *K, *V, *G;   // raw tensors, [BH, N, D] / [BH, N, M]
    const float *rden;           // [BH, N] 1/den_i             (reverse passes; written by the dQ pass)
    const float *delta;          // [BH, N] -(dO_i.O_i)/den_i   (reverse passes; written by the dQ pass)
    void *out;                   // [BH, N, DZ]  (reverse_pass_kernel: dV; kFwd, kGlobal: may be null,
                                 // the pass then only writes the denominators)
    void *out2;                  // reverse_pass_kernel only: dK [BH, N, D]
    float *den;                  // [BH, N] or null             (kFwd, kGlobal)
    const float *den_in;         // kDq: the forward's denominators [BH, N]
    float *rden_out, *delta_out; // kDq: [BH, N] 1/den_i and delta_i for the reverse passes (or both null)
    float *totals;               // kDq: [BH, nseg, state_stride] per-segment sums of
                                 // phi(Q)^T dO/den and delta phi(Q), or null
    const float *state;          // [BH, nseg, state_stride] exclusive states; null = zero state
    // `state` may have been laid out for a finer cut: state_nseg segments per sequence (0: nseg),
    // of which this pass's segment `seg` starts at segment seg * state_step (0: step 1)
    int state_nseg, state_step;
    // fold = 0: every slot of `state` holds a finished sum (the scan kernel has run): a pass reads
    //           the one slot it starts from;
    // fold = 1: the slots hold per-segment totals and each pass adds up the ones before (after)
    //           its segment itself, in slot order.  Pays when a sequence has few segments: one
    //           launch and one sweep over the states less.
    int fold;
    // State at the end a pass starts from, used when the sequences are not cut (nseg == 1),
    // [BH, D, M] / [BH, D], may be null: kFwd, kDq the sums before token 0; kDv (matrix) and
    // kDk (vector) the gradient that arrives at the state after the last token.
    const float *init_S, *init_z;
    // kFwd: state after the last token; kDv / kDk: gradient for the state before token 0.
    float *final_S, *final_z;      // same shapes; may be null
    int N, nseg, chunks_per_seg;
    float eps;
    // Layout of the [., N, .] tensors (Q, K, V, dO and the outputs; not the [BH, N] scalars):
    // tok_heads <= 1: [B, H, N, F], every sequence contiguous (kernels with kStrided = false);
    // tok_heads = H = heads: [B, N, H, F], consecutive tokens of a sequence H * F elements
    // apart (kernels with kStrided = true).
    int heads, tok_heads;
    // 1: the tiles are fetched with non-temporal loads (every element is touched once per kernel
    // and need not stay in the caches); 0, the host's default: plain loads, so that a later kernel
    // of the same step finds in the last-level cache what fits there.
    int stream;
};

// element offset of token 0 of sequence bh in a tensor of row width F, and the distance
// between consecutive tokens, for the two layouts
// (kStrided is a template parameter of the kernels: the contiguous layout keeps compile-time
// strides, which matters for the instruction-bound bf16 kernels)
template <bool kStrided>
__device__ __forceinline__ size_t seq_base(int N, int heads, int bh, int F) {
    if constexpr (!kStrided) return (size_t)bh * N * F;
    else return ((size_t)(bh / heads) * N * heads + (size_t)(bh % heads)) * F;
}
template <bool kStrided>
__device__ __forceinline__ int tok_stride(int tok_heads, int F) {
    if constexpr (!kStrided) return F;
    else return tok_heads * F;
}

// Which slots of a sequence's state array a pass adds up to get the sum it starts from:
// the tokens before its segment, the tokens after it, or all of them.
enum StateKind { kStatePrefix = 0, kStateSuffix = 1, kStateTotal = 2 };
__device__ __forceinline__ void state_slots(const PassArgs &a, const int seg, const int kind,
                                            int &nslots, int &lo, int &hi) {
    nslots = a.state_nseg != 0 ? a.state_nseg : a.nseg;
    const int at = seg * (a.state_step != 0 ? a.state_step : 1);
    if (a.fold == 0) {
        lo = kind == kStateTotal ? 0 : at;
        hi = lo + 1;
    } else if (kind == kStatePrefix) {
        lo = 0, hi = at;
    } else if (kind == kStateSuffix) {
        lo = at + 1, hi = nslots;
    } else {
        lo = 0, hi = nslots;
    }
}

enum Map { kMapId = 0, kMapPhi = 1, kMapDphi = 2, kMapScale = 3, kMapOne = 4, kMapFinite = 5 };

// kMapFinite: the value itself, with +-Inf and NaN replaced by finite values (one instruction:
// the median of (v, -big, big), which returns the smallest operand when one is a NaN; big is the
// largest finite bf16, so that it survives the operand packing of every element type).  It is
// the map of V in the causal forward: the in-chunk term adds mask(scores)_ab V_b over the whole
// 16-token tile, masked entries being exact zeros, and 0 * Inf would carry a non-finite value of
// token b back to the tokens before it.  The scores need no such care: they are masked by a
// select on the product's result.
template <int MAP>
__device__ __forceinline__ float map_value(float v, float scale) {
    if constexpr (MAP == kMapPhi) return phi(v);
    if constexpr (MAP == kMapDphi) return dphi(v);
    if constexpr (MAP == kMapScale) return v * scale;
    if constexpr (MAP == kMapOne) return 1.0f;
    if constexpr (MAP == kMapFinite) return __builtin_amdgcn_fmed3f(v, -3.3895314e38f, 3.3895314e38f);
    return v;
}

// Which passes of a bf16 call run their tile products as plain bf16 products (operands rounded
// to 8 significant bits): the forward ones, kFwd and kGlobal.  The backward passes carry every
// operand to 16 bits (two bf16 parts, see run_pass): their results are differences of nearly equal
// terms (dphi(Q)_a = A_a + delta_a z_a vanishes for constant V; R v + rho likewise), and with
// features phi(x) = 1 + x + ... of small x an 8-bit mantissa of the operands would cost up to
// 1.5e-2 of the gradient's scale (measured on inputs scaled by 1/8; worse for smaller inputs),
// too close to the 2e-2 gate.
template <int PASS, typename T>
constexpr bool bf16_products = is_bf16<T> && (PASS == kFwd || PASS == kGlobal);

// Park a staged tile in LDS: apply the map; kFull = false also zeroes the rows past the end
// of the sequence.  The parked values stay fp32 for every element type: a pass that multiplies
// on the bf16 MFMA rounds them when it packs its operands.
// kFeat (the caller has applied the feature map): phi becomes the identity, phi' becomes 1.
template <int F, int MAP_, bool kFull, bool kFeat, typename ST>
__device__ __forceinline__ void park_tile(float *tile, const ST (&st)[F / 16],
                                          const float (&scale)[F / 16], int nvalid, int lane) {
    constexpr int MAP = !kFeat ? MAP_ : MAP_ == kMapPhi ? kMapId : MAP_ == kMapDphi ? kMapOne : MAP_;
#pragma unroll
    for (int i = 0; i < F / 16; ++i) {
        const int row = stage_row<F>(lane, i);
        const f32x4 w = widen(st[i]);
        f32x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float m = map_value<MAP>(w[r], scale[i]);
            v[r] = (kFull || row < nvalid) ? m : 0.0f;
        }
        lds_store4(tile + row * tile_stride(F) + stage_col<F>(lane, i), v);
    }
}

// A 16 x F output tile from the MFMA layout (lane (c, g), out[zt][r]: token 4g + r, column
// 16zt + c) to memory through one LDS tile private to the calling wave: written as it is, read
// back so that a lane holds consecutive columns of one token (four fp32, or eight values that
// are rounded to bf16 in pairs) and stored 16 bytes per lane.  A wave instruction then writes
// whole rows (F = 64: four tokens of 256 bytes, or eight of 128 bytes for bf16) where
// element-wise stores write 64-byte (bf16: 32-byte) pieces, one element per lane.
// `tile_out` points at column 0 of the tile's first token, `tso` is the token stride in elements.
template <int F, typename T>
__device__ __forceinline__ void store_tile(float *lds_o, const f32x4 (&out)[F / 16], T *tile_out,
                                           const int tso, const int nvalid, const int lane) {
    const int c = lane & 15, g = lane >> 4;
#pragma unroll
    for (int zt = 0; zt < F / 16; ++zt)
#pragma unroll
        for (int r = 0; r < 4; ++r) lds_o[(4 * g + r) * tile_stride(F) + 16 * zt + c] = out[zt][r];
    constexpr int kPerLane = is_bf16<T> ? 8 : 4;                  // elements per 16-byte store
    constexpr int kLanesPerRow = F / kPerLane, kRowsPerStore = kWave / kLanesPerRow;
#pragma unroll
    for (int h = 0; h < kChunk / kRowsPerStore; ++h) {
        const int row = h * kRowsPerStore + lane / kLanesPerRow, col = kPerLane * (lane % kLanesPerRow);
        const f32x4 lo = *reinterpret_cast<const f32x4 *>(lds_o + row * tile_stride(F) + col);
        if constexpr (is_bf16<T>) {
            const f32x4 hi = *reinterpret_cast<const f32x4 *>(lds_o + row * tile_stride(F) + col + 4);
            const u32x4_t packed = {round_pair(lo[0], lo[1]), round_pair(lo[2], lo[3]),
                                    round_pair(hi[0], hi[1]), round_pair(hi[2], hi[3])};
            if (row < nvalid) *reinterpret_cast<u32x4_t *>(tile_out + (size_t)row * tso + col) = packed;
        } else {
            static_assert(sizeof(T) == 4, "fp32 element types");
            f32x4 *p = reinterpret_cast<f32x4 *>(tile_out + (size_t)row * tso + col);
            if (row < nvalid) {
                if constexpr (LA_NT_STORES != 0) __builtin_nontemporal_store(lo, p);
                else *p = lo;
            }
        }
    }
}

// Which raw tensor feeds which operand of a pass, and how it is mapped when parked.
template <int PASS, int D, int M>
struct PassTraits {
    static constexpr int BP = base_pass(PASS);
    static constexpr bool kXisD = (BP == kFwd || BP == kDv);
    static constexpr int DX = kXisD ? D : M;     // contraction width of X . Y and of X . U
    static constexpr int DZ = kXisD ? M : D;     // width of Z, of the output and of U's columns
    static constexpr bool kReverse = (PASS == kDv || PASS == kDk);
    static constexpr bool kHasRaw = (BP == kDq || BP == kDk);         // phi' under the output
    static constexpr bool kHasYZ = (PASS < kGlobal);                  // false: read-out only
    static constexpr int kMapX = (BP == kDq) ? kMapScale : (BP == kDk) ? kMapId : kMapPhi;
    static constexpr int kMapY = (PASS == kDq) ? kMapId : (PASS == kDk) ? kMapScale : kMapPhi;
    static constexpr int kMapZ = (PASS == kFwd) ? kMapFinite : (PASS == kDv) ? kMapScale : kMapPhi;
};

// Staging of a pass run by one wave on its own (kFwd and the read-out-only passes kGlobal,
// kGlobalDv, kGlobalDk): the wave fetches and parks all its tiles.
template <int PASS, int D, int M, typename T, bool kStrided = false, int kDepth_ = 1>
struct PassStager {
    static constexpr bool kStridedLayout = kStrided;
    using Tr = PassTraits<PASS, D, M>;
    static_assert(PASS == kFwd || PASS == kGlobal || PASS == kGlobalDv || PASS == kGlobalDk,
                  "the other passes have stagers of their own");
    static constexpr int DX = Tr::DX, DZ = Tr::DZ, XT = DX / 16, ZT = DZ / 16;
    // X is phi(Q) (kFwd, kGlobal) or phi(K) (kGlobalDv): a Q / K tensor (qk_width elements per
    // token, expanded on fetch for the polynomial map); otherwise it is V
    static constexpr bool kXqk = (Tr::BP == kFwd || Tr::BP == kDv);
    const T *Xs, *Ys, *Zs, *Rs;
    float *lds_x, *lds_y, *lds_z, *lds_r;
    int N, lane;
    bool nt;                            // non-temporal fetches (PassArgs::stream)
    int tsx, tsy, tsz, tsr;             // token strides of X, of K as Y, of V as Z, of K under the output
    static constexpr int kDepth = kDepth_;    // chunks in flight = sets of staging registers (1 or 2)
    staged_t<T> sx[kDepth][XT], sy[kDepth][XT], sz[kDepth][ZT], sr[kDepth][ZT];
    float onex[XT], onez[ZT];
    float dl1, dl4[4];                  // unused by these passes (interface of run_pass)
    float xraw[kPolyRaw], n_xraw[kDepth][kPolyRaw];   // polynomial map, kGlobalDk: raw K of token lane / 4

    __device__ __forceinline__ PassStager(const PassArgs &a, int bh, int lane_, float *lx,
                                          float *ly, float *lz, float *lr)
        : lds_x(lx), lds_y(ly), lds_z(lz), lds_r(lr), N(a.N), lane(lane_), nt(a.stream != 0) {
        constexpr int BP = Tr::BP;
        constexpr int wx = kXqk ? qk_width<T>(DX) : DX, wy = qk_width<T>(DX), wr = qk_width<T>(DZ);
        tsx = tok_stride<kStrided>(a.tok_heads, wx);
        tsy = tok_stride<kStrided>(a.tok_heads, wy);
        tsz = tok_stride<kStrided>(a.tok_heads, DZ);
        tsr = tok_stride<kStrided>(a.tok_heads, wr);
        Xs = static_cast<const T *>(BP == kFwd ? a.Q : BP == kDv ? a.K : a.V) + seq_base<kStrided>(a.N, a.heads, bh, wx);
        Ys = static_cast<const T *>(a.K) + seq_base<kStrided>(a.N, a.heads, bh, wy);      // kFwd
        Zs = static_cast<const T *>(a.V) + seq_base<kStrided>(a.N, a.heads, bh, DZ);      // kFwd
        Rs = static_cast<const T *>(a.K) + seq_base<kStrided>(a.N, a.heads, bh, wr);      // kGlobalDk
        dl1 = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) dl4[s] = 0.f;
#pragma unroll
        for (int i = 0; i < XT; ++i) onex[i] = 1.0f;
#pragma unroll
        for (int i = 0; i < ZT; ++i) onez[i] = 1.0f;
#pragma unroll
        for (int j = 0; j < kPolyRaw; ++j) {
            xraw[j] = 0.f;
#pragma unroll
            for (int k = 0; k < kDepth; ++k) n_xraw[k][j] = 0.f;
        }
    }

    template <int SLOT, bool kFull, bool kNt>
    __device__ __forceinline__ void fetch_impl(const int t0, const int nvalid) {
        if constexpr (kXqk) stage_load_qk<DX, kFull, kNt>(Xs + (size_t)t0 * tsx, tsx, nvalid, lane, sx[SLOT]);
        else stage_load<DX, kFull, kNt>(Xs + (size_t)t0 * tsx, tsx, nvalid, lane, sx[SLOT]);
        if constexpr (Tr::kHasYZ) {
            stage_load_qk<DX, kFull, kNt>(Ys + (size_t)t0 * tsy, tsy, nvalid, lane, sy[SLOT]);
            stage_load<DZ, kFull, kNt>(Zs + (size_t)t0 * tsz, tsz, nvalid, lane, sz[SLOT]);
        }
        if constexpr (Tr::kHasRaw) {
            if constexpr (is_poly<T>) load_raw8(Rs + (size_t)t0 * tsr, tsr, nvalid, lane, n_xraw[SLOT]);
            else stage_load<DZ, kFull, kNt>(Rs + (size_t)t0 * tsr, tsr, nvalid, lane, sr[SLOT]);
        }
    }

    template <int SLOT>
    __device__ __forceinline__ void fetch(const int ch) {
        const int t0 = ch * kChunk;
        const int nvalid = min(kChunk, N - t0);
        if (nt) {                            // uniform branches
            if (nvalid == kChunk) fetch_impl<SLOT, true, true>(t0, nvalid);
            else fetch_impl<SLOT, false, true>(t0, nvalid);
        } else {
            if (nvalid == kChunk) fetch_impl<SLOT, true, false>(t0, nvalid);
            else fetch_impl<SLOT, false, false>(t0, nvalid);
        }
    }

    template <int SLOT, bool kFull>
    __device__ __forceinline__ void park_impl(const int nvalid) {
        park_tile<DX, Tr::kMapX, kFull, is_feat<T>>(lds_x, sx[SLOT], onex, nvalid, lane);
        if constexpr (Tr::kHasYZ) {
            park_tile<DX, Tr::kMapY, kFull, is_feat<T>>(lds_y, sy[SLOT], onex, nvalid, lane);
            park_tile<DZ, Tr::kMapZ, kFull, is_feat<T>>(lds_z, sz[SLOT], onez, nvalid, lane);
        }
        if constexpr (Tr::kHasRaw) {
            if constexpr (is_poly<T>) {       // lds_r serves as the scratch of poly2_chain instead
#pragma unroll
                for (int j = 0; j < kPolyRaw; ++j) xraw[j] = n_xraw[SLOT][j];
            } else {
                park_tile<DZ, kMapDphi, kFull, is_feat<T>>(lds_r, sr[SLOT], onez, nvalid, lane);
            }
        }
    }

    template <int SLOT>
    __device__ __forceinline__ void park(const int nvalid) {
        if (nvalid == kChunk) park_impl<SLOT, true>(nvalid);
        else park_impl<SLOT, false>(nvalid);
    }
};

// Staging of the two reverse passes run side by side by the two waves of one workgroup:
// the four input tiles are fetched once and shared.  Wave 0 (the kDv role) brings Q and
// dO, wave 1 (the kDk role) brings K (parked twice, as phi and as phi') and V.
template <int ROLE, int D, int M, typename T, bool kStrided = false>
struct ReverseStager {
    static constexpr bool kStridedLayout = kStrided;
    static constexpr int DT = D / 16, MT = M / 16;
    static constexpr int kDepth = 1;    // chunks in flight = sets of staging registers (1 or 2)
    const T *As, *Bs;                   // role 0: Q, dO; role 1: K, V
    const float *rden, *delta;
    float *lds_a, *lds_a2, *lds_b;      // role 0: phi(Q), -, dO/den; role 1: phi(K), phi'(K), V
    int N, lane, g;
    bool nt;                            // non-temporal fetches (PassArgs::stream)
    int tsd, tsm;                       // token strides of the D-wide and M-wide tensors
    staged_t<T> sa[kDepth][DT], sb[kDepth][MT];
    float scd[DT], scb[kDepth][MT];
    float n_dl4[kDepth][4];
    float dl1, dl4[4];
    float xraw[kPolyRaw], n_xraw[kDepth][kPolyRaw];   // polynomial map, role 1: raw K of token lane / 4

    __device__ __forceinline__ ReverseStager(const PassArgs &a, int bh, int lane_, float *la,
                                             float *la2, float *lb)
        : lds_a(la), lds_a2(la2), lds_b(lb), N(a.N), lane(lane_), g(lane_ >> 4), nt(a.stream != 0),
          tsd(tok_stride<kStrided>(a.tok_heads, qk_width<T>(D))), tsm(tok_stride<kStrided>(a.tok_heads, M)) {
        const size_t rowbase = (size_t)bh * a.N;
        As = static_cast<const T *>(ROLE == 0 ? a.Q : a.K) + seq_base<kStrided>(a.N, a.heads, bh, qk_width<T>(D));
#pragma unroll
        for (int j = 0; j < kPolyRaw; ++j) {
            xraw[j] = 0.f;
#pragma unroll
            for (int k = 0; k < kDepth; ++k) n_xraw[k][j] = 0.f;
        }
        Bs = static_cast<const T *>(ROLE == 0 ? a.G : a.V) + seq_base<kStrided>(a.N, a.heads, bh, M);
        rden = a.rden + rowbase;
        delta = a.delta + rowbase;
        dl1 = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) dl4[s] = 0.f;
#pragma unroll
        for (int i = 0; i < DT; ++i) scd[i] = 1.0f;
#pragma unroll
        for (int k = 0; k < kDepth; ++k) {
#pragma unroll
            for (int s = 0; s < 4; ++s) n_dl4[k][s] = 0.f;
#pragma unroll
            for (int i = 0; i < MT; ++i) scb[k][i] = 1.0f;
        }
    }

    template <int SLOT, bool kFull, bool kNt>
    __device__ __forceinline__ void fetch_impl(const int t0, const int nvalid) {
        stage_load_qk<D, kFull, kNt>(As + (size_t)t0 * tsd, tsd, nvalid, lane, sa[SLOT]);
        stage_load<M, kFull, kNt>(Bs + (size_t)t0 * tsm, tsm, nvalid, lane, sb[SLOT]);
        if constexpr (ROLE == 0) stage_rows<M, kFull>(rden + t0, nvalid, lane, scb[SLOT]);
        else rows4<kFull>(delta + t0, nvalid, g, n_dl4[SLOT]);
        if constexpr (ROLE == 1 && is_poly<T>) load_raw8(As + (size_t)t0 * tsd, tsd, nvalid, lane, n_xraw[SLOT]);
    }

    template <int SLOT>
    __device__ __forceinline__ void fetch(const int ch) {
        const int t0 = ch * kChunk;
        const int nvalid = min(kChunk, N - t0);
        if (nt) {                            // uniform branches
            if (nvalid == kChunk) fetch_impl<SLOT, true, true>(t0, nvalid);
            else fetch_impl<SLOT, false, true>(t0, nvalid);
        } else {
            if (nvalid == kChunk) fetch_impl<SLOT, true, false>(t0, nvalid);
            else fetch_impl<SLOT, false, false>(t0, nvalid);
        }
    }

    template <int SLOT, bool kFull>
    __device__ __forceinline__ void park_impl(const int nvalid) {
        park_tile<D, kMapPhi, kFull, is_feat<T>>(lds_a, sa[SLOT], scd, nvalid, lane);
        if constexpr (ROLE == 0) {
            park_tile<M, kMapScale, kFull, is_feat<T>>(lds_b, sb[SLOT], scb[SLOT], nvalid, lane);
        } else {
            // (polynomial map: there is no phi' tile; lds_a2 is the scratch of poly2_chain)
            if constexpr (!is_poly<T>) park_tile<D, kMapDphi, kFull, is_feat<T>>(lds_a2, sa[SLOT], scd, nvalid, lane);
            park_tile<M, kMapId, kFull, is_feat<T>>(lds_b, sb[SLOT], scb[SLOT], nvalid, lane);
        }
    }

    template <int SLOT>
    __device__ __forceinline__ void park(const int nvalid) {
        if (nvalid == kChunk) park_impl<SLOT, true>(nvalid);
        else park_impl<SLOT, false>(nvalid);
#pragma unroll
        for (int s = 0; s < 4; ++s) dl4[s] = n_dl4[SLOT][s];
        if constexpr (ROLE == 1 && is_poly<T>) {
#pragma unroll
            for (int j = 0; j < kPolyRaw; ++j) xraw[j] = n_xraw[SLOT][j];
        }
    }
};

// One pass over the chunks [ch_begin, ch_end) of sequence bh by the calling wave.  `stg`
// fetches the next chunk and parks the current one; lds_* are the parked tiles this pass
// reads its operands from (they may be shared with the other wave of the workgroup).
//
// kStateMode: kOwnState    the wave carries U in its accumulators (the usual case);
//             kPublishState as kOwnState, and before each chunk it also writes U to `lds_u` for the
//                          other wave of the workgroup (layout [column][row], stride rows + 4);
//             kBorrowState  the wave keeps no U of its own: each chunk it reads the partner's U from
//                          `lds_u` as its own TRANSPOSE (this wave's U is the partner's U^T), and
//                          skips the update.  Only its ones-column vector is its own.
enum StateMode { kOwnState = 0, kPublishState = 1, kBorrowState = 2 };

template <int PASS, int D, int M, typename T, int kStateMode = kOwnState, typename Stager>
__device__ __forceinline__ void run_pass(const PassArgs &a, Stager &stg, const float *lds_x,
                                         const float *lds_y, const float *lds_z,
                                         const float *lds_r, void *out_tensor, const int bh,
                                         const int seg, const int lane, float *lds_u = nullptr,
                                         float *lds_scratch = nullptr, float *lds_o = nullptr) {
    // lds_scratch: polynomial map, passes that end in a gradient for Q or K: one tile
    // (16 x tile_stride(64) floats) private to the calling wave, for poly2_chain
    // lds_o: one tile (16 x tile_stride(DZ) floats) private to the calling wave, through which
    // the output tile is stored (store_tile); nullptr: element-wise stores
    using Tr = PassTraits<PASS, D, M>;
    constexpr bool kXisD = Tr::kXisD;
    constexpr int DX = Tr::DX, DZ = Tr::DZ;
    constexpr int XT = DX / 16, ZT = DZ / 16;
    constexpr bool kReverse = Tr::kReverse;
    constexpr bool kHasRaw = Tr::kHasRaw;
    constexpr bool kHasYZ = Tr::kHasYZ;
    // bf16 tensors, forward passes: the tile products run on the bf16 MFMA (operands rounded to
    // bf16, fp32 accumulation); the sums that ride on MFMAs against ones stay fp32
    constexpr bool kBf = bf16_products<PASS, T>;
    // fp32 products whose operands are tile values shared by several products (the in-chunk
    // term, the running sum inside the chunk, the update of U) run on split bf16 operands, to
    // fp32 accuracy (see split3); the products against U itself and the scores stay on the fp32
    // MFMA: splitting their operands would cost more than it saves.
    constexpr bool kSplit = !kBf && (LA_SPLIT_SUMS != 0);
    // bf16 tensors (backward passes; the forward ones are kBf): the results are rounded to 8
    // significant bits, so 16-bit operands (two parts) are ample, and at 12 vector instructions
    // per quad the split then pays for the state operand of the read-out as well
    constexpr int kParts = is_bf16<T> ? 2 : 3;
    constexpr bool kSplitState = kSplit && is_bf16<T>;

    const int c = lane & 15, g = lane >> 4;
    const int nchunks = (a.N + kChunk - 1) / kChunk;
    const int ch_begin = seg * a.chunks_per_seg;
    const int ch_end = min(ch_begin + a.chunks_per_seg, nchunks);
    const int count = ch_end - ch_begin;
    const size_t rowbase = (size_t)bh * a.N;
    constexpr bool kStrided = Stager::kStridedLayout;
    // width of the output tensor: DZ, or the raw width when the output is a gradient for Q or K
    // of the polynomial map
    constexpr bool kRawGrad = is_poly<T> && (Tr::BP == kDq || Tr::BP == kDk);
    constexpr int WO = kRawGrad ? qk_width<T>(DZ) : DZ;
    const int tso = tok_stride<kStrided>(a.tok_heads, WO);
    T *outs = static_cast<T *>(out_tensor) + seq_base<kStrided>(a.N, a.heads, bh, WO);

    // ---- carried state --------------------------------------------------------------------
    f32x4 U[XT][ZT];
    f32x4 zg[XT];      // kFwd/kGlobal: z[16xt + 4g + r]  (lines up with the token-lane X)
    float ecp[ZT];     // kDq: z[16zt + c], kDk: rho[16zt + c], as per-lane partial sums: the
                       // four lanes (c, g = 0..3) together hold the value (an MFMA adds them up)
    float rho[ZT];     // kDq: this segment's sum of delta_b phi(Q_b)[16zt + c], same partial form
#pragma unroll
    for (int xt = 0; xt < XT; ++xt) {
#pragma unroll
        for (int zt = 0; zt < ZT; ++zt) U[xt][zt] = f32x4{0.f, 0.f, 0.f, 0.f};
        zg[xt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int zt = 0; zt < ZT; ++zt) ecp[zt] = rho[zt] = 0.f;

    // The sum the pass starts from: the caller's state at that end (if any) plus the slots of
    // the state array that state_slots() names (one finished sum, or the totals to add up).
    // sm: [D][M] matrix, sv: the D-vector of the ones column.
    auto add_state = [&](const float *sm, const float *sv) {
#pragma unroll
        for (int xt = 0; xt < XT; ++xt)
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt) {
                if constexpr (kStateMode == kBorrowState) continue;
                if constexpr (kXisD) {        // U[d][m], d = 16xt + 4g + r, m = 16zt + c
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        U[xt][zt][r] += sm[(16 * xt + 4 * g + r) * M + 16 * zt + c];
                } else {                      // U[m][d] = S[d][m], m = 16xt + 4g + r, d = 16zt + c
                    U[xt][zt] += load4_state(sm + (16 * zt + c) * M + 16 * xt + 4 * g);
                }
            }
        if constexpr (PASS == kFwd || PASS == kGlobal) {
#pragma unroll
            for (int xt = 0; xt < XT; ++xt) zg[xt] += load4_state(sv + 16 * xt + 4 * g);
        }
        if constexpr (Tr::BP == kDq || Tr::BP == kDk) {
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt) ecp[zt] += g == 0 ? sv[16 * zt + c] : 0.f;
        }
    };
    if constexpr (kHasYZ) {
        if (a.init_S != nullptr) add_state(a.init_S + (size_t)bh * D * M, a.init_z + (size_t)bh * D);
    }
    if (a.state != nullptr) {
        int nslots, lo, hi;
        state_slots(a, seg, !kHasYZ ? kStateTotal : kReverse ? kStateSuffix : kStatePrefix, nslots, lo, hi);
        for (int j = lo; j < hi; ++j) {
            const float *st = a.state + ((size_t)bh * nslots + j) * state_stride(D, M);
            add_state(st, st + D * M);
        }
    }

    // Read-out-only passes: U never changes, so it is cut into its bf16 parts (three for fp32
    // tensors, two for bf16 tensors) once, here, and every chunk's read-out runs on the bf16 pipe
    // (section on split3 in la_device.h); only the chunk's own operand is split per chunk.
    constexpr bool kConstState = !kHasYZ && kSplit;
    SplitA<kParts> us[XT][ZT];
    if constexpr (kConstState) {
#pragma unroll
        for (int xt = 0; xt < XT; ++xt)
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt) us[xt][zt] = split_a<kParts>(U[xt][zt]);
    }

    // Chunks are visited in steps of `dir`; the stager keeps kDepth chunks in flight, each in
    // its own set of staging registers (the set is a compile-time index, hence the tag).
    constexpr int kDepth = Stager::kDepth;
    constexpr int dir = kReverse ? -1 : 1;
    const int ch0 = kReverse ? ch_end - 1 : ch_begin;
    if (count > 0) stg.template fetch<0>(ch0);
    if constexpr (kDepth == 2) {
        if (count > 1) stg.template fetch<1>(ch0 + dir);
    }

    auto step = [&](auto slot_tag, const int it) {
        constexpr int kSlot = decltype(slot_tag)::value;
        const int ch = ch0 + dir * it;
        const int t0 = ch * kChunk;
        const int nvalid = min(kChunk, a.N - t0);

        // ---- park the staged chunk in LDS, refill its staging registers ---------------------
        __syncthreads();                 // every operand read of the previous chunk is done
        stg.template park<kSlot>(nvalid);
        const float dl1 = stg.dl1;
        const float dl4[4] = {stg.dl4[0], stg.dl4[1], stg.dl4[2], stg.dl4[3]};
        float rd4[4] = {0.f, 0.f, 0.f, 0.f};          // kDq: 1/den of tokens 4g + s (0 past the end)
        if constexpr (Tr::BP == kDq) {
#pragma unroll
            for (int s = 0; s < 4; ++s) rd4[s] = stg.rd4[s];
        }
        if (it + kDepth < count) stg.template fetch<kSlot>(ch + dir * kDepth);
        if constexpr (kStateMode == kPublishState) {
            // U as it stands before this chunk (the exclusive state), element (row 16xt + 4g + r,
            // column 16zt + c) at lds_u[column][row]: four rows per 16-byte write
#pragma unroll
            for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt)
                    lds_store4(lds_u + (16 * zt + c) * (DX + 4) + 16 * xt + 4 * g, U[xt][zt]);
        }
        // Let the loads leave the wave before the matrix instructions start: measured on
        // MI355X, a burst of MFMAs issued right behind a batch of global loads delays those
        // loads by the length of the burst (the chunk then arrives one iteration late).
        __builtin_amdgcn_s_sleep(LA_SLEEP_AFTER_FETCH);
        __builtin_amdgcn_sched_barrier(0);   // keep the prefetch ahead of the arithmetic
        __syncthreads();

        if constexpr (kStateMode == kBorrowState) {
            // this wave's U[row 16xt + 4g + r][column 16zt + c] is the partner's U[16zt + c][16xt + 4g + r],
            // parked at lds_u[partner column = 16xt + 4g + r][partner row = 16zt + c]
#pragma unroll
            for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        U[xt][zt][r] = lds_u[(16 * xt + 4 * g + r) * (DZ + 4) + 16 * zt + c];
        }

        // ---- state term: out = X U  (lane (c, g), register r: token 4g + r, column 16zt + c)
        float xa[XT][4];                 // X, token-lane
        lds_token_lane<DX>(lds_x, c, g, xa);
        f32x4 out[ZT];
#pragma unroll
        for (int zt = 0; zt < ZT; ++zt) out[zt] = f32x4{0.f, 0.f, 0.f, 0.f};
        bf16x4_t xp[XT];                 // X packed (bf16 path)
        Split2 x2[XT];                   // X in two parts (bf16 tensors, backward passes)
        // bf16 tensors, the dK passes: X is V itself, exact in bf16, and needs no second part
        constexpr bool kExactX = is_bf16<T> && Tr::BP == kDk;
        ExactBf16 xe[XT];
        if constexpr (kBf) {
#pragma unroll
            for (int xt = 0; xt < XT; ++xt) {
                xp[xt] = pack_bf16x4(xa[xt]);
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt)
                    out[zt] = mfma16_bf16(xp[xt], pack_bf16x4(U[xt][zt]), out[zt]);
            }
        } else if constexpr (kConstState) {
#pragma unroll
            for (int xt = 0; xt < XT; ++xt) {
                if constexpr (kExactX) {
                    xe[xt] = exact_bf16(xa[xt]);
#pragma unroll
                    for (int zt = 0; zt < ZT; ++zt) out[zt] = mfma16_split_ba(xe[xt], us[xt][zt], out[zt]);
                } else {
                    const SplitB<kParts> xs = split_b<kParts>(xa[xt]);
#pragma unroll
                    for (int zt = 0; zt < ZT; ++zt) out[zt] = mfma16_split_ba(xs, us[xt][zt], out[zt]);
                }
            }
        } else if constexpr (kSplitState) {
#pragma unroll
            for (int xt = 0; xt < XT; ++xt) {
                if constexpr (kExactX) {
                    xe[xt] = exact_bf16(xa[xt]);
#pragma unroll
                    for (int zt = 0; zt < ZT; ++zt)
                        out[zt] = mfma16_split(xe[xt], split_b<2>(U[xt][zt]), out[zt]);
                } else {
                    // the state quads, cut anew every chunk, take the narrow form (the wide one
                    // costs four register copies per quad), the tile quad the wide one
                    x2[xt] = split2(xa[xt]);
                    const SplitB<2> xs = as_b(x2[xt]);
#pragma unroll
                    for (int zt = 0; zt < ZT; ++zt) {
                        // The cut overwrites its input, and U must live on: a wave that has
                        // just published U cuts the copy in LDS (one 16-byte read per quad)
                        // instead of four register copies.  (Cutting the four quads of a row
                        // stage by stage, as the dQ kernel does, costs this kernel 24 registers
                        // and 2 % of its time.)
                        f32x4 uq = U[xt][zt];
                        if constexpr (kStateMode == kPublishState)
                            uq = *reinterpret_cast<const f32x4 *>(lds_u + (16 * zt + c) * (DX + 4) + 16 * xt + 4 * g);
                        out[zt] = mfma16_split_ba(xs, split_a<2>(uq), out[zt]);
                    }
                }
            }
        } else {
#pragma unroll
            for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int zt = 0; zt < ZT; ++zt)
                        out[zt] = mfma16(xa[xt][r], U[xt][zt][r], out[zt]);
        }

        // kFwd / kGlobal: den4[r] = denominator of token 4g + r.  Each lane (c = a, g) holds a
        // partial sum of token a's denominator; one MFMA against a matrix of ones adds the four
        // partials and lands the totals in the row layout of `out` (eps is the addend).
        f32x4 den4 = {1.f, 1.f, 1.f, 1.f};
        const f32x4 eps4 = {a.eps, a.eps, a.eps, a.eps};
        float zf[ZT][4];                 // Z, feature-lane
        bf16x4_t zp[ZT];                 // ... packed (bf16 path)
        SplitB<kParts> zs[ZT];           // ... split (fp32 on the bf16 pipe)
        if constexpr (!kHasYZ) {
            if constexpr (PASS == kGlobal) {
                float p = 0.f;
#pragma unroll
                for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) p = fmaf(xa[xt][r], zg[xt][r], p);
                den4 = mfma16(p, 1.0f, eps4);
            } else if constexpr (PASS == kGlobalDk) {
                // the ones-column part: rho (kGlobalDq adds its own further down)
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt) out[zt] = mfma16(1.0f, ecp[zt], out[zt]);
            }
        } else {
            // ---- W[a][b] = X_a . Y_b, lane (c = a, g), register r: b = 4g + r --------------
            float ya[XT][4];             // Y, token-lane
            lds_token_lane<DX>(lds_y, c, g, ya);
            f32x4 w0 = {0.f, 0.f, 0.f, 0.f}, w1 = {0.f, 0.f, 0.f, 0.f};
            // (never plain bf16 products: in the forward pass the row sums of the scores are the
            // in-chunk part of the denominator, and the backward divides by it)
            if constexpr (kSplitState) {
#pragma unroll
                for (int xt = 0; xt < XT; xt += 2) {
                    if constexpr (kExactX) {
                        w0 = mfma16_split(split_a<2>(ya[xt]), xe[xt], w0);
                        w1 = mfma16_split(split_a<2>(ya[xt + 1]), xe[xt + 1], w1);
                    } else {
                        w0 = mfma16_split(split_a<2>(ya[xt]), as_b(x2[xt]), w0);
                        w1 = mfma16_split(split_a<2>(ya[xt + 1]), as_b(x2[xt + 1]), w1);
                    }
                }
            } else if constexpr (kBf) {       // 16-bit operands: den is good to 2^-16
#pragma unroll
                for (int xt = 0; xt < XT; xt += 2) {
                    w0 = mfma16_split(split_a<2>(ya[xt]), split_b<2>(xa[xt]), w0);
                    w1 = mfma16_split(split_a<2>(ya[xt + 1]), split_b<2>(xa[xt + 1]), w1);
                }
            } else {
#pragma unroll
                for (int xt = 0; xt < XT; xt += 2)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        w0 = mfma16(ya[xt][r], xa[xt][r], w0);
                        w1 = mfma16(ya[xt + 1][r], xa[xt + 1][r], w1);
                    }
            }
            f32x4 w;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = w0[r] + w1[r];
                if constexpr (PASS == kDk) v += dl4[r];
                const bool keep = kReverse ? (4 * g + r) >= c : (4 * g + r) <= c;
                w[r] = keep ? v : 0.f;               // select, never multiply
            }
            if constexpr (PASS == kFwd) {
                float p = (w[0] + w[1]) + (w[2] + w[3]);
#pragma unroll
                for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) p = fmaf(xa[xt][r], zg[xt][r], p);
                den4 = mfma16(p, 1.0f, eps4);
            }
            // the ones-column part of the state term: rho (kDk; kDq adds its own further down)
            if constexpr (PASS == kDk) {
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt) out[zt] = mfma16(1.0f, ecp[zt], out[zt]);
            }
            // ---- in-chunk term: out += W Z -------------------------------------------------
            lds_feature_lane<DZ>(lds_z, c, g, zf);
            if constexpr (kBf) {
                const bf16x4_t wp = pack_bf16x4(w);
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt) {
                    zp[zt] = pack_bf16x4(zf[zt]);
                    out[zt] = mfma16_bf16(wp, zp[zt], out[zt]);
                }
            } else if constexpr (kSplit) {
                const float wq[4] = {w[0], w[1], w[2], w[3]};
                const SplitA<kParts> ws = split_a<kParts>(wq);
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt) {
                    zs[zt] = split_b<kParts>(zf[zt]);
                    out[zt] = mfma16_split(ws, zs[zt], out[zt]);
                }
            } else {
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int zt = 0; zt < ZT; ++zt) out[zt] = mfma16(w[s], zf[zt][s], out[zt]);
            }
        }

        // ---- finish and store ---------------------------------------------------------------
        if constexpr (PASS == kFwd || PASS == kGlobal) {
            {
                // lanes c < 4 of each group write den of token 4g + c: 16 consecutive floats
                const float dsel = c == 0 ? den4[0] : c == 1 ? den4[1] : c == 2 ? den4[2] : den4[3];
                if (a.den != nullptr && c < 4 && 4 * g + c < nvalid) a.den[rowbase + t0 + 4 * g + c] = dsel;
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float ri = __builtin_amdgcn_rcpf(den4[r]);
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt) out[zt][r] *= ri;
            }
        }
        if constexpr (Tr::BP == kDq) {
            // `out` is A_a = S_a dO_a/den_a so far (rows: tokens 4g + r, columns: features
            // 16zt + c).  delta_a = -(phi(Q_a) . A_a)/den_a: multiply by phi(Q) in the same
            // layout, add up the 16 lanes of the group and the ZT registers.
            float fq[ZT][4];
            lds_feature_lane<DZ>(lds_r, c, g, fq);
            float d4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float p = out[0][r] * fq[0][r];
#pragma unroll
                for (int zt = 1; zt < ZT; ++zt) p = fmaf(out[zt][r], fq[zt][r], p);
                d4[r] = -row_sum16(p) * rd4[r];
            }
            // z_a = z before the chunk (an MFMA against ones adds the four partial sums and
            // leaves the total in every register) + running sum of phi(K) up to token a (the
            // constant lower-triangular mask times the phi(K) tile)
            f32x4 cz[ZT];
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt) cz[zt] = mfma16(1.0f, ecp[zt], f32x4{0.f, 0.f, 0.f, 0.f});
            if constexpr (kHasYZ) {       // (kGlobalDq: z is the sum over the whole sequence)
                float m[4];
#pragma unroll
                for (int s = 0; s < 4; ++s) m[s] = (4 * g + s) <= c ? 1.0f : 0.0f;
                if constexpr (kBf) {
                    const bf16x4_t mp = pack_bf16x4(m);
#pragma unroll
                    for (int zt = 0; zt < ZT; ++zt) cz[zt] = mfma16_bf16(mp, zp[zt], cz[zt]);
                } else if constexpr (kSplit) {
                                        const u32x2_t mk = {(m[0] != 0.f ? 0x3f80u : 0u) | (m[1] != 0.f ? 0x3f800000u : 0u),
                                        (m[2] != 0.f ? 0x3f80u : 0u) | (m[3] != 0.f ? 0x3f800000u : 0u)};
#pragma unroll
                    for (int zt = 0; zt < ZT; ++zt) cz[zt] = mfma16_mask(mk, zs[zt], cz[zt]);
                } else {
#pragma unroll
                    for (int s = 0; s < 4; ++s)
#pragma unroll
                        for (int zt = 0; zt < ZT; ++zt) cz[zt] = mfma16(m[s], zf[zt][s], cz[zt]);
                }
            }
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt) {
                float rp = 0.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    rp = fmaf(d4[r], fq[zt][r], rp);
                    out[zt][r] = fmaf(d4[r], cz[zt][r], out[zt][r]) * feature_slope<T>(fq[zt][r]);
                }
                rho[zt] += rp;
            }
            // lanes c < 4 of each group write 1/den and delta of token 4g + c
            const float dsel = c == 0 ? d4[0] : c == 1 ? d4[1] : c == 2 ? d4[2] : d4[3];
            const float rsel = c == 0 ? rd4[0] : c == 1 ? rd4[1] : c == 2 ? rd4[2] : rd4[3];
            if (a.delta_out != nullptr && c < 4 && 4 * g + c < nvalid) {
                a.delta_out[rowbase + t0 + 4 * g + c] = dsel;
                a.rden_out[rowbase + t0 + 4 * g + c] = rsel;
            }
        } else if constexpr (kHasRaw && !is_poly<T>) {
            float dp[ZT][4];             // phi' of the raw K under the output
            lds_feature_lane<DZ>(lds_r, c, g, dp);
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt)
#pragma unroll
                for (int r = 0; r < 4; ++r) out[zt][r] *= dp[zt][r];
        }
        // uniform chunk base + one lane offset; the 16 stores differ by constants only
        T *lane_out = outs + (size_t)t0 * tso + (4 * g * tso + c);
        if constexpr (kRawGrad) {
            // `out` is the gradient for the 64 features: back to the 8 raw values of each token
            float g0, g1;
            poly2_chain(lds_scratch, out, stg.xraw, lane, g0, g1);
            if ((lane >> 2) < nvalid) {
                T *p = outs + (size_t)(t0 + (lane >> 2)) * tso + 2 * (lane & 3);
                store_elem(p, g0);
                store_elem(p + 1, g1);
            }
        } else if ((PASS == kFwd || PASS == kGlobal) && out_tensor == nullptr) {
            // a forward that is run for its denominators only (uniform branch)
        } else if (lds_o != nullptr) {      // uniform
            store_tile<DZ>(lds_o, out, outs + (size_t)t0 * tso, tso, nvalid, lane);
        } else if (nvalid == kChunk) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt) store_elem(lane_out + (r * tso + 16 * zt), out[zt][r]);
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (4 * g + r < nvalid) {
#pragma unroll
                    for (int zt = 0; zt < ZT; ++zt)
                        store_elem(lane_out + (r * tso + 16 * zt), out[zt][r]);
                }
        }

        // ---- carry: U += Y^T Z, and the ones-column vector --------------------------------
        if constexpr (kHasYZ) {
            float yf[XT][4];             // Y, feature-lane
            if constexpr (kStateMode != kBorrowState || PASS == kFwd)
                lds_feature_lane<DX>(lds_y, c, g, yf);
            if constexpr (kStateMode != kBorrowState) {
                if constexpr (kBf) {
#pragma unroll
                    for (int xt = 0; xt < XT; ++xt) {
                        const bf16x4_t yp = pack_bf16x4(yf[xt]);
#pragma unroll
                        for (int zt = 0; zt < ZT; ++zt) U[xt][zt] = mfma16_bf16(yp, zp[zt], U[xt][zt]);
                    }
                } else if constexpr (kSplit) {
#pragma unroll
                    for (int xt = 0; xt < XT; ++xt) {
                        const SplitA<kParts> ys = split_a<kParts>(yf[xt]);
#pragma unroll
                        for (int zt = 0; zt < ZT; ++zt) U[xt][zt] = mfma16_split(ys, zs[zt], U[xt][zt]);
                    }
                } else {
#pragma unroll
                    for (int s = 0; s < 4; ++s)
#pragma unroll
                        for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                            for (int zt = 0; zt < ZT; ++zt)
                                U[xt][zt] = mfma16(yf[xt][s], zf[zt][s], U[xt][zt]);
                }
            }
            if constexpr (PASS == kFwd) {
                // z += column sums of the chunk's phi(K).  Each lane adds up its four tokens;
                // an MFMA against ones adds the four groups and delivers the sums of features
                // 16xt + 4g + r in register r: the very layout z is kept in.
#pragma unroll
                for (int xt = 0; xt < XT; ++xt)
                    zg[xt] = mfma16((yf[xt][0] + yf[xt][1]) + (yf[xt][2] + yf[xt][3]), 1.0f, zg[xt]);
            }
        }
        if constexpr (PASS == kDq) {
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt)
                ecp[zt] += (zf[zt][0] + zf[zt][1]) + (zf[zt][2] + zf[zt][3]);
        }
        if constexpr (PASS == kDk) {
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt) {
                float p = dl4[0] * zf[zt][0];
#pragma unroll
                for (int s = 1; s < 4; ++s) p = fmaf(dl4[s], zf[zt][s], p);
                ecp[zt] += p;
            }
        }
    };

    for (int it = 0; it < count; it += kDepth) {
        step(std::integral_constant<int, 0>{}, it);
        if constexpr (kDepth == 2) {
            if (it + 1 < count) step(std::integral_constant<int, 1>{}, it + 1);
        }
    }

    if constexpr (PASS == kFwd) {       // the wave of the last segment ends with the final state
        if (a.final_S != nullptr && seg == a.nseg - 1) {
            float *s1 = a.final_S + (size_t)bh * D * M;
            float *z1 = a.final_z + (size_t)bh * D;
#pragma unroll
            for (int xt = 0; xt < XT; ++xt) {
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        s1[(16 * xt + 4 * g + r) * M + 16 * zt + c] = U[xt][zt][r];
                if (c == 0) *reinterpret_cast<f32x4 *>(z1 + 16 * xt + 4 * g) = zg[xt];
            }
        }
    }
    if constexpr (Tr::BP == kDq) {      // this segment's sum of delta_b phi(Q_b)
        if (a.totals != nullptr) {
            float *st = a.totals + ((size_t)bh * a.nseg + seg) * state_stride(D, M) + D * M;
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt) {
                const float e = sum_over_groups(rho[zt]);
                if (g == 0) st[16 * zt + c] = e;
            }
        }
    }
    // reverse passes: what has piled up when the wave of the first segment is through is the
    // gradient that leaves through the initial state (kDv carries the matrix, kDk the vector)
    if constexpr (PASS == kDv) {
        if (a.final_S != nullptr && seg == 0) {
            float *s1 = a.final_S + (size_t)bh * D * M;
#pragma unroll
            for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        s1[(16 * xt + 4 * g + r) * M + 16 * zt + c] = U[xt][zt][r];
        }
    }
    if constexpr (PASS == kDk) {
        if (a.final_z != nullptr && seg == 0) {
            float *z1 = a.final_z + (size_t)bh * D;
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt) {
                const float e = sum_over_groups(ecp[zt]);
                if (g == 0) z1[16 * zt + c] = e;
            }
        }
    }
}

// Chunks a pass of the non-causal entry points keeps in flight per wave (sets of staging
// registers).  Measured with bf16 tensors, where a tile is half as many bytes and there is
// register room for a second set: two chunks in flight change nothing (step 0.564 against
// 0.565 ms), these passes wait for instruction issue, not for their loads; so one set it is.
template <typename T>
constexpr int kGlobalDepth = LA_GLOBAL_DEPTH(T);

template <int PASS, int D, int M, typename T, bool kStrided = false>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(2))) void causal_pass_kernel(
    const PassArgs a) {
    using Tr = PassTraits<PASS, D, M>;
    __shared__ float lds_x[tile_floats(Tr::DX)];
    __shared__ float lds_y[Tr::kHasYZ ? tile_floats(Tr::DX) : 4];
    __shared__ float lds_z[Tr::kHasYZ ? tile_floats(Tr::DZ) : 4];
    __shared__ float lds_r[Tr::kHasRaw ? tile_floats(Tr::DZ) : 4];
    // The output goes to memory tile-wise (store_tile) for bf16 tensors and in the non-causal
    // read-out (measured: bf16 causal forward 0.119 -> 0.115 ms, non-causal read-out 0.086 ->
    // 0.073 ms, fp32 0.119 -> 0.114 ms; the fp32 causal forward gains nothing and stores
    // element-wise).
    constexpr bool kTileStore = is_bf16<T> || PASS == kGlobal;
    __shared__ __attribute__((aligned(16))) float lds_o[kTileStore ? tile_floats(Tr::DZ) : 4];
    const int lane = threadIdx.x;
    const int seg = blockIdx.x % a.nseg, bh = blockIdx.x / a.nseg;
    PassStager<PASS, D, M, T, kStrided, PASS >= kGlobal ? kGlobalDepth<T> : 1> stg(a, bh, lane, lds_x, lds_y, lds_z, lds_r);
    run_pass<PASS, D, M, T>(a, stg, lds_x, lds_y, lds_z, lds_r, a.out, bh, seg, lane, nullptr, lds_r,
                            kTileStore ? lds_o : nullptr);
}

// Both reverse passes of the backward (eq. 14 and eq. 15) on one fetch of Q, K, V, dO:
// wave 0 produces dV (a.out), wave 1 produces dK (a.out2).  Wave 0 carries the reverse state R
// (D x M) and republishes it in LDS before every chunk; wave 1, whose read-out needs R^T, reads
// it from there transposed instead of keeping (and updating) a second copy.
template <int D, int M, typename T, bool kStrided = false>
__global__ __launch_bounds__(2 * kWave) __attribute__((amdgpu_waves_per_eu(2))) void reverse_pass_kernel(
    const PassArgs a) {
    __shared__ float lds_fq[tile_floats(D)];    // phi(Q)
    __shared__ float lds_g[tile_floats(M)];     // dO / den
    __shared__ float lds_fk[tile_floats(D)];    // phi(K)
    __shared__ float lds_dk[tile_floats(D)];    // phi'(K)
    __shared__ float lds_v[tile_floats(M)];     // V
    __shared__ float lds_R[M * (D + 4)];        // R before the current chunk, as [m][d]
    const int lane = threadIdx.x & (kWave - 1);
    const int role = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform
    const int seg = blockIdx.x % a.nseg, bh = blockIdx.x / a.nseg;
    if (role == 0) {
        __builtin_amdgcn_s_setprio(LA_PRIO_REV_DV_WAVE);
        ReverseStager<0, D, M, T, kStrided> stg(a, bh, lane, lds_fq, nullptr, lds_g);
        run_pass<kDv, D, M, T, kPublishState>(a, stg, lds_fk, lds_fq, lds_g, nullptr, a.out, bh, seg,
                                              lane, lds_R);
    } else {
        __builtin_amdgcn_s_setprio(LA_PRIO_REV_DK_WAVE);
        ReverseStager<1, D, M, T, kStrided> stg(a, bh, lane, lds_fk, lds_dk, lds_v);
        run_pass<kDk, D, M, T, kBorrowState>(a, stg, lds_v, lds_g, lds_fq, lds_dk, a.out2, bh, seg,
                                             lane, lds_R, lds_dk);
    }
}

// Staging of the two read-outs of the non-causal backward that sweep K and V (dV and dK against
// the grand total of phi(Q)^T dO/den), run side by side by the two waves of one workgroup so
// that K is fetched once for both.  Wave 0 (the dV role) brings K, parked as phi and, for the
// chain rule under dK, as phi'; wave 1 (the dK role) brings V.
template <int ROLE, int D, int M, typename T, bool kStrided = false, int kDepth_ = 1>
struct GlobalBwdStager {
    static constexpr bool kStridedLayout = kStrided;
    static constexpr int kDepth = kDepth_;    // chunks in flight = sets of staging registers (1 or 2)
    static constexpr int F = ROLE == 0 ? D : M, FT = F / 16;
    const T *Src;                       // role 0: K; role 1: V
    const T *Kraw;                      // role 1, polynomial map: K again, for the raw vectors
    float *lds_a, *lds_a2;              // role 0: phi(K), phi'(K); role 1: V, -
    int N, lane;
    bool nt;                            // non-temporal fetches (PassArgs::stream)
    int ts, tsk;
    staged_t<T> st[kDepth][FT];
    float one[FT];
    float dl1, dl4[4];                  // unused by these passes (interface of run_pass)
    float xraw[kPolyRaw], n_xraw[kDepth][kPolyRaw];   // polynomial map, role 1: raw K of token lane / 4

    __device__ __forceinline__ GlobalBwdStager(const PassArgs &a, int bh, int lane_, float *la, float *la2)
        : lds_a(la), lds_a2(la2), N(a.N), lane(lane_), nt(a.stream != 0) {
        constexpr int wk = qk_width<T>(D);
        tsk = tok_stride<kStrided>(a.tok_heads, wk);
        ts = ROLE == 0 ? tsk : tok_stride<kStrided>(a.tok_heads, M);
        Kraw = static_cast<const T *>(a.K) + seq_base<kStrided>(a.N, a.heads, bh, wk);
        Src = ROLE == 0 ? Kraw : static_cast<const T *>(a.V) + seq_base<kStrided>(a.N, a.heads, bh, M);
        dl1 = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) dl4[s] = 0.f;
#pragma unroll
        for (int i = 0; i < FT; ++i) one[i] = 1.0f;
#pragma unroll
        for (int j = 0; j < kPolyRaw; ++j) {
            xraw[j] = 0.f;
#pragma unroll
            for (int k = 0; k < kDepth; ++k) n_xraw[k][j] = 0.f;
        }
    }

    template <int SLOT, bool kFull, bool kNt>
    __device__ __forceinline__ void fetch_impl(const int t0, const int nvalid) {
        if constexpr (ROLE == 0) {
            stage_load_qk<D, kFull, kNt>(Src + (size_t)t0 * ts, ts, nvalid, lane, st[SLOT]);
        } else {
            stage_load<M, kFull, kNt>(Src + (size_t)t0 * ts, ts, nvalid, lane, st[SLOT]);
            if constexpr (is_poly<T>) load_raw8(Kraw + (size_t)t0 * tsk, tsk, nvalid, lane, n_xraw[SLOT]);
        }
    }
    template <int SLOT>
    __device__ __forceinline__ void fetch(const int ch) {
        const int t0 = ch * kChunk;
        const int nvalid = min(kChunk, N - t0);
        if (nt) {                            // uniform branches
            if (nvalid == kChunk) fetch_impl<SLOT, true, true>(t0, nvalid);
            else fetch_impl<SLOT, false, true>(t0, nvalid);
        } else {
            if (nvalid == kChunk) fetch_impl<SLOT, true, false>(t0, nvalid);
            else fetch_impl<SLOT, false, false>(t0, nvalid);
        }
    }

    template <int SLOT, bool kFull>
    __device__ __forceinline__ void park_impl(const int nvalid) {
        if constexpr (ROLE == 0) {
            park_tile<D, kMapPhi, kFull, is_feat<T>>(lds_a, st[SLOT], one, nvalid, lane);
            // (polynomial map: no phi' tile; the dK wave uses that memory as the scratch of poly2_chain)
            if constexpr (!is_poly<T>) park_tile<D, kMapDphi, kFull, is_feat<T>>(lds_a2, st[SLOT], one, nvalid, lane);
        } else {
            park_tile<M, kMapId, kFull, is_feat<T>>(lds_a, st[SLOT], one, nvalid, lane);
        }
    }
    template <int SLOT>
    __device__ __forceinline__ void park(const int nvalid) {
        if (nvalid == kChunk) park_impl<SLOT, true>(nvalid);
        else park_impl<SLOT, false>(nvalid);
        if constexpr (ROLE == 1 && is_poly<T>) {
#pragma unroll
            for (int j = 0; j < kPolyRaw; ++j) xraw[j] = n_xraw[SLOT][j];
        }
    }
};

// dV (a.out, wave 0) and dK (a.out2, wave 1) of the non-causal form (eq. 4-6 differentiated) on
// one sweep over K and V: both are read-outs against the same total, dV_b = phi(K_b) R and
// dphi(K)_b = R V_b + rho, so the only thing the waves share is the K tile.
template <int D, int M, typename T, bool kStrided = false>
__global__ __launch_bounds__(2 * kWave) __attribute__((amdgpu_waves_per_eu(2))) void global_dkdv_kernel(
    const PassArgs a) {
    __shared__ float lds_fk[tile_floats(D)];    // phi(K)
    __shared__ float lds_dk[tile_floats(D)];    // phi'(K) (polynomial map: wave 1's chain-rule scratch)
    __shared__ float lds_v[tile_floats(M)];     // V
    const int lane = threadIdx.x & (kWave - 1);
    const int role = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform
    const int seg = blockIdx.x % a.nseg, bh = blockIdx.x / a.nseg;
    if (role == 0) {
        GlobalBwdStager<0, D, M, T, kStrided, kGlobalDepth<T>> stg(a, bh, lane, lds_fk, lds_dk);
        // Each wave stores its output tile-wise (store_tile) through its own operand tile, which
        // nobody else reads and the wave itself only at the top of a chunk (if it is wide
        // enough).  Measured: this kernel 0.135 -> 0.121 ms with bf16 tensors, 0.233 -> 0.224 ms
        // with fp32; the compute-bound causal backward kernels and the non-causal dQ kernel gain
        // nothing or lose 2-4 %, they store element-wise.
        run_pass<kGlobalDv, D, M, T>(a, stg, lds_fk, nullptr, nullptr, nullptr, a.out, bh, seg, lane, nullptr,
                                     nullptr, D >= M ? lds_fk : nullptr);
    } else {
        GlobalBwdStager<1, D, M, T, kStrided, kGlobalDepth<T>> stg(a, bh, lane, lds_v, nullptr);
        run_pass<kGlobalDk, D, M, T>(a, stg, lds_v, nullptr, nullptr, lds_dk, a.out2, bh, seg, lane,
                                     nullptr, lds_dk, M >= D ? lds_v : nullptr);
    }
}

// Staging of the non-causal dQ pass, shared by the two waves of its workgroup.  Wave 0 (the dQ
// role) brings dO, parked as dO/den (den being the forward's denominator); wave 1 brings Q,
// parked as phi.  There is no in-chunk part and no running sum: V and K are not needed.
template <int ROLE, int D, int M, typename T, bool kStrided = false, int kDepth_ = 1>
struct DqStager {
    static constexpr bool kStridedLayout = kStrided;
    static constexpr int F = ROLE == 0 ? M : D;
    static constexpr int FT = F / 16;
    static constexpr int kDepth = kDepth_;    // chunks in flight = sets of staging registers (1 or 2)
    const T *As;                        // role 0: dO; role 1: Q
    const float *den;
    float *lds_a;                       // role 0: dO/den; role 1: phi(Q)
    int N, lane, g, ts;                 // ts: token stride of this role's tensor
    bool nt;                            // non-temporal fetches (PassArgs::stream)
    staged_t<T> sa[kDepth][FT];
    float sca[kDepth][FT], one[FT];
    float n_den4[kDepth][4];
    float dl1, dl4[4];                  // unused by this pass (interface of run_pass)
    float rd4[4];                       // 1/den of tokens 4g + s of the parked chunk, 0 past the end
    // polynomial map, role 0 (the wave that finishes dQ): raw Q of token lane / 4
    const T *Qraw;
    int tsq;
    float xraw[kPolyRaw], n_xraw[kDepth][kPolyRaw];
    static constexpr int W = ROLE == 0 ? F : qk_width<T>(F);    // elements per token of this role's tensor

    __device__ __forceinline__ DqStager(const PassArgs &a, int bh, int lane_, float *la)
        : lds_a(la), N(a.N), lane(lane_), g(lane_ >> 4), ts(tok_stride<kStrided>(a.tok_heads, W)),
          nt(a.stream != 0) {
        const size_t rowbase = (size_t)bh * a.N;
        As = static_cast<const T *>(ROLE == 0 ? a.G : a.Q) + seq_base<kStrided>(a.N, a.heads, bh, W);
        tsq = tok_stride<kStrided>(a.tok_heads, qk_width<T>(D));
        Qraw = static_cast<const T *>(a.Q) + seq_base<kStrided>(a.N, a.heads, bh, qk_width<T>(D));
#pragma unroll
        for (int j = 0; j < kPolyRaw; ++j) {
            xraw[j] = 0.f;
#pragma unroll
            for (int k = 0; k < kDepth; ++k) n_xraw[k][j] = 0.f;
        }
        den = a.den_in + rowbase;
        dl1 = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            dl4[s] = rd4[s] = 0.f;
#pragma unroll
            for (int k = 0; k < kDepth; ++k) n_den4[k][s] = 1.f;
        }
#pragma unroll
        for (int i = 0; i < FT; ++i) {
            one[i] = 1.0f;
#pragma unroll
            for (int k = 0; k < kDepth; ++k) sca[k][i] = 1.0f;
        }
    }

    template <int SLOT, bool kFull, bool kNt>
    __device__ __forceinline__ void fetch_impl(const int t0, const int nvalid) {
        if constexpr (ROLE == 1) {
            stage_load_qk<F, kFull, kNt>(As + (size_t)t0 * ts, ts, nvalid, lane, sa[SLOT]);
        } else {
            stage_load<F, kFull, kNt>(As + (size_t)t0 * ts, ts, nvalid, lane, sa[SLOT]);
            if constexpr (is_poly<T>) load_raw8(Qraw + (size_t)t0 * tsq, tsq, nvalid, lane, n_xraw[SLOT]);
            stage_rows<F, kFull>(den + t0, nvalid, lane, sca[SLOT]);      // den of the staged rows
#pragma unroll
            for (int s = 0; s < 4; ++s)                                   // den of tokens 4g + s
                n_den4[SLOT][s] = den[t0 + (kFull ? 4 * g + s : min(4 * g + s, nvalid - 1))];
        }
    }

    template <int SLOT>
    __device__ __forceinline__ void fetch(const int ch) {
        const int t0 = ch * kChunk;
        const int nvalid = min(kChunk, N - t0);
        if (nt) {                            // uniform branches
            if (nvalid == kChunk) fetch_impl<SLOT, true, true>(t0, nvalid);
            else fetch_impl<SLOT, false, true>(t0, nvalid);
        } else {
            if (nvalid == kChunk) fetch_impl<SLOT, true, false>(t0, nvalid);
            else fetch_impl<SLOT, false, false>(t0, nvalid);
        }
    }

    template <int SLOT, bool kFull>
    __device__ __forceinline__ void park_impl(const int nvalid) {
        if constexpr (ROLE == 0) {
#pragma unroll
            for (int i = 0; i < FT; ++i) sca[SLOT][i] = __builtin_amdgcn_rcpf(sca[SLOT][i]);
            park_tile<F, kMapScale, kFull, is_feat<T>>(lds_a, sa[SLOT], sca[SLOT], nvalid, lane);
#pragma unroll
            for (int s = 0; s < 4; ++s)
                rd4[s] = (kFull || 4 * g + s < nvalid) ? __builtin_amdgcn_rcpf(n_den4[SLOT][s]) : 0.f;
            if constexpr (is_poly<T>) {
#pragma unroll
                for (int j = 0; j < kPolyRaw; ++j) xraw[j] = n_xraw[SLOT][j];
            }
        } else {
            park_tile<F, kMapPhi, kFull, is_feat<T>>(lds_a, sa[SLOT], one, nvalid, lane);
        }
    }

    template <int SLOT>
    __device__ __forceinline__ void park(const int nvalid) {
        if (nvalid == kChunk) park_impl<SLOT, true>(nvalid);
        else park_impl<SLOT, false>(nvalid);
    }
};

// Wave 1 of the non-causal dQ kernel.  It brings the Q tile in step with wave 0 (same
// barriers, same chunk order) and owns this segment's sum of phi(Q_b) dO_b^T/den_b (eq. 14-15
// restricted to the segment), whose total over the sequence the dV and dK read-outs start
// from: an outer product over the chunk's 16 tokens, 8 operand quads, split once, for 48 (fp32
// tensors) or 32 (bf16 tensors) bf16 MFMAs.
template <int D, int M, typename T, typename Stager>
__device__ __forceinline__ void run_dq_sums(const PassArgs &a, Stager &stg, const float *lds_fq,
                                            const float *lds_g, const int bh, const int seg,
                                            const int lane) {
    constexpr int XT = D / 16, ZT = M / 16;
    const int c = lane & 15, g = lane >> 4;
    const int nchunks = (a.N + kChunk - 1) / kChunk;
    const int ch_begin = seg * a.chunks_per_seg;
    const int ch_end = min(ch_begin + a.chunks_per_seg, nchunks);
    const bool want = a.totals != nullptr;         // uniform
    constexpr int kParts = is_bf16<T> ? 2 : 3;     // see run_pass

    f32x4 R[XT][ZT];                               // element (d = 16xt + 4g + r, m = 16zt + c)
#pragma unroll
    for (int xt = 0; xt < XT; ++xt)
#pragma unroll
        for (int zt = 0; zt < ZT; ++zt) R[xt][zt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // kDepth chunks in flight, each in its own set of staging registers (as in run_pass)
    constexpr int kDepth = Stager::kDepth;
    if (ch_begin < ch_end) stg.template fetch<0>(ch_begin);
    if constexpr (kDepth == 2) {
        if (ch_begin + 1 < ch_end) stg.template fetch<1>(ch_begin + 1);
    }
    auto step = [&](auto slot_tag, const int ch) {
        constexpr int kSlot = decltype(slot_tag)::value;
        const int nvalid = min(kChunk, a.N - ch * kChunk);
        __syncthreads();
        stg.template park<kSlot>(nvalid);
        if (ch + kDepth < ch_end) stg.template fetch<kSlot>(ch + kDepth);
        __builtin_amdgcn_s_sleep(LA_SLEEP_AFTER_FETCH);    // see run_pass
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        if (want) {
            float qf[XT][4], gf[ZT][4];
            lds_feature_lane<D>(lds_fq, c, g, qf);
            lds_feature_lane<M>(lds_g, c, g, gf);
            if constexpr (LA_SPLIT_SUMS) {
                SplitA<kParts> qa[XT];
#pragma unroll
                for (int xt = 0; xt < XT; ++xt) qa[xt] = split_a<kParts>(qf[xt]);
#pragma unroll
                for (int zt = 0; zt < ZT; ++zt) {
                    const SplitB<kParts> gb = split_b<kParts>(gf[zt]);
#pragma unroll
                    for (int xt = 0; xt < XT; ++xt) R[xt][zt] = mfma16_split(qa[xt], gb, R[xt][zt]);
                }
            } else {
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                        for (int zt = 0; zt < ZT; ++zt)
                            R[xt][zt] = mfma16(qf[xt][s], gf[zt][s], R[xt][zt]);
            }
        }
    };
    for (int ch = ch_begin; ch < ch_end; ch += kDepth) {
        step(std::integral_constant<int, 0>{}, ch);
        if constexpr (kDepth == 2) {
            if (ch + 1 < ch_end) step(std::integral_constant<int, 1>{}, ch + 1);
        }
    }
    if (want) {
        float *st = a.totals + ((size_t)bh * a.nseg + seg) * state_stride(D, M);
#pragma unroll
        for (int xt = 0; xt < XT; ++xt)
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    st[(16 * xt + 4 * g + r) * M + 16 * zt + c] = R[xt][zt][r];
    }
}

// dQ of the non-causal form (eq. 4-6 differentiated): a read-out of dO/den against the sum of
// phi(K) V^T over the whole sequence (a.state: its grand total, or the segment totals to add up),
// which wave 0 keeps in registers; delta as in the causal pass (see the top of this file), then
// times phi'(Q).  On the way wave 1 sums phi(Q)^T dO/den per segment for the dV and dK read-outs
// (run_dq_sums).  Reads Q, dO and the forward's denominators.
template <int D, int M, typename T, bool kStrided = false>
__global__ __launch_bounds__(2 * kWave) __attribute__((amdgpu_waves_per_eu(2))) void dq_pass_kernel(
    const PassArgs a) {
    __shared__ float lds_g[tile_floats(M)];                       // dO / den
    __shared__ float lds_fq[tile_floats(D)];                      // phi(Q)
    __shared__ float lds_chain[is_poly<T> ? tile_floats(D) : 4];  // polynomial map: scratch of poly2_chain
    const int lane = threadIdx.x & (kWave - 1);
    const int role = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform
    const int seg = blockIdx.x % a.nseg, bh = blockIdx.x / a.nseg;
    if (role == 0) {
        DqStager<0, D, M, T, kStrided, kGlobalDepth<T>> stg(a, bh, lane, lds_g);
        run_pass<kGlobalDq, D, M, T>(a, stg, lds_g, nullptr, nullptr, lds_fq, a.out, bh, seg, lane,
                                     nullptr, lds_chain);
    } else {
        DqStager<1, D, M, T, kStrided, kGlobalDepth<T>> stg(a, bh, lane, lds_fq);
        run_dq_sums<D, M, T>(a, stg, lds_fq, lds_g, bh, seg, lane);
    }
}

// The causal dQ pass (eq. 13), the forward-direction half of the backward: dQ, plus everything
// the reverse half needs (1/den, delta, and per-segment sums of phi(Q)^T [dO/den, delta] when the
// sequences are cut).  Reads Q, K, V, dO and the forward's denominators; the forward's output O
// is not needed.  It is organised so that neither wave waits long for the other.  (Its
// predecessor handed the whole running sum S from one wave to the other through LDS every
// chunk, 16 KB, and its first wave then carried 84 fp32 MFMAs in one dependent chain while the
// second idled at the barrier: measured, that chain set the pace, fp32 0.344 -> 0.320 ms, bf16
// 0.293 -> 0.255 ms.)  The work of a chunk is cut along the data flow:
//   wave 1 ("state wave") owns S^T (M x D) in accumulators.  It reads out A0 = (dO/den) S^T (the
//          part of eq. 13 that comes from the tokens before the chunk, 64 fp32 MFMAs), hands
//          the 16 x D result to wave 0 through LDS (4 KB), then adds the chunk's V^T phi(K) to S^T
//          and, when the sequences are cut, phi(Q)^T dO/den to this segment's sum for the reverse
//          passes (96 bf16 MFMAs on split operands);
//   wave 0 ("chunk wave") forms the masked scores (dO/den) V^T, their product with phi(K), the
//          running sum of phi(K) for the ones column, and after adding A0 finishes dQ: delta,
//          the chain rule through phi, the stores.
// The input tiles are double-buffered in LDS: each wave parks its two tiles of the next chunk
// while the other is still reading the current ones, so a chunk costs two barriers and the
// feature map (32 exponentials per lane and chunk, wave 0) is off the critical path.
template <int D, int M, typename T, bool kStrided = false>
__global__ __launch_bounds__(2 * kWave) __attribute__((amdgpu_waves_per_eu(2))) void dq_causal_kernel(
    const PassArgs a) {
    constexpr int DT = D / 16, MT = M / 16;
    // fp32 tensors: three-part operands where a product runs on the bf16 pipe, fp32 MFMAs for the
    // scores and the read-out; bf16 tensors: two-part operands everywhere (see run_pass)
    constexpr int kParts = is_bf16<T> ? 2 : 3;
    __shared__ float lds_g[2][tile_floats(M)];       // dO / den
    __shared__ float lds_v[2][tile_floats(M)];       // V
    __shared__ float lds_fk[2][tile_floats(D)];      // phi(K)
    __shared__ float lds_fq[2][tile_floats(D)];      // phi(Q)
    // A0 in wave 1's register layout, [DT][kWave][4].  With the polynomial map the same memory is
    // wave 0's scratch for poly2_chain: wave 0 has taken A0 out by then, and wave 1 writes the next
    // A0 only after the barrier that follows (a separate array would cost the fourth workgroup
    // per compute unit).
    constexpr int kA0Floats = DT * kWave * 4;
    __shared__ __attribute__((aligned(16))) float lds_a0_mem[is_poly<T> && tile_floats(D) > kA0Floats ? tile_floats(D) : kA0Floats];
    float (*lds_a0)[kWave][4] = reinterpret_cast<float (*)[kWave][4]>(lds_a0_mem);
    float *lds_chain = lds_a0_mem;
    const int lane = threadIdx.x & (kWave - 1), c = lane & 15, g = lane >> 4;
    const int role = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform
    const bool nt = a.stream != 0;                                       // non-temporal fetches
    const int seg = blockIdx.x % a.nseg, bh = blockIdx.x / a.nseg;
    const int nchunks = (a.N + kChunk - 1) / kChunk;
    const int ch_begin = seg * a.chunks_per_seg;
    const int count = min(ch_begin + a.chunks_per_seg, nchunks) - ch_begin;
    const size_t rowbase = (size_t)bh * a.N;
    // the sums before this segment: the caller's initial state (if any) plus the slots of the
    // state array that state_slots() names
    int nslots = 0, slot_lo = 0, slot_hi = 0;
    if (a.state != nullptr) state_slots(a, seg, kStatePrefix, nslots, slot_lo, slot_hi);
    const float *slots = a.state != nullptr ? a.state + (size_t)bh * nslots * state_stride(D, M) : nullptr;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

    if (role == 0) {
        // ---- chunk wave: brings Q and K --------------------------------------------------------
        __builtin_amdgcn_s_setprio(LA_PRIO_DQ_CHUNK_WAVE);
        constexpr int W = qk_width<T>(D);          // elements per token of Q, K and dQ
        const int ts = tok_stride<kStrided>(a.tok_heads, W);
        const T *Qs = static_cast<const T *>(a.Q) + seq_base<kStrided>(a.N, a.heads, bh, W);
        const T *Ks = static_cast<const T *>(a.K) + seq_base<kStrided>(a.N, a.heads, bh, W);
        T *outs = static_cast<T *>(a.out) + seq_base<kStrided>(a.N, a.heads, bh, W);
        const float *den = a.den_in + rowbase;
        staged_t<T> sq[DT], sk[DT];
        float one[DT], nden[4], rd4[4];
        float xraw[kPolyRaw], n_xraw[kPolyRaw];    // polynomial map: raw Q of token lane / 4
#pragma unroll
        for (int j = 0; j < kPolyRaw; ++j) xraw[j] = n_xraw[j] = 0.f;
        float ecp[DT];     // z[16zt + c] before the chunk, as four per-lane partial sums (lanes (c, g = 0..3))
        float rho[DT];     // this segment's sum of delta_b phi(Q_b)[16zt + c], same partial form
#pragma unroll
        for (int zt = 0; zt < DT; ++zt) {
            one[zt] = 1.0f;
            rho[zt] = 0.f;
            ecp[zt] = (a.init_z != nullptr && g == 0) ? a.init_z[(size_t)bh * D + 16 * zt + c] : 0.f;
        }
        for (int j = slot_lo; j < slot_hi; ++j) {
            const float *sv = slots + (size_t)j * state_stride(D, M) + D * M;
#pragma unroll
            for (int zt = 0; zt < DT; ++zt) ecp[zt] += g == 0 ? sv[16 * zt + c] : 0.f;
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) nden[s] = 1.f, rd4[s] = 0.f;
        // constant lower-triangular mask (token 4g + s <= token c) as bf16 ones
        const u32x2_t mk = {((4 * g + 0) <= c ? 0x3f80u : 0u) | ((4 * g + 1) <= c ? 0x3f800000u : 0u),
                            ((4 * g + 2) <= c ? 0x3f80u : 0u) | ((4 * g + 3) <= c ? 0x3f800000u : 0u)};

        auto fetch_tiles = [&](auto full_tag, auto nt_tag, const int t0, const int nvalid) {
            constexpr bool kFull = decltype(full_tag)::value, kNt = decltype(nt_tag)::value;
            stage_load_qk<D, kFull, kNt>(Qs + (size_t)t0 * ts, ts, nvalid, lane, sq);
            stage_load_qk<D, kFull, kNt>(Ks + (size_t)t0 * ts, ts, nvalid, lane, sk);
        };
        auto fetch = [&](const int ch) {
            const int t0 = ch * kChunk;
            const int nvalid = min(kChunk, a.N - t0);
            if (nt) {                        // uniform branches
                if (nvalid == kChunk) fetch_tiles(std::true_type{}, std::true_type{}, t0, nvalid);
                else fetch_tiles(std::false_type{}, std::true_type{}, t0, nvalid);
            } else {
                if (nvalid == kChunk) fetch_tiles(std::true_type{}, std::false_type{}, t0, nvalid);
                else fetch_tiles(std::false_type{}, std::false_type{}, t0, nvalid);
            }
            if constexpr (is_poly<T>) load_raw8(Qs + (size_t)t0 * ts, ts, nvalid, lane, n_xraw);
#pragma unroll
            for (int s = 0; s < 4; ++s) nden[s] = den[t0 + min(4 * g + s, nvalid - 1)];
        };
        auto park = [&](const int ch, const int buf) {
            const int nvalid = min(kChunk, a.N - ch * kChunk);
            if (nvalid == kChunk) {
                park_tile<D, kMapPhi, true, is_feat<T>>(lds_fq[buf], sq, one, nvalid, lane);
                park_tile<D, kMapPhi, true, is_feat<T>>(lds_fk[buf], sk, one, nvalid, lane);
            } else {
                park_tile<D, kMapPhi, false, is_feat<T>>(lds_fq[buf], sq, one, nvalid, lane);
                park_tile<D, kMapPhi, false, is_feat<T>>(lds_fk[buf], sk, one, nvalid, lane);
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) rd4[s] = 4 * g + s < nvalid ? __builtin_amdgcn_rcpf(nden[s]) : 0.f;
            if constexpr (is_poly<T>) {
#pragma unroll
                for (int j = 0; j < kPolyRaw; ++j) xraw[j] = n_xraw[j];
            }
        };

        if (count > 0) {
            fetch(ch_begin);
            park(ch_begin, 0);
            if (count > 1) fetch(ch_begin + 1);
        }
        for (int n = 0; n < count; ++n) {
            const int buf = n & 1, ch = ch_begin + n, t0 = ch * kChunk;
            const int nvalid = min(kChunk, a.N - t0);
            __builtin_amdgcn_s_sleep(LA_SLEEP_AFTER_FETCH);    // see run_pass
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();                 // the tiles of this chunk are parked (both waves)

            // scores W[a][b] = (dO_a/den_a) . V_b: lane (c = a, g), register r: b = 4g + r
            float xa[MT][4], ya[MT][4];
            lds_token_lane<M>(lds_g[buf], c, g, xa);
            lds_token_lane<M>(lds_v[buf], c, g, ya);
            f32x4 w0 = zero4, w1 = zero4;
            if constexpr (is_bf16<T>) {       // V of a bf16 tensor is exact in bf16
#pragma unroll
                for (int xt = 0; xt < MT; xt += 2) {
                    w0 = mfma16_split(exact_bf16(ya[xt]), split_b<2>(xa[xt]), w0);
                    w1 = mfma16_split(exact_bf16(ya[xt + 1]), split_b<2>(xa[xt + 1]), w1);
                }
            } else {
#pragma unroll
                for (int xt = 0; xt < MT; xt += 2)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        w0 = mfma16(ya[xt][r], xa[xt][r], w0);
                        w1 = mfma16(ya[xt + 1][r], xa[xt + 1][r], w1);
                    }
            }
            float wq[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) wq[r] = (4 * g + r) <= c ? w0[r] + w1[r] : 0.f;   // select, never multiply
            // in-chunk part of eq. 13: W phi(K); and z_a = z + running sum of phi(K) up to token a
            float zf[DT][4];
            lds_feature_lane<D>(lds_fk[buf], c, g, zf);
            const SplitA<kParts> ws = split_a<kParts>(wq);
            f32x4 out[DT], cz[DT];
#pragma unroll
            for (int zt = 0; zt < DT; ++zt) {
                const SplitB<kParts> zs = split_b<kParts>(zf[zt]);
                out[zt] = mfma16_split(ws, zs, zero4);
                cz[zt] = mfma16_mask(mk, zs, mfma16(1.0f, ecp[zt], zero4));
            }
            float fq[DT][4];                 // phi(Q): token 4g + r, feature 16zt + c
            lds_feature_lane<D>(lds_fq[buf], c, g, fq);
            __syncthreads();                 // wave 1 has put A0 into LDS
#pragma unroll
            for (int zt = 0; zt < DT; ++zt) out[zt] += *reinterpret_cast<const f32x4 *>(&lds_a0[zt][lane][0]);

            // delta_a = -(phi(Q_a) . A_a)/den_a, then dphi(Q)_a = A_a + delta_a z_a, times phi'(Q_a)
            float d4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float p = out[0][r] * fq[0][r];
#pragma unroll
                for (int zt = 1; zt < DT; ++zt) p = fmaf(out[zt][r], fq[zt][r], p);
                d4[r] = -row_sum16(p) * rd4[r];
            }
#pragma unroll
            for (int zt = 0; zt < DT; ++zt) {
                float rp = 0.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    rp = fmaf(d4[r], fq[zt][r], rp);
                    out[zt][r] = fmaf(d4[r], cz[zt][r], out[zt][r]) * feature_slope<T>(fq[zt][r]);
                }
                rho[zt] += rp;
                ecp[zt] += (zf[zt][0] + zf[zt][1]) + (zf[zt][2] + zf[zt][3]);
            }
            const int tso = ts;
            T *lane_out = outs + (size_t)t0 * tso + (4 * g * tso + c);
            if constexpr (is_poly<T>) {
                // `out` is the gradient for the 64 features: back to the 8 raw values of each token
                float g0, g1;
                poly2_chain(lds_chain, out, xraw, lane, g0, g1);
                if ((lane >> 2) < nvalid) {
                    T *p = outs + (size_t)(t0 + (lane >> 2)) * tso + 2 * (lane & 3);
                    store_elem(p, g0);
                    store_elem(p + 1, g1);
                }
            } else if (nvalid == kChunk) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int zt = 0; zt < DT; ++zt) store_elem(lane_out + (r * tso + 16 * zt), out[zt][r]);
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (4 * g + r < nvalid) {
#pragma unroll
                        for (int zt = 0; zt < DT; ++zt) store_elem(lane_out + (r * tso + 16 * zt), out[zt][r]);
                    }
            }
            // lanes c < 4 of each group write 1/den and delta of token 4g + c
            const float dsel = c == 0 ? d4[0] : c == 1 ? d4[1] : c == 2 ? d4[2] : d4[3];
            const float rsel = c == 0 ? rd4[0] : c == 1 ? rd4[1] : c == 2 ? rd4[2] : rd4[3];
            if (a.delta_out != nullptr && c < 4 && 4 * g + c < nvalid) {
                a.delta_out[rowbase + t0 + 4 * g + c] = dsel;
                a.rden_out[rowbase + t0 + 4 * g + c] = rsel;
            }
            // the next chunk's tiles go into the other buffer (nobody reads it any more)
            if (n + 1 < count) {
                park(ch + 1, buf ^ 1);
                if (n + 2 < count) fetch(ch + 2);
            }
        }
        if (a.totals != nullptr) {          // this segment's sum of delta_b phi(Q_b)
            float *tot = a.totals + ((size_t)bh * a.nseg + seg) * state_stride(D, M) + D * M;
#pragma unroll
            for (int zt = 0; zt < DT; ++zt) {
                const float e = sum_over_groups(rho[zt]);
                if (g == 0) tot[16 * zt + c] = e;
            }
        }
    } else {
        // ---- state wave: brings dO (parked as dO/den) and V --------------------------------------
        __builtin_amdgcn_s_setprio(LA_PRIO_DQ_STATE_WAVE);
        const int ts = tok_stride<kStrided>(a.tok_heads, M);
        const T *Gs = static_cast<const T *>(a.G) + seq_base<kStrided>(a.N, a.heads, bh, M);
        const T *Vs = static_cast<const T *>(a.V) + seq_base<kStrided>(a.N, a.heads, bh, M);
        const float *den = a.den_in + rowbase;
        const bool want = a.totals != nullptr;         // uniform
        staged_t<T> sg[MT], sv[MT];
        float sca[MT], one[MT];
        f32x4 U[MT][DT];      // S^T: element (m = 16xt + 4g + r, d = 16zt + c)
        f32x4 R[DT][MT];      // this segment's phi(Q)^T dO/den: element (d = 16xt + 4g + r, m = 16zt + c)
#pragma unroll
        for (int xt = 0; xt < MT; ++xt) {
            sca[xt] = one[xt] = 1.0f;
#pragma unroll
            for (int zt = 0; zt < DT; ++zt) U[xt][zt] = R[zt][xt] = zero4;
        }
        auto add_state = [&](const float *sm) {     // sm: S as [D][M]
#pragma unroll
            for (int xt = 0; xt < MT; ++xt)
#pragma unroll
                for (int zt = 0; zt < DT; ++zt) U[xt][zt] += load4_state(sm + (16 * zt + c) * M + 16 * xt + 4 * g);
        };
        if (a.init_S != nullptr) add_state(a.init_S + (size_t)bh * D * M);
        for (int j = slot_lo; j < slot_hi; ++j) add_state(slots + (size_t)j * state_stride(D, M));
        auto fetch_tiles = [&](auto full_tag, auto nt_tag, const int t0, const int nvalid) {
            constexpr bool kFull = decltype(full_tag)::value, kNt = decltype(nt_tag)::value;
            stage_load<M, kFull, kNt>(Gs + (size_t)t0 * ts, ts, nvalid, lane, sg);
            stage_load<M, kFull, kNt>(Vs + (size_t)t0 * ts, ts, nvalid, lane, sv);
            stage_rows<M, kFull>(den + t0, nvalid, lane, sca);
        };
        auto fetch = [&](const int ch) {
            const int t0 = ch * kChunk;
            const int nvalid = min(kChunk, a.N - t0);
            if (nt) {                        // uniform branches
                if (nvalid == kChunk) fetch_tiles(std::true_type{}, std::true_type{}, t0, nvalid);
                else fetch_tiles(std::false_type{}, std::true_type{}, t0, nvalid);
            } else {
                if (nvalid == kChunk) fetch_tiles(std::true_type{}, std::false_type{}, t0, nvalid);
                else fetch_tiles(std::false_type{}, std::false_type{}, t0, nvalid);
            }
        };
        auto park = [&](const int ch, const int buf) {
            const int nvalid = min(kChunk, a.N - ch * kChunk);
#pragma unroll
            for (int i = 0; i < MT; ++i) sca[i] = __builtin_amdgcn_rcpf(sca[i]);
            if (nvalid == kChunk) {
                park_tile<M, kMapScale, true, is_feat<T>>(lds_g[buf], sg, sca, nvalid, lane);
                park_tile<M, kMapId, true, is_feat<T>>(lds_v[buf], sv, one, nvalid, lane);
            } else {
                park_tile<M, kMapScale, false, is_feat<T>>(lds_g[buf], sg, sca, nvalid, lane);
                park_tile<M, kMapId, false, is_feat<T>>(lds_v[buf], sv, one, nvalid, lane);
            }
        };

        if (count > 0) {
            fetch(ch_begin);
            park(ch_begin, 0);
            if (count > 1) fetch(ch_begin + 1);
        }
        for (int n = 0; n < count; ++n) {
            const int buf = n & 1, ch = ch_begin + n;
            __builtin_amdgcn_s_sleep(LA_SLEEP_AFTER_FETCH);    // see run_pass
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();                 // the tiles of this chunk are parked (both waves)

            // A0 = (dO/den) S^T: lane (c, g), register r: token 4g + r, feature 16zt + c
            float xa[MT][4];
            lds_token_lane<M>(lds_g[buf], c, g, xa);
            f32x4 out[DT];
#pragma unroll
            for (int zt = 0; zt < DT; ++zt) out[zt] = zero4;
            if constexpr (is_bf16<T>) {
#pragma unroll
                for (int xt = 0; xt < MT; ++xt) {
                    // the state quads take the narrow form (see run_pass), the tile quad the wide one
                    const SplitB<2> xs = split_b<2>(xa[xt]);
                    Split2 us[DT];
                    split2_batch(U[xt], us);
#pragma unroll
                    for (int zt = 0; zt < DT; ++zt) out[zt] = mfma16_split_ba(xs, as_a(us[zt]), out[zt]);
                }
            } else {
#pragma unroll
                for (int xt = 0; xt < MT; ++xt)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
#pragma unroll
                        for (int zt = 0; zt < DT; ++zt) out[zt] = mfma16(xa[xt][r], U[xt][zt][r], out[zt]);
            }
#pragma unroll
            for (int zt = 0; zt < DT; ++zt) lds_store4(&lds_a0[zt][lane][0], out[zt]);
            __syncthreads();                 // A0 is there for wave 0

            if (n + 1 < count) {
                park(ch + 1, buf ^ 1);
                if (n + 2 < count) fetch(ch + 2);
                __builtin_amdgcn_s_sleep(LA_SLEEP_AFTER_FETCH);
                __builtin_amdgcn_sched_barrier(0);
            }
            // S^T += V^T phi(K) over the chunk's tokens (eq. 10)
            float yf[MT][4], zf[DT][4];
            lds_feature_lane<M>(lds_v[buf], c, g, yf);
            lds_feature_lane<D>(lds_fk[buf], c, g, zf);
            {
                SplitB<kParts> zs[DT];
#pragma unroll
                for (int zt = 0; zt < DT; ++zt) zs[zt] = split_b<kParts>(zf[zt]);
#pragma unroll
                for (int xt = 0; xt < MT; ++xt) {
                    if constexpr (is_bf16<T>) {
                        const ExactBf16 ys = exact_bf16(yf[xt]);
#pragma unroll
                        for (int zt = 0; zt < DT; ++zt) U[xt][zt] = mfma16_split(ys, zs[zt], U[xt][zt]);
                    } else {
                        const SplitA<kParts> ys = split_a<kParts>(yf[xt]);
#pragma unroll
                        for (int zt = 0; zt < DT; ++zt) U[xt][zt] = mfma16_split(ys, zs[zt], U[xt][zt]);
                    }
                }
            }
            // this segment's phi(Q)^T dO/den (eq. 14-15 restricted to the segment)
            if (want) {
                float qf[DT][4], gf[MT][4];
                lds_feature_lane<D>(lds_fq[buf], c, g, qf);
                lds_feature_lane<M>(lds_g[buf], c, g, gf);
                SplitA<kParts> qa[DT];
#pragma unroll
                for (int xt = 0; xt < DT; ++xt) qa[xt] = split_a<kParts>(qf[xt]);
#pragma unroll
                for (int zt = 0; zt < MT; ++zt) {
                    const SplitB<kParts> gb = split_b<kParts>(gf[zt]);
#pragma unroll
                    for (int xt = 0; xt < DT; ++xt) R[xt][zt] = mfma16_split(qa[xt], gb, R[xt][zt]);
                }
            }
        }
        if (want) {
            float *tot = a.totals + ((size_t)bh * a.nseg + seg) * state_stride(D, M);
#pragma unroll
            for (int xt = 0; xt < DT; ++xt)
#pragma unroll
                for (int zt = 0; zt < MT; ++zt)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        tot[(16 * xt + 4 * g + r) * M + 16 * zt + c] = R[xt][zt][r];
        }
    }
}

// ---- per-segment totals (first phase of the segment scan) ---------------------------------
// S = sum phi(K_b)^T V_b, z = sum phi(K_b) over the tokens of one segment (eq. 10-11), written
// as [D][M] row-major followed by the D-vector.  (The matching sums of the backward, over Q and
// dO, come out of the dQ kernel.)
struct SegArgs {
    const void *Y;        // K [BH, N, D]
    const void *Z;        // V [BH, N, M]
    float *state;         // [BH, nseg, state_stride]
    int N, nseg, chunks_per_seg;
    int skip_seg;         // segment whose total nobody reads (-1: none)
    int heads, tok_heads; // layout of K and V, as in PassArgs
    int stream;           // as in PassArgs
};

template <int D, int M, typename T, bool kStrided = false>
__global__ __launch_bounds__(kWave) void segment_state_kernel(const SegArgs a) {
    constexpr int XT = D / 16, ZT = M / 16;
    // bf16 tensors: 16-bit operands (two parts), not plain bf16 products.  These sums also
    // serve the backward passes (as the states at the segment borders, and as the grand total
    // of the non-causal gradient), which need S and z built from the same feature values
    // to better than 8 bits: their results are differences of nearly equal terms.
    constexpr int kParts = is_bf16<T> ? 2 : 3;
    __shared__ float lds_y[tile_floats(D)];
    __shared__ float lds_z[tile_floats(M)];
    const int lane = threadIdx.x, c = lane & 15, g = lane >> 4;
    const bool nt = a.stream != 0;        // non-temporal fetches
    const int seg = blockIdx.x % a.nseg, bh = blockIdx.x / a.nseg;
    if (seg == a.skip_seg) return;
    const int nchunks = (a.N + kChunk - 1) / kChunk;
    const int ch_begin = seg * a.chunks_per_seg;
    const int ch_end = min(ch_begin + a.chunks_per_seg, nchunks);
    const int tsy = tok_stride<kStrided>(a.tok_heads, qk_width<T>(D)), tsz = tok_stride<kStrided>(a.tok_heads, M);
    const T *Ys = static_cast<const T *>(a.Y) + seq_base<kStrided>(a.N, a.heads, bh, qk_width<T>(D));
    const T *Zs = static_cast<const T *>(a.Z) + seq_base<kStrided>(a.N, a.heads, bh, M);

    f32x4 U[XT][ZT];
    float ec[XT];
#pragma unroll
    for (int xt = 0; xt < XT; ++xt) {
        ec[xt] = 0.f;
#pragma unroll
        for (int zt = 0; zt < ZT; ++zt) U[xt][zt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    staged_t<T> sy[XT], sz[ZT];
    float oney[XT], onez[ZT];
#pragma unroll
    for (int i = 0; i < XT; ++i) oney[i] = 1.0f;
#pragma unroll
    for (int i = 0; i < ZT; ++i) onez[i] = 1.0f;

    auto fetch_tiles = [&](auto full_tag, auto nt_tag, const int t0, const int nvalid) {
        constexpr bool kFull = decltype(full_tag)::value, kNt = decltype(nt_tag)::value;
        stage_load_qk<D, kFull, kNt>(Ys + (size_t)t0 * tsy, tsy, nvalid, lane, sy);
        stage_load<M, kFull, kNt>(Zs + (size_t)t0 * tsz, tsz, nvalid, lane, sz);
    };
    auto fetch = [&](const int ch) {
        const int t0 = ch * kChunk;
        const int nvalid = min(kChunk, a.N - t0);
        if (nt) {                            // uniform branches
            if (nvalid == kChunk) fetch_tiles(std::true_type{}, std::true_type{}, t0, nvalid);
            else fetch_tiles(std::false_type{}, std::true_type{}, t0, nvalid);
        } else {
            if (nvalid == kChunk) fetch_tiles(std::true_type{}, std::false_type{}, t0, nvalid);
            else fetch_tiles(std::false_type{}, std::false_type{}, t0, nvalid);
        }
    };

    if (ch_begin < ch_end) fetch(ch_begin);
    for (int ch = ch_begin; ch < ch_end; ++ch) {
        const int nvalid = min(kChunk, a.N - ch * kChunk);
        __syncthreads();
        if (nvalid == kChunk) {
            park_tile<D, kMapPhi, true, is_feat<T>>(lds_y, sy, oney, nvalid, lane);
            park_tile<M, kMapId, true, is_feat<T>>(lds_z, sz, onez, nvalid, lane);
        } else {
            park_tile<D, kMapPhi, false, is_feat<T>>(lds_y, sy, oney, nvalid, lane);
            park_tile<M, kMapId, false, is_feat<T>>(lds_z, sz, onez, nvalid, lane);
        }
        if (ch + 1 < ch_end) fetch(ch + 1);
        __builtin_amdgcn_s_sleep(LA_SLEEP_AFTER_FETCH);    // see run_pass
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();

        float yf[XT][4], zf[ZT][4];
        lds_feature_lane<D>(lds_y, c, g, yf);
        lds_feature_lane<M>(lds_z, c, g, zf);
        if constexpr (LA_SPLIT_SUMS != 0 || is_bf16<T>) {
            SplitA<kParts> ys[XT];
#pragma unroll
            for (int xt = 0; xt < XT; ++xt) ys[xt] = split_a<kParts>(yf[xt]);
#pragma unroll
            for (int zt = 0; zt < ZT; ++zt) {
                if constexpr (is_bf16<T>) {     // V of a bf16 tensor is exact in bf16
                    const ExactBf16 zs = exact_bf16(zf[zt]);
#pragma unroll
                    for (int xt = 0; xt < XT; ++xt) U[xt][zt] = mfma16_split(ys[xt], zs, U[xt][zt]);
                } else {
                    const SplitB<kParts> zs = split_b<kParts>(zf[zt]);
#pragma unroll
                    for (int xt = 0; xt < XT; ++xt) U[xt][zt] = mfma16_split(ys[xt], zs, U[xt][zt]);
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int xt = 0; xt < XT; ++xt)
#pragma unroll
                    for (int zt = 0; zt < ZT; ++zt)
                        U[xt][zt] = mfma16(yf[xt][s], zf[zt][s], U[xt][zt]);
        }
#pragma unroll
        for (int xt = 0; xt < XT; ++xt) ec[xt] += (yf[xt][0] + yf[xt][1]) + (yf[xt][2] + yf[xt][3]);
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
