// Device-side building blocks shared by the gfx950 linear-attention kernels:
// feature map, element conversion, coalesced tile fetch, the LDS image of a tile with
// the two MFMA operand layouts read from it, and the MFMA wrappers (fp32, bf16, and fp32
// products on the bf16 pipe through an exact operand split).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace la {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kChunk = 16;       // tokens per chunk = MFMA tile edge
constexpr int kWave = 64;

// ---- feature map (paper eq. 7): phi(x) = elu(x) + 1 ------------------------------------
// x > 0: x + 1; otherwise exp(x).  Written without a branch or a select:
//   t      = min(exp(x), 1) = exp(min(x, 0))      (one exponential, result clamped to [0, 1];
//                                                  an overflow to +inf for large x clamps to 1)
//   phi'(x) = t                                   (1 for x > 0, exp(x) otherwise)
//   phi(x)  = max(x + 1, t)                       (exp(x) >= x + 1 everywhere, and t = 1 < x + 1
//                                                  for x > 0)
// fp32 vector instructions and fp32 MFMAs share one pipeline on this chip, so every
// instruction saved here is matrix time won.
__device__ __forceinline__ float dphi(float x) {
    return __builtin_amdgcn_fmed3f(__expf(x), 0.0f, 1.0f);
}
__device__ __forceinline__ float phi(float x) { return fmaxf(x + 1.0f, dphi(x)); }
// phi' from phi: x + 1 > 1 for x > 0, exp(x) <= 1 otherwise, so phi' = min(phi, 1) (phi > 0)
__device__ __forceinline__ float dphi_from_phi(float f) { return __builtin_amdgcn_fmed3f(f, 0.0f, 1.0f); }

// ---- element types ------------------------------------------------------------------------
struct bf16_t { uint16_t bits; };
// The same two storage types for calls whose Q and K already hold feature values phi(Q), phi(K)
// of a map the caller applied (any non-negative map, section 3.2): the kernels then apply no
// map, and gradients are with respect to those features.  (V, O, dO and the gradients share
// the element type; for them the tag changes nothing.)
struct feat_f32 { float v; };
struct feat_bf16 { uint16_t bits; };
// fp32 tensors with the feature map of the degree-2 polynomial kernel (section 3.2),
// phi(x) = vec(x x^T): Q and K hold kPolyRaw = 8 raw values per token, a tile of phi(Q) or phi(K)
// has 64 features (feature 8i + j = x_i x_j) and is built in the staging registers when it is
// fetched (stage_load_poly2); inside the kernels it is a tile of given features like any other.
// Gradients go back to the raw vectors (poly2_chain).
struct poly2_f32 { float v; };
constexpr int kPolyRaw = 8;

template <typename T>
constexpr bool is_bf16 = std::is_same<T, bf16_t>::value || std::is_same<T, feat_bf16>::value;
template <typename T>
constexpr bool is_poly = std::is_same<T, poly2_f32>::value;
template <typename T>
constexpr bool is_feat = std::is_same<T, feat_f32>::value || std::is_same<T, feat_bf16>::value || is_poly<T>;
// elements per token of a Q or K tensor (and of dQ, dK) whose feature width is F
template <typename T> __host__ __device__ constexpr int qk_width(int F) { return is_poly<T> ? kPolyRaw : F; }

// feature value of a raw element of Q or K: eq. 7, or the element itself when the caller has
// applied the map; and the slope of the map recovered from the feature value
template <typename T> __device__ __forceinline__ float feature(float x) {
    if constexpr (is_feat<T>) return x;
    else return phi(x);
}
template <typename T> __device__ __forceinline__ float feature_slope(float f) {
    if constexpr (is_feat<T>) return 1.0f;
    else return dphi_from_phi(f);
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }
__device__ __forceinline__ float to_f32(feat_f32 x) { return x.v; }
__device__ __forceinline__ float to_f32(feat_bf16 x) { return __uint_as_float(((uint32_t)x.bits) << 16); }
__device__ __forceinline__ float to_f32(poly2_f32 x) { return x.v; }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {      // round to nearest even
    return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));     // v_cvt_pk_bf16_f32
}

template <typename T> __device__ __forceinline__ void store_elem(T *p, float v);
// The outputs are written once and not read again inside a step, so the fp32 stores are marked
// non-temporal (the lines need not stay in the caches).  Measured on MI355X at B=2, H=8, N=65536:
// the kernel that follows a storing one reads faster (the segment sums 0.096 instead of 0.116 ms),
// the step 2.4 % faster, the non-causal step 4 %.  The two-byte bf16 stores stay plain: marked
// non-temporal they make the non-causal backward 20 % slower.  Loads are plain unless the caller
// of the kernel asks otherwise (PassArgs::stream).
#ifndef LA_NT_STORES
#define LA_NT_STORES 1
#endif
#ifndef LA_NT_LOADS
#define LA_NT_LOADS 1
#endif
template <> __device__ __forceinline__ void store_elem<float>(float *p, float v) {
    if constexpr (LA_NT_STORES != 0) __builtin_nontemporal_store(v, p);
    else *p = v;
}
template <> __device__ __forceinline__ void store_elem<bf16_t>(bf16_t *p, float v) {
    p->bits = f32_to_bf16_bits(v);
}
template <> __device__ __forceinline__ void store_elem<feat_f32>(feat_f32 *p, float v) { p->v = v; }
template <> __device__ __forceinline__ void store_elem<poly2_f32>(poly2_f32 *p, float v) {
    store_elem(reinterpret_cast<float *>(p), v);
}
template <> __device__ __forceinline__ void store_elem<feat_bf16>(feat_bf16 *p, float v) {
    p->bits = f32_to_bf16_bits(v);
}

// four consecutive floats of a state (written by the kernel before, read once per workgroup:
// a plain load, so that it is found in the cache)
__device__ __forceinline__ f32x4 load4_state(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }

// four consecutive elements, 16-byte (fp32) or 8-byte (bf16) aligned
__device__ __forceinline__ f32x4 load4(const float *p) {
    if constexpr (LA_NT_LOADS != 0) return __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
    else return *reinterpret_cast<const f32x4 *>(p);
}
__device__ __forceinline__ f32x4 load4(const bf16_t *p) {
    const uint2 u = *reinterpret_cast<const uint2 *>(p);
    f32x4 r;
    r[0] = __uint_as_float(u.x << 16);
    r[1] = __uint_as_float(u.x & 0xffff0000u);
    r[2] = __uint_as_float(u.y << 16);
    r[3] = __uint_as_float(u.y & 0xffff0000u);
    return r;
}
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

// What one fetch leaves in a lane's staging registers: the four elements as they are in memory.
// bf16 elements are widened when the tile is parked, not at the load: widening there would make
// the wave wait for the data right behind the fetch, a whole chunk before it is needed.
template <typename T> struct Staged { using type = f32x4; };
template <> struct Staged<bf16_t> { using type = u32x2_t; };
template <> struct Staged<feat_bf16> { using type = u32x2_t; };
template <typename T> using staged_t = typename Staged<T>::type;
__device__ __forceinline__ f32x4 widen(f32x4 v) { return v; }
__device__ __forceinline__ f32x4 widen(u32x2_t u) {
    f32x4 r;
    r[0] = __uint_as_float(u[0] << 16);
    r[1] = __uint_as_float(u[0] & 0xffff0000u);
    r[2] = __uint_as_float(u[1] << 16);
    r[3] = __uint_as_float(u[1] & 0xffff0000u);
    return r;
}
// kNt: non-temporal (the tensors of a call that streams more than the caches hold) or plain
template <bool kNt> __device__ __forceinline__ u32x2_t load4_staged(const bf16_t *p) {
    if constexpr (kNt && LA_NT_LOADS != 0) return __builtin_nontemporal_load(reinterpret_cast<const u32x2_t *>(p));
    else return *reinterpret_cast<const u32x2_t *>(p);
}
template <bool kNt> __device__ __forceinline__ u32x2_t load4_staged(const feat_bf16 *p) {
    return load4_staged<kNt>(reinterpret_cast<const bf16_t *>(p));
}
__device__ __forceinline__ f32x4 load4(const feat_f32 *p) {
    return load4(reinterpret_cast<const float *>(p));
}
__device__ __forceinline__ f32x4 load4(const feat_bf16 *p) {
    return load4(reinterpret_cast<const bf16_t *>(p));
}
__device__ __forceinline__ f32x4 load4(const poly2_f32 *p) {
    return load4(reinterpret_cast<const float *>(p));
}
template <bool kNt> __device__ __forceinline__ f32x4 load4_staged(const float *p) {
    if constexpr (kNt) return load4(p);
    else return *reinterpret_cast<const f32x4 *>(p);
}
template <bool kNt> __device__ __forceinline__ f32x4 load4_staged(const feat_f32 *p) {
    return load4_staged<kNt>(reinterpret_cast<const float *>(p));
}
template <bool kNt> __device__ __forceinline__ f32x4 load4_staged(const poly2_f32 *p) {
    return load4_staged<kNt>(reinterpret_cast<const float *>(p));
}

// ---- wave-level helpers ---------------------------------------------------------------------
// A wave is viewed as 4 groups (g = lane / 16) of 16 lanes (c = lane % 16).
__device__ __forceinline__ float sum_over_groups(float v) {          // over g, result in all lanes
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

// Sum over the 16 lanes of a group (same g), result in all 16: four rotate-and-add steps on
// the DPP path (row_ror 8, 4, 2, 1), no LDS traffic.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row_sum16(float v) {
    v += dpp_move<0x128>(v);
    v += dpp_move<0x124>(v);
    v += dpp_move<0x122>(v);
    v += dpp_move<0x121>(v);
    return v;
}

// D = A * B + C for one 16x16 tile, contraction depth 4.  Lane (c, g) supplies
// A[c][g] and B[g][c]; register r of the accumulator holds C[4g + r][c].
__device__ __forceinline__ f32x4 mfma16(float a, float b, f32x4 acc) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc, 0, 0, 0);
}

// bf16 tensors: the same tile products on `v_mfma_f32_16x16x16_bf16`.  Lane (c, g) supplies
// A[c][4g + j] and B[4g + j][c], j = 0..3, packed as four bf16; the accumulator layout is that of
// the fp32 instruction.  One such MFMA is the sum over r (or s) of four mfma16 calls, with the
// operands rounded to bf16 (round to nearest even) and the products accumulated in fp32.
typedef short bf16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x4_t pack_bf16x4(float a, float b, float c, float d) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const f32x2 lo = {a, b}, hi = {c, d};
    const u32x2 u = {__builtin_bit_cast(unsigned, __builtin_convertvector(lo, bf16x2)),
                     __builtin_bit_cast(unsigned, __builtin_convertvector(hi, bf16x2))};
    return __builtin_bit_cast(bf16x4_t, u);
}
__device__ __forceinline__ bf16x4_t pack_bf16x4(const float (&x)[4]) {
    return pack_bf16x4(x[0], x[1], x[2], x[3]);
}
__device__ __forceinline__ bf16x4_t pack_bf16x4(f32x4 x) { return pack_bf16x4(x[0], x[1], x[2], x[3]); }
__device__ __forceinline__ f32x4 mfma16_bf16(bf16x4_t a, bf16x4_t b, f32x4 acc) {
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, acc, 0, 0, 0);
}

// fp32 products on the bf16 matrix pipe, to fp32 accuracy.  Every fp32 value is cut into three
// bf16 parts, x = h + m + l exactly: h is x rounded to 8 significant bits, m the remainder
// rounded to 8 bits, l the rest (it fits 8 bits).  A product keeps the six part products down to
// 2^-16 of its size (hh, hm, mh, hl, lh, mm; what is dropped is below 2^-23), and
// `v_mfma_f32_16x16x32_bf16` takes two part products per instruction: its 32 contraction slots
// are the 16 of a 16x16x16 tile twice, with any pair of parts on the two halves.  Lane (c, g)
// supplies the same four values per operand as for four mfma16 calls; three instructions of 16
// cycles replace four of 32, and they leave the vector pipe free.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
struct Split3 {
    u32x2_t h, m, l;        // four bf16 each, element j in the low / high half of word j / 2
};
// Two fp32 values -> their bf16 roundings (round to nearest even) packed in one word, and the
// exact remainders.  The rounding is one instruction for the pair (v_cvt_pk_bf16_f32); each
// remainder x - h is one v_dot2c_f32_bf16: h . (-1, -0) + x picks the low element of the pair,
// h . (-0, -1) + x the high one.  Both products and the sum are exact (x and its rounding differ
// by a value that fits fp32), so no masking, shifting or unpacking is needed.  (The zeros are
// negative so that neither constant is one the assembler can encode as an inline operand.)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned round_pair(float a, float b) {
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2_t{a, b}, bf16x2_t));
}
__device__ __forceinline__ float minus_low(unsigned pair, float x) {
    const bf16x2_t sel = {(__bf16)-1.0f, (__bf16)-0.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pair), sel, x, false);
}
__device__ __forceinline__ float minus_high(unsigned pair, float x) {
    const bf16x2_t sel = {(__bf16)-0.0f, (__bf16)-1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pair), sel, x, false);
}
__device__ __forceinline__ Split3 split3(const float (&x)[4]) {
    Split3 s;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const unsigned h = round_pair(x[2 * j], x[2 * j + 1]);
        const float r0 = minus_low(h, x[2 * j]), r1 = minus_high(h, x[2 * j + 1]);
        const unsigned m = round_pair(r0, r1);
        s.h[j] = h;
        s.m[j] = m;
        s.l[j] = round_pair(minus_low(m, r0), minus_high(m, r1));     // what is left has <= 8 bits
    }
    return s;
}
__device__ __forceinline__ bf16x8_t cat_parts(u32x2_t lo, u32x2_t hi) {
    return __builtin_bit_cast(bf16x8_t, u32x4_t{lo[0], lo[1], hi[0], hi[1]});
}
// The operand pairs of the two sides of a product, built once per operand quad and reused over
// the other side's tiles.  Each side keeps its parts in one run of registers and the instructions
// take windows of it.  (The compiler gives every window registers of its own, so each part that
// sits in two windows costs a copy: the layouts below have one such part per run.)
//   P = 3 (fp32 accuracy): both sides hold [l h m] (windows l|h and h|m): A(l|h) B(h|m) is
//         lh + hm, A(h|m) B(l|h) is hl + mh, A(h|m) B(h|m) is hh + mm: the six products.
//   P = 2 (x ~ h + m, 16 significant bits, for bf16 tensors whose results are rounded to 8):
//         side A holds [h m], side B holds [h h m 0] (windows h|h, h|m, m|0): hh + mh and hm
//         are the three products, two instructions.  (Measured: [h m h] with windows h|m and
//         m|h, which adds the product mm, makes the bf16 dV + dK kernel 3 % slower.)
typedef unsigned u32x6_t __attribute__((ext_vector_type(6)));
typedef unsigned u32x8_t __attribute__((ext_vector_type(8)));
template <int P> struct SplitA;
template <int P> struct SplitB;
#define LA_WINDOW(name, v, i0)                                                                 \
    __device__ __forceinline__ bf16x8_t name() const {                                          \
        return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(v, v, i0, i0 + 1, i0 + 2, i0 + 3)); \
    }
template <> struct SplitA<3> {
    u32x6_t v;
    LA_WINDOW(lh, v, 0)
    LA_WINDOW(hm, v, 2)
};
template <> struct SplitB<3> {
    u32x6_t v;
    LA_WINDOW(lh, v, 0)
    LA_WINDOW(hm, v, 2)
};
template <> struct SplitA<2> {
    u32x4_t v;
    LA_WINDOW(hm, v, 0)
};
template <> struct SplitB<2> {
    u32x8_t v;
    LA_WINDOW(hh, v, 0)
    LA_WINDOW(hm, v, 2)
    LA_WINDOW(m0, v, 4)
};
#undef LA_WINDOW

// x ~ h + m: x rounded to 8 significant bits and the remainder rounded to 8 bits (16 bits in all)
struct Split2 {
    u32x2_t h, m;
};
__device__ __forceinline__ Split2 split2(const float (&x)[4]) {
    Split2 s;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const unsigned h = round_pair(x[2 * j], x[2 * j + 1]);
        s.h[j] = h;
        s.m[j] = round_pair(minus_low(h, x[2 * j]), minus_high(h, x[2 * j + 1]));
    }
    return s;
}

// N quads cut into two parts stage by stage (all first roundings, then all remainders, then the
// second roundings), so that an instruction and the one that needs its result are several
// instructions apart (a remainder right behind its rounding costs idle cycles).
template <int N>
__device__ __forceinline__ void split2_batch(const f32x4 (&q)[N], Split2 (&s)[N]) {
    float r[N][4];
#pragma unroll
    for (int n = 0; n < N; ++n)
#pragma unroll
        for (int j = 0; j < 2; ++j) s[n].h[j] = round_pair(q[n][2 * j], q[n][2 * j + 1]);
#pragma unroll
    for (int n = 0; n < N; ++n)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            r[n][2 * j] = minus_low(s[n].h[j], q[n][2 * j]);
            r[n][2 * j + 1] = minus_high(s[n].h[j], q[n][2 * j + 1]);
        }
#pragma unroll
    for (int n = 0; n < N; ++n)
#pragma unroll
        for (int j = 0; j < 2; ++j) s[n].m[j] = round_pair(r[n][2 * j], r[n][2 * j + 1]);
}

__device__ __forceinline__ SplitA<2> as_a(const Split2 &s) {
    return SplitA<2>{u32x4_t{s.h[0], s.h[1], s.m[0], s.m[1]}};
}
__device__ __forceinline__ SplitB<2> as_b(const Split2 &s) {
    return SplitB<2>{u32x8_t{s.h[0], s.h[1], s.h[0], s.h[1], s.m[0], s.m[1], 0u, 0u}};
}
template <int P> __device__ __forceinline__ SplitA<P> split_a(const float (&x)[4]) {
    if constexpr (P == 3) {
        const Split3 s = split3(x);
        return SplitA<3>{u32x6_t{s.l[0], s.l[1], s.h[0], s.h[1], s.m[0], s.m[1]}};
    } else {
        return as_a(split2(x));
    }
}
template <int P> __device__ __forceinline__ SplitB<P> split_b(const float (&x)[4]) {
    if constexpr (P == 3) {
        const Split3 s = split3(x);
        return SplitB<3>{u32x6_t{s.l[0], s.l[1], s.h[0], s.h[1], s.m[0], s.m[1]}};
    } else {
        return as_b(split2(x));
    }
}
template <int P> __device__ __forceinline__ SplitB<P> split_b(f32x4 x) {
    const float q[4] = {x[0], x[1], x[2], x[3]};
    return split_b<P>(q);
}
__device__ __forceinline__ f32x4 mfma32_bf16(bf16x8_t a, bf16x8_t b, f32x4 acc) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
}
// acc + sum over the four contraction steps of a * b: the small terms first
__device__ __forceinline__ f32x4 mfma16_split(const SplitA<3> &a, const SplitB<3> &b, f32x4 acc) {
    acc = mfma32_bf16(a.lh(), b.hm(), acc);    // lh + hm
    acc = mfma32_bf16(a.hm(), b.lh(), acc);    // hl + mh
    acc = mfma32_bf16(a.hm(), b.hm(), acc);    // hh + mm
    return acc;
}
__device__ __forceinline__ f32x4 mfma16_split(const SplitA<2> &a, const SplitB<2> &b, f32x4 acc) {
    acc = mfma32_bf16(a.hm(), b.m0(), acc);    // hm
    acc = mfma32_bf16(a.hm(), b.hh(), acc);    // hh + mh
    return acc;
}
// the same product with the sides exchanged: `x` (kept in side-B form) is the first operand of
// the MFMA, `u` (kept in side-A form) the second
__device__ __forceinline__ f32x4 mfma16_split_ba(const SplitB<3> &x, const SplitA<3> &u, f32x4 acc) {
    acc = mfma32_bf16(x.lh(), u.hm(), acc);    // lh + hm
    acc = mfma32_bf16(x.hm(), u.lh(), acc);    // hl + mh
    acc = mfma32_bf16(x.hm(), u.hm(), acc);    // hh + mm
    return acc;
}
__device__ __forceinline__ f32x4 mfma16_split_ba(const SplitB<2> &x, const SplitA<2> &u, f32x4 acc) {
    acc = mfma32_bf16(x.m0(), u.hm(), acc);    // mh
    acc = mfma32_bf16(x.hh(), u.hm(), acc);    // hh + hm
    return acc;
}
template <int P> __device__ __forceinline__ SplitA<P> split_a(f32x4 x) {
    const float q[4] = {x[0], x[1], x[2], x[3]};
    return split_a<P>(q);
}
// acc + mask * b for a mask of zeros and ones (exact in bf16), four bf16 per lane in `mk`
__device__ __forceinline__ f32x4 mfma16_mask(u32x2_t mk, const SplitB<3> &b, f32x4 acc) {
    acc = mfma32_bf16(cat_parts(mk, mk), b.lh(), acc);                  // mask (l + h)
    acc = mfma32_bf16(cat_parts(u32x2_t{0u, 0u}, mk), b.hm(), acc);     // mask m
    return acc;
}
__device__ __forceinline__ f32x4 mfma16_mask(u32x2_t mk, const SplitB<2> &b, f32x4 acc) {
    return mfma32_bf16(cat_parts(mk, mk), b.hm(), acc);                 // mask (h + m)
}

// An operand quad whose values are exact in bf16 (V of a bf16 tensor, widened to fp32 when the
// tile was parked): it has no second part, so the product against a two-part operand is the two
// halves of one instruction, (h + m) * v, where the general two-part product takes two.
struct ExactBf16 {
    u32x2_t v;
};
__device__ __forceinline__ ExactBf16 exact_bf16(const float (&x)[4]) {
    return ExactBf16{__builtin_bit_cast(u32x2_t, pack_bf16x4(x))};
}
__device__ __forceinline__ f32x4 mfma16_split(const ExactBf16 &a, const SplitB<2> &b, f32x4 acc) {
    return mfma32_bf16(cat_parts(a.v, a.v), b.hm(), acc);
}
__device__ __forceinline__ f32x4 mfma16_split(const SplitA<2> &a, const ExactBf16 &b, f32x4 acc) {
    return mfma32_bf16(a.hm(), cat_parts(b.v, b.v), acc);
}
__device__ __forceinline__ f32x4 mfma16_split_ba(const ExactBf16 &x, const SplitA<2> &u, f32x4 acc) {
    return mfma32_bf16(cat_parts(x.v, x.v), u.hm(), acc);
}

// ---- tiles ------------------------------------------------------------------------------------
// A tile is 16 consecutive tokens x F features of one [N, F] slab, F in {32, 64}.
//
// Fetch: the tile is one contiguous run of 16*F elements.  Load i of lane l takes the four
// elements starting at 4*(l + 64*i): a wave reads 1 KiB (fp32) of consecutive memory per
// instruction.  Rows at or beyond `nvalid` are redirected to the last valid row, so every
// address stays inside the tensor without a branch; park_tile() zeroes them afterwards.
template <int F> __device__ __forceinline__ int stage_row(int lane, int i) { return (4 * (lane + 64 * i)) / F; }
template <int F> __device__ __forceinline__ int stage_col(int lane, int i) { return (4 * (lane + 64 * i)) % F; }

// kFull: all 16 rows exist (the common case): no clamping.  `ts` is the distance between
// consecutive tokens in elements: F when the sequence is contiguous ([B, H, N, F] tensors, the
// tile is then one run of 16 * F elements), H * F for [B, N, H, F] tensors.
// kNt: the call streams its tensors (see PassArgs::stream)
template <int F, bool kFull, bool kNt, typename T>
__device__ __forceinline__ void stage_load(const T *base, int ts, int nvalid, int lane, staged_t<T> (&st)[F / 16]) {
    const T *lane_base = base + (size_t)stage_row<F>(lane, 0) * ts + stage_col<F>(lane, 0);
#pragma unroll
    for (int i = 0; i < F / 16; ++i) {
        if constexpr (kFull) {
            st[i] = load4_staged<kNt>(lane_base + (size_t)(i * (256 / F)) * ts);
        } else {
            const int row = min(stage_row<F>(lane, i), nvalid - 1);
            st[i] = load4_staged<kNt>(base + (size_t)row * ts + stage_col<F>(lane, i));
        }
    }
}


// A 16 x 64 tile of phi(Q) or phi(K) for the degree-2 polynomial map: `base` points at the 8
// raw values of the tile's first token, rows are `ts` elements apart.  The lane that stages
// features col .. col + 3 of a row (col = 4 * (lane % 16), the same assignment as stage_load<64>)
// needs x_i with i = col / 8 and x_j for j = col % 8 .. + 3: one scalar and one 16-byte load.
template <bool kFull, typename T>
__device__ __forceinline__ void stage_load_poly2(const T *base, int ts, int nvalid, int lane, f32x4 (&st)[4]) {
    const int i = (lane & 15) >> 1, j0 = 4 * (lane & 1);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int row = kFull ? stage_row<64>(lane, k) : min(stage_row<64>(lane, k), nvalid - 1);
        const T *p = base + (size_t)row * ts;
        st[k] = to_f32(p[i]) * load4(p + j0);
    }
}
// fetch of a Q or K tile: the plain tile, or the expanded one
template <int F, bool kFull, bool kNt, typename T>
__device__ __forceinline__ void stage_load_qk(const T *base, int ts, int nvalid, int lane, staged_t<T> (&st)[F / 16]) {
    if constexpr (is_poly<T>) {
        static_assert(F == 64, "the degree-2 map of 8 raw values has 64 features");
        stage_load_poly2<kFull>(base, ts, nvalid, lane, st);
    } else {
        stage_load<F, kFull, kNt>(base, ts, nvalid, lane, st);
    }
}
// the 8 raw values of token min(lane / 4, nvalid - 1) of the tile (for poly2_chain)
template <typename T>
__device__ __forceinline__ void load_raw8(const T *base, int ts, int nvalid, int lane, float (&x)[kPolyRaw]) {
    const T *p = base + (size_t)min(lane >> 2, nvalid - 1) * ts;
    const f32x4 a = load4(p), b = load4(p + 4);
#pragma unroll
    for (int j = 0; j < 4; ++j) x[j] = a[j], x[4 + j] = b[j];
}

// per-token fp32 scalars (1/den) of the rows a lane stages
template <int F, bool kFull>
__device__ __forceinline__ void stage_rows(const float *base, int nvalid, int lane, float (&sc)[F / 16]) {
#pragma unroll
    for (int i = 0; i < F / 16; ++i)
        sc[i] = base[kFull ? stage_row<F>(lane, i) : min(stage_row<F>(lane, i), nvalid - 1)];
}

// four per-token fp32 scalars of tokens 4g + s, zero past the end
template <bool kFull>
__device__ __forceinline__ void rows4(const float *base, int nvalid, int g, float (&x)[4]) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const float v = base[kFull ? 4 * g + s : min(4 * g + s, nvalid - 1)];
        x[s] = (kFull || (4 * g + s) < nvalid) ? v : 0.f;
    }
}

// LDS image of a tile: row-major with 4 floats of padding per row.  With that stride the
// 16-byte token-lane reads, the 4-byte feature-lane reads and the 16-byte parking writes
// all spread over the banks without conflicts (for F = 32 and F = 64 alike).
__host__ __device__ constexpr int tile_stride(int F) { return F + 4; }
__host__ __device__ constexpr int tile_floats(int F) { return 16 * (F + 4); }

__device__ __forceinline__ void lds_store4(float *p, f32x4 v) { *reinterpret_cast<f32x4 *>(p) = v; }

// The two operand layouts of a 16x16x4 MFMA:
// token-lane:   lane (c, g) holds token c, features 16*ft + 4g + r   -> x[ft][r]
//               (operand whose non-contracted index is the token; contraction step
//               (ft, r) pairs feature 16*ft + 4g + r on both sides)
// feature-lane: lane (c, g) holds feature 16*ft + c of tokens 4g + s -> x[ft][s]
//               (operand whose non-contracted index is the feature; contraction step s
//               pairs token 4g + s on both sides)
template <int F>
__device__ __forceinline__ void lds_token_lane(const float *tile, int c, int g, float (&x)[F / 16][4]) {
    const float *p = tile + c * tile_stride(F) + 4 * g;
#pragma unroll
    for (int ft = 0; ft < F / 16; ++ft) {
        const f32x4 v = *reinterpret_cast<const f32x4 *>(p + 16 * ft);
#pragma unroll
        for (int r = 0; r < 4; ++r) x[ft][r] = v[r];
    }
}

template <int F>
__device__ __forceinline__ void lds_feature_lane(const float *tile, int c, int g, float (&x)[F / 16][4]) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const float *p = tile + (4 * g + s) * tile_stride(F) + c;
#pragma unroll
        for (int ft = 0; ft < F / 16; ++ft) x[ft][s] = p[16 * ft];
    }
}

// Chain rule of x -> vec(x x^T) for one 16-token tile.  `out` is the gradient for the 64
// features in the accumulator layout (lane (c, g), register r of out[zt]: token 4g + r, feature
// 16zt + c); d(x_i x_j)/dx_k = delta_ik x_j + delta_jk x_i gives
//   dx_k = sum_j (dphi[8k + j] + dphi[8j + k]) x_j.
// The tile goes through `scratch` (16 rows of tile_stride(64) floats, private to the calling
// wave, which both writes and reads it: LDS operations of one wave execute in order); lane
// (t = lane / 4, p = lane % 4) returns dx[t][2p] and dx[t][2p + 1]; `x` holds the raw vector of
// token t (load_raw8).
__device__ __forceinline__ void poly2_chain(float *scratch, const f32x4 (&out)[4], const float (&x)[kPolyRaw],
                                            int lane, float &g0, float &g1) {
    const int c = lane & 15, g = lane >> 4;
#pragma unroll
    for (int zt = 0; zt < 4; ++zt)
#pragma unroll
        for (int r = 0; r < 4; ++r) scratch[(4 * g + r) * tile_stride(64) + 16 * zt + c] = out[zt][r];
    __builtin_amdgcn_wave_barrier();
    const float *row = scratch + (lane >> 2) * tile_stride(64);
    const int k0 = 2 * (lane & 3);
    float acc[2] = {0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int k = k0 + kk;
        const f32x4 a = *reinterpret_cast<const f32x4 *>(row + 8 * k);
        const f32x4 b = *reinterpret_cast<const f32x4 *>(row + 8 * k + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[kk] = fmaf(a[j] + row[8 * j + k], x[j], acc[kk]);
            acc[kk] = fmaf(b[j] + row[8 * (j + 4) + k], x[j + 4], acc[kk]);
        }
    }
    __builtin_amdgcn_wave_barrier();     // the next tile's writes stay behind these reads
    g0 = acc[0], g1 = acc[1];
}

}  // namespace la
