// Device-side building blocks shared by the gfx950 kernels of this library.
//
// Everything here works on FP32 bit patterns.  A BF16 input is widened first
// (bits << 16), which is exact, so one code path serves both input types.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bdr_mx.h"

namespace bdr {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// 8-byte vector that is only dword aligned: global memory takes multi-dword
// accesses at any dword boundary.
typedef uint32_t u32x2_a4 __attribute__((ext_vector_type(2), aligned(4)));

constexpr uint32_t kAbsMask = 0x7fffffffu;
constexpr uint32_t kExpMask = 0x7f800000u;
// Magnitudes are clamped into [2^-126, FLT_MAX] before their exponent field is
// read: zero and subnormals then carry exponent code 1, Inf and NaN carry 254.
constexpr uint32_t kMagLo = 0x00800000u;
constexpr uint32_t kMagHi = 0x7f7fffffu;
constexpr float kMagic = 8388608.0f;  // 2^23: adding it rounds to an integer, ties to even

// DPP lane selectors (dpp_ctrl encodings).
constexpr int kQuadXor1 = 0xB1;  // quad_perm:[1,0,3,2]
constexpr int kQuadXor2 = 0x4E;  // quad_perm:[2,3,0,1]
constexpr int kQuadNext = 0xF9;  // quad_perm:[1,2,3,3]  lane i reads lane i+1 of its quad
constexpr int kQuadPrev = 0x90;  // quad_perm:[0,0,1,2]  lane i reads lane i-1 of its quad
constexpr int kRowHalfMirror = 0x141;
constexpr int kRowMirror = 0x140;

template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }

// Exponent-clamped magnitude of a pair / of one value.
__device__ __forceinline__ uint32_t clamp_mag(uint32_t a) { return umin(umax(a, kMagLo), kMagHi); }

// (a & mask) | (b & ~mask)
__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b)
{
    return (a & mask) | (b & ~mask);
}

// low 32 bits of ({hi,lo} >> s), 0 <= s < 32
__device__ __forceinline__ uint32_t funnel_r(uint32_t hi, uint32_t lo, uint32_t s)
{
    return __builtin_amdgcn_alignbit(hi, lo, s);
}

__device__ __forceinline__ float as_f(uint32_t b) { return __uint_as_float(b); }
__device__ __forceinline__ uint32_t as_u(float f) { return __float_as_uint(f); }

// Cache hints, chosen by measurement on MI355X (1 GiB tensors):
//  - a lane's two adjacent 16-byte FP32 loads do best as plain loads (with the
//    streaming hint the second one is fetched again);
//  - one 16-byte access per lane (BF16 rows, FP32 with 4 elements per lane) is
//    best with the streaming hint;
//  - FP32 output written as two 16-byte stores per lane must be plain stores
//    (streaming partial-line stores halve the write rate);
//  - the small packed planes do best with the streaming hint.
constexpr bool kNtPairLoad = false;
constexpr bool kNtPairStore = false;
constexpr bool kNtPlanes = true;

template <bool NT, typename V>
__device__ __forceinline__ V ldg(const V *p)
{
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}
template <bool NT, typename V>
__device__ __forceinline__ void stg(V v, V *p)
{
    if (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

// ------------------------------------------------------------------ MX core
//
// Quantize the 2*NP consecutive elements one lane holds of a Table II block
// (k1 16, k2 2, d2 1, nearest-even, MB magnitude bits).  The block spans
// 16 / (2*NP) adjacent lanes (XL = log2 of that: 0, 1 or 2); its maximum is
// combined across them with DPP quad permutes.
//
//   w     the lane's 2*NP codes packed little-endian, MB+1 bits each
//   se    biased shared exponent of the block (Sec. IX: exponent of the maximum)
//   tau   one bit per pair: 1 when the pair's largest exponent is below se
//   yb    (DEQ only) bit patterns of the dequantized values
//
// Instruction economy, because these kernels are only ~2x away from VALU-bound:
//   - pair maximum and the lower exponent clamp are one v_max3_u32;
//   - |x| * 2^sh, min with 2^m - 1 and + 2^23 (round to nearest-even integer)
//     are three VALU ops; the 2^23 bias in every term is removed once per word by
//     starting the word at minus the sum of the biases, so a magnitude is packed
//     with a single shift-add;
//   - sign bits are OR-ed into a second accumulator (shift, and-or); for 8-bit
//     codes they are instead gathered four at a time with byte permutes.
template <int MB, int NP>
struct MxWords {
    static constexpr int kCB = MB + 1;
    static constexpr int kN = (2 * NP * kCB + 31) / 32;
};

constexpr uint32_t kMagicBits = 0x4B000000u;  // bit pattern of 2^23

// sum over the non-straddling elements of word k of (2^23 bits << shift), mod 2^32
template <int MB, int NP>
__device__ __forceinline__ constexpr uint32_t mx_bias(int k)
{
    uint32_t b = 0;
    for (int i = 0; i < 2 * NP; ++i) {
        const int off = i * (MB + 1);
        if ((off >> 5) == k && (off & 31) + (MB + 1) <= 32) b += kMagicBits << (off & 31);
    }
    return b;
}

template <int MB, int NP, int XL, bool DEQ>
__device__ __forceinline__ void mx_quant_lane(const uint32_t (&xb)[2 * NP],
                                              uint32_t (&w)[MxWords<MB, NP>::kN], uint32_t &se,
                                              uint32_t &tau, uint32_t (&yb)[2 * NP])
{
    constexpr int CB = MB + 1;
    constexpr int NW = MxWords<MB, NP>::kN;
    constexpr uint32_t MMASK = (1u << MB) - 1u;
    constexpr float TOP = (float)MMASK;

    // pair maxima, clamped below at 2^-126 (exponent code 1 for zero / subnormal)
    uint32_t p[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j)
        p[j] = umax(umax(xb[2 * j] & kAbsMask, xb[2 * j + 1] & kAbsMask), kMagLo);
    uint32_t bm = p[0];
#pragma unroll
    for (int j = 1; j < NP; ++j) bm = umax(bm, p[j]);
    if (XL >= 1) bm = umax(bm, dpp<kQuadXor1>(bm));
    if (XL >= 2) bm = umax(bm, dpp<kQuadXor2>(bm));
    bm = umin(bm, kMagHi);  // Inf / NaN count as exponent code 254
    const uint32_t thr = bm & kExpMask;
    se = bm >> 23;
    const int c0 = (MB - 1) + 127 - (int)se;  // x * 2^c0 puts the block maximum in [2^(m-1), 2^m)
    const int c1 = c0 + 1;

    uint32_t mag[NW], sgn[NW];
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        mag[k] = 0u - mx_bias<MB, NP>(k);
        sgn[k] = 0;
    }
    tau = 0;
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        const bool below = p[j] < thr;  // pair exponent below the shared one: shift by one
        const int sh = below ? c1 : c0;
        tau |= (below ? 1u : 0u) << j;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int i = 2 * j + e;
            const float y =
                __builtin_fminf(__builtin_ldexpf(__builtin_fabsf(as_f(xb[i])), sh), TOP);
            const uint32_t zb = as_u(y + kMagic);  // 2^23 bits + nearest-even integer
            const int off = i * CB, k = off >> 5, s = off & 31;
            if (s + CB <= 32) {
                mag[k] += zb << s;
                if (CB != 8) sgn[k] |= (xb[i] >> (31 - s - MB)) & (1u << (s + MB));
            } else {  // code straddles two words: place a clean copy in both
                const uint32_t c = (zb & MMASK) | ((xb[i] >> 31) << MB);
                sgn[k] |= c << s;
                sgn[k + 1] |= c >> (32 - s);
            }
            if (DEQ) {
                const float v = __builtin_ldexpf(as_f(zb) - kMagic, -sh);
                yb[i] = bfi(kAbsMask, as_u(v), xb[i]);
            }
        }
    }
    if (CB == 8) {
        // sign of element i sits at bit 8 i + 7 of its word: gather the top bytes
#pragma unroll
        for (int k = 0; k < NW; ++k) {
            const uint32_t t01 = __builtin_amdgcn_perm(xb[4 * k + 1], xb[4 * k], 0x0c0c0703u);
            const uint32_t t23 = __builtin_amdgcn_perm(xb[4 * k + 3], xb[4 * k + 2], 0x07030c0cu);
            w[k] = bfi(0x80808080u, t01 | t23, mag[k]);
        }
    } else {
#pragma unroll
        for (int k = 0; k < NW; ++k) w[k] = mag[k] | sgn[k];
    }
}


// Two dwords at a dword-aligned (not 8-byte-aligned) address, as one access.
__device__ __forceinline__ void store_pair_a4(uint32_t a, uint32_t b, void *p)
{
    u32x2_a4 v = {a, b};
    if (kNtPlanes)
        __builtin_nontemporal_store(v, reinterpret_cast<u32x2_a4 *>(p));
    else
        *reinterpret_cast<u32x2_a4 *>(p) = v;
}
__device__ __forceinline__ void load_pair_a4(const void *p, uint32_t &a, uint32_t &b)
{
    u32x2_a4 v = *reinterpret_cast<const u32x2_a4 *>(p);
    a = v.x;
    b = v.y;
}

// Load 8 consecutive elements as FP32 bit patterns.
__device__ __forceinline__ void load8(const float *p, uint32_t (&xb)[8])
{
    const u32x4 *q = reinterpret_cast<const u32x4 *>(p);
    u32x4 a = ldg<kNtPairLoad>(q);
    u32x4 b = ldg<kNtPairLoad>(q + 1);
    xb[0] = a.x; xb[1] = a.y; xb[2] = a.z; xb[3] = a.w;
    xb[4] = b.x; xb[5] = b.y; xb[6] = b.z; xb[7] = b.w;
}

// 8 BF16 values (16 bytes) as FP32 bit patterns
__device__ __forceinline__ void widen8(const u32x4 &a, uint32_t (&xb)[8])
{
    xb[0] = a.x << 16; xb[1] = a.x & 0xffff0000u;
    xb[2] = a.y << 16; xb[3] = a.y & 0xffff0000u;
    xb[4] = a.z << 16; xb[5] = a.z & 0xffff0000u;
    xb[6] = a.w << 16; xb[7] = a.w & 0xffff0000u;
}

__device__ __forceinline__ void load8(const uint16_t *p, uint32_t (&xb)[8])
{
    widen8(ldg<true>(reinterpret_cast<const u32x4 *>(p)), xb);
}

// Store 8 consecutive FP32 bit patterns as the output type.  For BF16 the low
// halves are dropped; callers only use it where those are zero.
__device__ __forceinline__ void store8(float *p, const uint32_t (&yb)[8])
{
    u32x4 *q = reinterpret_cast<u32x4 *>(p);
    u32x4 a = {yb[0], yb[1], yb[2], yb[3]};
    u32x4 b = {yb[4], yb[5], yb[6], yb[7]};
    stg<kNtPairStore>(a, q);
    stg<kNtPairStore>(b, q + 1);
}

// A wave's 512 consecutive floats, 8 per lane, written as two fully contiguous
// 1 KiB rows (lane L stores floats 4L.. of each row) instead of two stores with a
// 32-byte lane stride: a store instruction then fills whole 64-byte lines, and the
// L2 takes a quarter of the write requests.  The exchange goes through kWaveStage
// floats of LDS private to the wave; 4 floats of padding after every 64 keep both
// the 32-byte-strided writes and the 16-byte-strided reads free of bank conflicts.
// All 64 lanes must call it; n_left = floats from dst to the end of the tensor.
constexpr int kWaveStage = 512 + 4 * 8;
__device__ __forceinline__ void wave_store512(float *dst, const uint32_t (&yb)[8], int64_t n_left,
                                              float *stage)
{
    const int L = threadIdx.x & 63;
    u32x4 *w = reinterpret_cast<u32x4 *>(stage + 8 * L + 4 * (L >> 3));
    w[0] = u32x4{yb[0], yb[1], yb[2], yb[3]};
    w[1] = u32x4{yb[4], yb[5], yb[6], yb[7]};
    // LDS operations of one wave complete in order; keep the compiler from moving them
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int i = 256 * k + 4 * L;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(stage + i + 4 * (i >> 6));
        if (i < n_left) stg<true>(v, reinterpret_cast<u32x4 *>(dst + i));
    }
    // the staging area may be refilled right away
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// The reverse: two fully contiguous 1 KiB loads per wave, handed out as 8
// consecutive floats per lane (zeros beyond n_left).
__device__ __forceinline__ void wave_load512(const float *src, uint32_t (&xb)[8], int64_t n_left,
                                             float *stage)
{
    const int L = threadIdx.x & 63;
    u32x4 v[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int i = 256 * k + 4 * L;
        v[k] = u32x4{0, 0, 0, 0};
        if (i < n_left) v[k] = ldg<true>(reinterpret_cast<const u32x4 *>(src + i));
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int i = 256 * k + 4 * L;
        *reinterpret_cast<u32x4 *>(stage + i + 4 * (i >> 6)) = v[k];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const u32x4 *r = reinterpret_cast<const u32x4 *>(stage + 8 * L + 4 * (L >> 3));
    const u32x4 a = r[0], b = r[1];
    xb[0] = a.x, xb[1] = a.y, xb[2] = a.z, xb[3] = a.w;
    xb[4] = b.x, xb[5] = b.y, xb[6] = b.z, xb[7] = b.w;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ void store8(uint16_t *p, const uint32_t (&yb)[8])
{
    u32x4 a = {(yb[0] >> 16) | (yb[1] & 0xffff0000u), (yb[2] >> 16) | (yb[3] & 0xffff0000u),
               (yb[4] >> 16) | (yb[5] & 0xffff0000u), (yb[6] >> 16) | (yb[7] & 0xffff0000u)};
    __builtin_nontemporal_store(a, reinterpret_cast<u32x4 *>(p));
}

// One whole MX6 or MX4 block held by one lane, quantized (nearest even) straight into the
// 16-byte chunk the block-scaled FP6 matrix instruction takes as a lane's operand: the 16
// elements as E2M3 codes in dwords 0-2 (element j at bits 6 j .. 6 j + 5), the block's scale
// byte in dword 3 (byte 0 for an A operand, byte 2 for a B operand).  An element +-M 2^(SE - 127
// - tau - (m - 1)) is the E2M3 value (M << sh6) / 8 times 2^(scale - 127):
//   MX6: sh6 = 2 - tau - z, scale = SE - 2 + z, z = (SE == 1)     MX4: sh6 = 3 - tau, scale = SE - 1
// (M 2^-tau has at most 4 significant bits over 5 binades, Sec. III; the top binade of E2M3 is
// needed for M = 15, tau = 0; a block with SE = 1 moves one binade down instead, still exact).
// The quantizer is that of mx_quant_lane: same maxima, same shifts, same rounding.
// The element map (sign, M, tau, z) -> E2M3 code as a table in LDS: index = M | sign << MB |
// tau << (MB + 1) | z << (MB + 2), at most 128 bytes = 32 dwords, one per bank, so look-ups never
// conflict.  Filled by the first threads of a workgroup (a barrier must follow).
template <int MB>
__device__ __forceinline__ void fp6_map_fill(uint8_t *map)
{
    constexpr int CB = MB + 1;
    if (threadIdx.x < (4u << CB)) {
        const uint32_t idx = threadIdx.x;
        const uint32_t mag = idx & ((1u << MB) - 1u), sign = (idx >> MB) & 1u;
        const int tau = (int)((idx >> CB) & 1u), z = (int)(idx >> (CB + 1));
        const int sh = (MB == 4 ? 2 : 3) - tau - z;
        const uint32_t u = sh >= 0 ? mag << sh : 0u;  // element = u / 8, u <= 60 (MX4 has no z)
        // u >= 8: FP32 of u has exponent field 127 + p (p = 3 .. 5) and u's next three bits on top
        // of its fraction; E2M3 wants exponent field p - 2 and those bits
        const uint32_t em = u < 8u ? u : (as_u((float)u) >> 20) - ((127u + 2u) << 3);
        map[idx] = (uint8_t)((sign << 5) | em);
    }
}

template <int MB, bool B_OPERAND>
__device__ __forceinline__ u32x4 mx_quant_fp6_block(const uint32_t (&xb)[16], const uint8_t *map)
{
    static_assert(MB == 4 || MB == 2, "MX6 or MX4");
    constexpr uint32_t MMASK = (1u << MB) - 1u;
    constexpr float TOP = (float)MMASK;
    uint32_t p[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
        p[j] = umax(umax(xb[2 * j] & kAbsMask, xb[2 * j + 1] & kAbsMask), kMagLo);
    uint32_t bm = p[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) bm = umax(bm, p[j]);
    bm = umin(bm, kMagHi);
    const uint32_t thr = bm & kExpMask;
    const int se = (int)(bm >> 23);
    const int c0 = (MB - 1) + 127 - se, c1 = c0 + 1;
    const int z = (MB == 4 && se == 1) ? 1 : 0;
    const int scale = MB == 4 ? se - 2 + z : se - 1;  // se >= 1: never negative
    uint32_t w[3] = {0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const bool below = p[j] < thr;
        const int sh = below ? c1 : c0;
        const uint32_t tz = ((below ? 1u : 0u) << (MB + 1)) | ((uint32_t)z << (MB + 2));
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int i = 2 * j + e;
            const float y = __builtin_fminf(__builtin_ldexpf(__builtin_fabsf(as_f(xb[i])), sh), TOP);
            const uint32_t mag = as_u(y + kMagic) & MMASK;  // nearest-even integer
            const uint32_t c6 = map[mag | ((xb[i] >> 31) << MB) | tz];
            const int bit = 6 * i;
            w[bit >> 5] |= c6 << (bit & 31);
            if ((bit & 31) + 6 > 32) w[(bit >> 5) + 1] |= c6 >> (32 - (bit & 31));
        }
    }
    return u32x4{w[0], w[1], w[2], (uint32_t)scale << (B_OPERAND ? 16 : 0)};
}

// One whole MX4 block held by one lane, quantized (nearest even) into the 8 bytes the block-scaled
// FP4 matrix instruction takes: 16 E2M1 codes (sign, two exponent bits, one fraction bit: 0, 0.5,
// 1, 1.5, 2, 3, 4, 6), element j at bits 4 j .. 4 j + 3, and the block's scale byte.  An MX4
// element is +-M 2^(SE - 127 - tau - 1) with M <= 3 (Sec. III): M 2^-tau is 0, 0.5, 1, 1.5 (tau =
// 1: code M) or 0, 1, 2, 3 (tau = 0: codes 0, 2, 4, 5), the rest is the scale byte SE - 1.
__device__ __forceinline__ void mx_quant_fp4_block(const uint32_t (&xb)[16], uint32_t &w0, uint32_t &w1,
                                                   uint32_t &scale)
{
    uint32_t p[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
        p[j] = umax(umax(xb[2 * j] & kAbsMask, xb[2 * j + 1] & kAbsMask), kMagLo);
    uint32_t bm = p[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) bm = umax(bm, p[j]);
    bm = umin(bm, kMagHi);
    const uint32_t thr = bm & kExpMask;
    const int se = (int)(bm >> 23);
    const int c0 = 1 + 127 - se, c1 = c0 + 1;
    scale = (uint32_t)(se - 1);  // se >= 1
    uint32_t w[2] = {0u, 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const bool below = p[j] < thr;
        const int sh = below ? c1 : c0;
        // the code of magnitude M as nibble M (tau = 0) or 4 + M (tau = 1) of one constant
        const uint32_t lut = below ? 0x3210u : 0x5420u;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int i = 2 * j + e;
            const float y = __builtin_fminf(__builtin_ldexpf(__builtin_fabsf(as_f(xb[i])), sh), 3.0f);
            const uint32_t mag = as_u(y + kMagic) & 3u;  // nearest-even integer
            const uint32_t c4 = ((lut >> (4u * mag)) & 7u) | ((xb[i] >> 28) & 8u);
            w[i >> 3] |= c4 << (4 * (i & 7));
        }
    }
    w0 = w[0];
    w1 = w[1];
}

// One whole Table II block held by one lane, quantized (nearest even) and written out as its 16
// dequantized values in BF16 (exact: m + 1 <= 8 significant bits), two per dword: the 32 bytes
// the block takes in the BF16 operand image of the product kernel.
template <int MB>
__device__ __forceinline__ void mx_quant_bf16_block(const uint32_t (&xb)[16], u32x4 &lo, u32x4 &hi)
{
    uint32_t ww[MxWords<MB, 8>::kN], se, tau8, yb[16];
    mx_quant_lane<MB, 8, 0, true>(xb, ww, se, tau8, yb);
    uint32_t w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) w[j] = __builtin_amdgcn_perm(yb[2 * j + 1], yb[2 * j], 0x07060302u);
    lo = u32x4{w[0], w[1], w[2], w[3]};
    hi = u32x4{w[4], w[5], w[6], w[7]};
}

// A format tuple as the general (run-time-tuple) kernels take it.
struct GenFmt {
    int k1, k2, d2, m, rounding;
};

// |x| * 2^sh rounded to an integer in [0, top] by the format's rule.
__device__ __forceinline__ float gen_round(float ax, int sh, float top, int rounding)
{
    float y = __builtin_fminf(__builtin_ldexpf(ax, sh), top);
    if (rounding == BDR_RNE) return __builtin_rintf(y);
    const float t = __builtin_truncf(y);
    if (rounding == BDR_RNA) return (y - t) >= 0.5f ? t + 1.0f : t;
    return t;
}

// Formats the general kernels are also compiled for with the tuple as a compile-time
// constant (SPEC = index into this table; SPEC < 0 = tuple at run time): the formats of the
// design-space sweep of Sec. IV around Table II -- k1 8 .. 64, k2 1, 2, 4 or k1, d2 0 or 1,
// m 2 or 4, nearest-even.  d2 = 0 is listed once per (k1, m) with k2 = k1 (k2 plays no part
// then); Table II's own members have kernels of their own.  With the tuple known, every
// loop over group sizes unrolls and every shift is an immediate, which is what the
// run-time-format kernels spend their time on.
constexpr int kHotK1[4] = {8, 16, 32, 64};
constexpr int kHotM[2] = {2, 4};
constexpr int kHotCount = 4 * 2 * 5;  // per (k1, m): d2 = 0, then d2 = 1 with k2 = 1, 2, 4, k1
__host__ __device__ constexpr GenFmt hot_format(int spec)
{
    const int k1 = kHotK1[spec / 10], m = kHotM[(spec / 5) % 2], v = spec % 5;
    return GenFmt{k1, v == 0 || v == 4 ? k1 : 1 << (v - 1), v == 0 ? 0 : 1, m, BDR_RNE};
}
// index of a format in the table, or -1
static inline int hot_index(const bdr_format &f)
{
    for (int sp = 0; sp < kHotCount; ++sp) {
        const GenFmt h = hot_format(sp);
        if (f.k1 == h.k1 && f.m == h.m && f.d2 == h.d2 && f.rounding == h.rounding &&
            (f.d2 == 0 || f.k2 == h.k2))
            return sp;
    }
    return -1;
}

}  // namespace bdr
