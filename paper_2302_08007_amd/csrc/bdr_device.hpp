// Device-side building blocks shared by the gfx950 kernels of this library.
//
// Everything here works on FP32 bit patterns.  A BF16 input is widened first
// (bits << 16), which is exact, so one code path serves both input types.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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
//  - one 16-byte load per lane (BF16) is the same either way;
//  - FP32 output written as two 16-byte stores per lane must be plain stores
//    (streaming partial-line stores halve the write rate);
//  - the small packed planes do best with the streaming hint.
#ifndef BDR_EXP_NT_LOAD
#define BDR_EXP_NT_LOAD 0
#endif
#ifndef BDR_EXP_NT_CODES
#define BDR_EXP_NT_CODES 1
#endif
#ifndef BDR_EXP_NT_OUT
#define BDR_EXP_NT_OUT 0
#endif
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

// Two dwords at a dword-aligned (not 8-byte-aligned) address, as one access.
__device__ __forceinline__ void store_pair_a4(uint32_t a, uint32_t b, void *p)
{
    u32x2_a4 v = {a, b};
    if (BDR_EXP_NT_CODES)
        __builtin_nontemporal_store(v, reinterpret_cast<u32x2_a4 *>(p));
    else
        *reinterpret_cast<u32x2_a4 *>(p) = v;
}
__device__ __forceinline__ void load_pair_a4(const void *p, uint32_t &a, uint32_t &b)
{
#if defined(BDR_EXP_DEQ_TWO)
    a = reinterpret_cast<const uint32_t *>(p)[0];
    b = reinterpret_cast<const uint32_t *>(p)[1];
#elif defined(BDR_EXP_DEQ_NT)
    u32x2_a4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2_a4 *>(p));
    a = v.x;
    b = v.y;
#else
    u32x2_a4 v = *reinterpret_cast<const u32x2_a4 *>(p);
    a = v.x;
    b = v.y;
#endif
}

// Load 8 consecutive elements as FP32 bit patterns.
__device__ __forceinline__ void load8(const float *p, uint32_t (&xb)[8])
{
    const u32x4 *q = reinterpret_cast<const u32x4 *>(p);
    u32x4 a = ldg<BDR_EXP_NT_LOAD>(q);
    u32x4 b = ldg<BDR_EXP_NT_LOAD>(q + 1);
    xb[0] = a.x; xb[1] = a.y; xb[2] = a.z; xb[3] = a.w;
    xb[4] = b.x; xb[5] = b.y; xb[6] = b.z; xb[7] = b.w;
}

__device__ __forceinline__ void load8(const uint16_t *p, uint32_t (&xb)[8])
{
    u32x4 a = ldg<true>(reinterpret_cast<const u32x4 *>(p));
    xb[0] = a.x << 16; xb[1] = a.x & 0xffff0000u;
    xb[2] = a.y << 16; xb[3] = a.y & 0xffff0000u;
    xb[4] = a.z << 16; xb[5] = a.z & 0xffff0000u;
    xb[6] = a.w << 16; xb[7] = a.w & 0xffff0000u;
}

// Store 8 consecutive FP32 bit patterns as the output type.  For BF16 the low
// halves are dropped; callers only use it where those are zero.
__device__ __forceinline__ void store8(float *p, const uint32_t (&yb)[8])
{
    u32x4 *q = reinterpret_cast<u32x4 *>(p);
    u32x4 a = {yb[0], yb[1], yb[2], yb[3]};
    u32x4 b = {yb[4], yb[5], yb[6], yb[7]};
    stg<BDR_EXP_NT_OUT>(a, q);
    stg<BDR_EXP_NT_OUT>(b, q + 1);
}

__device__ __forceinline__ void store8(uint16_t *p, const uint32_t (&yb)[8])
{
    u32x4 a = {(yb[0] >> 16) | (yb[1] & 0xffff0000u), (yb[2] >> 16) | (yb[3] & 0xffff0000u),
               (yb[4] >> 16) | (yb[5] & 0xffff0000u), (yb[6] >> 16) | (yb[7] & 0xffff0000u)};
    __builtin_nontemporal_store(a, reinterpret_cast<u32x4 *>(p));
}

}  // namespace bdr
