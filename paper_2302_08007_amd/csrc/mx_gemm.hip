// C = Ahat * Bhat^T on MX-quantized operands (Sec. V: both inputs of a tensor
// operation are MX-quantized along the reduction dimension).
//
// A is the packed image of an [M x K] tensor, B of an [N x K] tensor, both
// blocked along K.  A workgroup owns a BM x BN tile of C and walks K in steps of
// 64: every thread pulls the packed bits of 32 elements of A and 32 of B (two
// blocks each) from global memory, expands them exactly to BF16 (a BF16 has 8
// significant bits, an MX element at most 7, and the scale is a power of two),
// and writes them to LDS; the waves then feed 32x32x16 BF16 MFMAs from LDS and
// accumulate in FP32.  Global loads for the next K step are issued before the
// MFMAs of the current one, and LDS is double buffered, so one barrier per step.
//
// The expansion, not the MFMA, is what this kernel is bound by (about 6.5 VALU
// operations per operand element against 32 matrix-pipe cycles per MFMA), so the
// tile is as large as LDS allows (256 x 256: every operand element is expanded
// once per 256 columns or rows of C) and the expansion is kept lean: field
// extract, integer-to-float, ldexp, sign insert, and one byte permute per pair to
// form the BF16 pair.
//
// That is the single-kernel form (mx_gemm_kernel).  The two-pass form rewrites each
// operand once in global memory, tiled along K, and runs gemm_ring_kernel on the two
// images: BF16 images when MX9 takes part; images of FP6 elements with one scale byte per
// block for MX6 / MX4, which the block-scaled matrix instruction of gfx950 multiplies at
// twice the BF16 rate (mx_to_fp6_kernel and the notes above it); images of FP4 elements
// for MX4 x MX4 (mx_to_fp4_kernel).  Formats outside Table II go through the general
// dequantize kernel and gemm_dl_kernel (row-major BF16).
//
// None of this is the dot-product engine of Sec. IV-B (integer Hadamard tree with
// a conditional shift and fixed-point accumulation): that design targets a custom
// datapath.  The FP6 form is the nearest thing this chip offers: small-integer
// elements under a shared power-of-two scale that the hardware applies.
#include <type_traits>
#include <utility>

#include "bdr_device.hpp"
#include "bdr_internal.hpp"

namespace bdr {

namespace {

constexpr int kBK = 64;
constexpr int kPitch = kBK * 2;  // bytes per LDS row: 64 BF16 = eight 16-byte chunks
// LDS rows are 128 bytes = half of the 64 banks, so rows of equal parity put the
// same chunk on the same banks.  A 16-byte access is served 16 lanes at a time, and
// the 16 lanes of a fragment read hold 16 consecutive rows: chunk c of row r is
// stored at position c ^ ((r >> 1) & 7), which gives each row pair its own
// position and leaves the two rows of a pair on opposite halves of the banks.
__device__ __forceinline__ int lds_chunk(int row, int chunk)
{
    return row * kPitch + ((chunk ^ ((row >> 1) & 7)) << 4);
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
// the same in LDS (address space 3: 32-bit addresses, ds_read instructions)
typedef __attribute__((address_space(3))) uint8_t lds_u8;
typedef __attribute__((address_space(3))) i32x4 lds_i32x4;
typedef __attribute__((address_space(3))) i32x2 lds_i32x2;
typedef __attribute__((address_space(3))) u32x2 lds_u32x2;
typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef uint32_t u32x3_a4 __attribute__((ext_vector_type(3), aligned(4)));
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));

// The packed bits one thread needs for 32 consecutive elements (two blocks) of a row.
template <int MB>
struct Packed {
    uint32_t c[MB + 1];   // 32 codes x (MB+1) bits = MB+1 dwords
    uint32_t se2, tau16;  // two exponent bytes, two microexponent bytes
};

template <int MB>
__device__ __forceinline__ void load_packed(const uint8_t *__restrict__ codes,
                                            const uint8_t *__restrict__ sexp,
                                            const uint8_t *__restrict__ mexp, int64_t blk,
                                            Packed<MB> &p)
{
    constexpr int CB = MB + 1;
    const uint8_t *cp = codes + blk * (2 * CB);  // a block is 16 * CB / 8 bytes
    if constexpr (CB == 8) {
        const u32x4 a = *reinterpret_cast<const u32x4 *>(cp);
        const u32x4 b = *reinterpret_cast<const u32x4 *>(cp + 16);
        p.c[0] = a.x; p.c[1] = a.y; p.c[2] = a.z; p.c[3] = a.w;
        p.c[4] = b.x; p.c[5] = b.y; p.c[6] = b.z; p.c[7] = b.w;
    } else if constexpr (CB == 5) {
        const u32x4_a4 a = *reinterpret_cast<const u32x4_a4 *>(cp);
        p.c[0] = a.x; p.c[1] = a.y; p.c[2] = a.z; p.c[3] = a.w;
        p.c[4] = *reinterpret_cast<const uint32_t *>(cp + 16);
    } else {
        const u32x3_a4 a = *reinterpret_cast<const u32x3_a4 *>(cp);
        p.c[0] = a.x; p.c[1] = a.y; p.c[2] = a.z;
    }
    p.se2 = *reinterpret_cast<const uint16_t *>(sexp + blk);
    p.tau16 = *reinterpret_cast<const uint16_t *>(mexp + blk);
}

// Expand the 32 elements to BF16, two per word.
// value = (-1)^s * M * 2^(se - 127 - tau - (MB-1)); ldexp makes it exact for every
// exponent, subnormal results included.
template <int MB>
__device__ __forceinline__ void unpack32(const Packed<MB> &p, uint32_t (&out)[16])
{
    constexpr int CB = MB + 1;
    int qb[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) qb[b] = (int)((p.se2 >> (8 * b)) & 0xffu) - (127 + MB - 1);
#pragma unroll
    for (int j = 0; j < 16; ++j) {  // pair j: elements 2j, 2j+1, one microexponent bit
        const int q = qb[j >> 3] - (int)((p.tau16 >> j) & 1u);
        uint32_t h[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int off = (2 * j + e) * CB;
            const int k = off >> 5;
            int s = off & 31;
            uint32_t win = p.c[k];
            if constexpr (CB != 8) {
                if (s + CB > 32) {  // the code straddles two words: funnel it down to bit 0
                    win = funnel_r(p.c[(k + 1) % CB], p.c[k], s);
                    s = 0;
                }
            }
            const float f = __builtin_ldexpf((float)((win >> s) & ((1u << MB) - 1u)), q);
            h[e] = bfi(kAbsMask, as_u(f), win << (31 - s - MB));  // sign bit from the code
        }
        // the two high halves (exact: the low halves are zero) as one BF16 pair
        out[j] = __builtin_amdgcn_perm(h[1], h[0], 0x07060302u);
    }
}

// The same for MX9 with fewer instructions (its codes are whole bytes): the magnitudes of four
// codes are converted by the byte-to-float instructions (the compiler's choice for these casts), scaled by a multiplication (exact:
// a power of two times at most 7 significant bits, subnormal results included), and the signs of a
// pair are moved from the code bytes into the packed BF16 pair by one byte permute and one and-or.
__device__ __forceinline__ void unpack32_mx9(const Packed<7> &p, uint32_t (&out)[16])
{
    float sc[2][2];  // 2^(se - 127 - 6 - tau) for tau = 0, 1 of each block
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int q = (int)((p.se2 >> (8 * b)) & 0xffu) - (127 + 6);
        sc[b][0] = __builtin_ldexpf(1.0f, q);
        sc[b][1] = __builtin_ldexpf(1.0f, q - 1);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {  // dword k: codes of elements 4k .. 4k+3 = pairs 2k, 2k+1
        const uint32_t c = p.c[k], m = c & 0x7f7f7f7fu;
        const float s0 = ((p.tau16 >> (2 * k)) & 1u) ? sc[k >> 2][1] : sc[k >> 2][0];
        const float s1 = ((p.tau16 >> (2 * k + 1)) & 1u) ? sc[k >> 2][1] : sc[k >> 2][0];
        const uint32_t f0 = as_u((float)(m & 0xffu) * s0), f1 = as_u((float)((m >> 8) & 0xffu) * s0);
        const uint32_t f2 = as_u((float)((m >> 16) & 0xffu) * s1), f3 = as_u((float)(m >> 24) * s1);
        // BF16 pair = the two high halves; signs: code byte 0 -> byte 1 of the pair, code byte 1 -> byte 3
        const uint32_t lo = __builtin_amdgcn_perm(f1, f0, 0x07060302u), hi = __builtin_amdgcn_perm(f3, f2, 0x07060302u);
        out[2 * k] = (__builtin_amdgcn_perm(c, c, 0x010c000cu) & 0x80008000u) | lo;
        out[2 * k + 1] = (__builtin_amdgcn_perm(c, c, 0x030c020cu) & 0x80008000u) | hi;
    }
}

// ... and store them as chunks 4*half .. 4*half+3 of LDS row `row` of the operand tile at `base`.
template <int MB>
__device__ __forceinline__ void unpack_to_lds(const Packed<MB> &p, uint8_t *base, int row, int half)
{
    uint32_t out[16];
    unpack32<MB>(p, out);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const u32x4 w = {out[4 * v], out[4 * v + 1], out[4 * v + 2], out[4 * v + 3]};
        *reinterpret_cast<u32x4 *>(base + lds_chunk(row, 4 * half + v)) = w;
    }
}

// Write the TM x TN accumulator tiles of a wave.  32 x 32 accumulator: register r of lane l
// is row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32.  Tiles on the lower or right edge
// of C may hang over it (M, N need not be multiples of the tile): those check every element.
// C is FP32, or BF16 when c_bf16 is set: each sum is then rounded once more, to nearest even
// (what a BF16 element-wise consumer of the product would do itself, Sec. V).
__device__ __forceinline__ uint16_t bf16_rne(float v)
{
    const uint32_t u = as_u(v);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

template <int TM, int TN>
__device__ __forceinline__ void store_tiles(const f32x16 (&acc)[TM][TN], void *__restrict__ C,
                                            int64_t ldc, int c_bf16, int M, int N, int row0, int col0,
                                            int lane, bool inside)
{
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = col0 + j * 32 + (lane & 31);
            const int row = row0 + i * 32 + 4 * (lane >> 5);
            if (c_bf16) {  // uniform
                uint16_t *cp = static_cast<uint16_t *>(C) + (int64_t)row * ldc + col;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = 8 * (r >> 2) + (r & 3);
                    if (inside || (row + dr < M && col < N))
                        __builtin_nontemporal_store(bf16_rne(acc[i][j][r]), cp + (int64_t)dr * ldc);
                }
            } else {
                float *cp = static_cast<float *>(C) + (int64_t)row * ldc + col;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = 8 * (r >> 2) + (r & 3);
                    if (inside || (row + dr < M && col < N))
                        __builtin_nontemporal_store(acc[i][j][r], cp + (int64_t)dr * ldc);
                }
            }
        }
}

// 256 x 256 tiles are taken only when there are enough of them for the chip's 256 CUs: a call with
// 48 or 96 of them (M = 256 or 512 against N = 12288) runs 2 and 1.2-1.7 times faster on 128 x 128
// tiles; from 144 on the large tile wins.
constexpr int64_t kBigTileMin = 128;

// WM x WN waves, each computing TM x TN MFMA tiles of 32 x 32.
template <int MBA, int MBB, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(64 * WM * WN) void mx_gemm_kernel(
    const uint8_t *__restrict__ a_codes, const uint8_t *__restrict__ a_sexp,
    const uint8_t *__restrict__ a_mexp, const uint8_t *__restrict__ b_codes,
    const uint8_t *__restrict__ b_sexp, const uint8_t *__restrict__ b_mexp, int M, int N, int K,
    void *__restrict__ C, int64_t ldc, int c_bf16)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr int THREADS = 64 * WM * WN;
    constexpr int A_BYTES = BM * kPitch, B_BYTES = BN * kPitch;
    constexpr int PA = 2 * BM / THREADS, PB = 2 * BN / THREADS;  // unpack passes per thread
    static_assert(PA >= 1 && PB >= 1 && 2 * BM % THREADS == 0 && 2 * BN % THREADS == 0, "tile");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];  // [2][A | B]

    // Tile order: workgroup ids go round-robin over the 8 XCDs, each with its own
    // L2, so give every XCD a contiguous range of tiles and walk that range in
    // groups of 8 tile rows per tile column to keep the operands of a group hot.
    const int ntm = (M + BM - 1) / BM, ntn = (N + BN - 1) / BN, total = ntm * ntn;
    int t = blockIdx.x;
    if (total % 8 == 0) t = (t % 8) * (total / 8) + t / 8;
    int tm, tn;
    if (ntm % 8 == 0) {
        const int group = t / (8 * ntn);
        tm = group * 8 + t % 8;
        tn = (t % (8 * ntn)) / 8;
    } else {
        tm = t / ntn;
        tn = t % ntn;
    }
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // unpack role: row tid/2 (+ THREADS/2 per pass), elements 32*(tid&1) .. +31 of the K step
    const int urow = tid >> 1, uhalf = tid & 1;
    const int64_t kblocks = K >> 4;
    int64_t a_blk[PA], b_blk[PB];
#pragma unroll
    for (int i = 0; i < PA; ++i)  // rows past the edge of an operand repeat its last row (never stored)
        a_blk[i] = (int64_t)min(m0 + urow + i * (THREADS / 2), M - 1) * kblocks + 2 * uhalf;
#pragma unroll
    for (int i = 0; i < PB; ++i)
        b_blk[i] = (int64_t)min(n0 + urow + i * (THREADS / 2), N - 1) * kblocks + 2 * uhalf;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Packed operands live in two register sets: while step kt is multiplied and
    // step kt+1 (already in registers) is expanded into the other LDS buffer, the
    // loads of step kt+2 are in flight.  A whole K step hides their latency.
    Packed<MBA> pa[2][PA];
    Packed<MBB> pb[2][PB];
    const int nk = K / kBK;

    auto load_step = [&](int set) {  // advances the block pointers by one K step
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            load_packed<MBA>(a_codes, a_sexp, a_mexp, a_blk[i], pa[set][i]);
            a_blk[i] += 4;
        }
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            load_packed<MBB>(b_codes, b_sexp, b_mexp, b_blk[i], pb[set][i]);
            b_blk[i] += 4;
        }
    };
    auto unpack_step = [&](int set, uint8_t *dst) {
#pragma unroll
        for (int i = 0; i < PA; ++i)
            unpack_to_lds<MBA>(pa[set][i], dst, urow + i * (THREADS / 2), uhalf);
#pragma unroll
        for (int i = 0; i < PB; ++i)
            unpack_to_lds<MBB>(pb[set][i], dst + A_BYTES, urow + i * (THREADS / 2), uhalf);
    };
    // fragment addresses: lane l feeds row l % 32, k offset 8 * (l / 32) of a 32 x 16 slab
    const int f_row = lane & 31, f_half = lane >> 5;
    auto mfma_step = [&](const uint8_t *cur) {
#pragma unroll
        for (int s = 0; s < kBK / 16; ++s) {
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const bf16x8 *>(
                    cur + lds_chunk((wm * TM + i) * 32 + f_row, 2 * s + f_half));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const bf16x8 *>(
                    cur + A_BYTES + lds_chunk((wn * TN + j) * 32 + f_row, 2 * s + f_half));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    };
    uint8_t *const buf0 = smem, *const buf1 = smem + A_BYTES + B_BYTES;

    load_step(0);
    unpack_step(0, buf0);
    if (nk > 1) load_step(0);  // step 1 waits in set 0
    __syncthreads();

    int kt = 0;
    // two K steps per trip so that register sets and LDS buffers have fixed names
    for (; kt + 3 < nk; kt += 2) {
        load_step(1);           // step kt+2
        mfma_step(buf0);        // step kt
        unpack_step(0, buf1);   // step kt+1
        __syncthreads();
        load_step(0);           // step kt+3
        mfma_step(buf1);        // step kt+1
        unpack_step(1, buf0);   // step kt+2
        __syncthreads();
    }
    // at most three steps left: kt (in buf0), kt+1 (in set 0), kt+2 (not loaded yet)
    if (kt + 2 < nk) load_step(1);
    mfma_step(buf0);
    if (kt + 1 < nk) {
        unpack_step(0, buf1);
        __syncthreads();
        mfma_step(buf1);
        if (kt + 2 < nk) {
            unpack_step(1, buf0);
            __syncthreads();
            mfma_step(buf0);
        }
    }

    store_tiles<TM, TN>(acc, C, ldc, c_bf16, M, N, m0 + wm * TM * 32, n0 + wn * TN * 32, lane,
                        m0 + BM <= M && n0 + BN <= N);
}

// The block-scaled FP6 MFMA of gfx950 multiplies E2M3 elements (sign, 2 exponent bits,
// 3 fraction bits: m / 8 for exponent field 0, else (1 + m / 8) 2^(e - 1)) and applies
// one power-of-two scale (a byte b meaning 2^(b - 127)) per lane, i.e. per 32 elements of
// K.  An MX6 or MX4 element is +-M 2^(SE - 127 - tau - (m - 1)) with M < 2^m, tau <= 1
// (Sec. III): M 2^-tau has at most 4 significant bits and spans 5 binades, which E2M3
// holds exactly, and the rest is a power of two per block of 16 that fits the scale
// byte.  The hardware block is 32 long and k1 is 16, so each lane gets one block in the
// lower half of its 32 values and zeros in the upper half.
//
// This kernel rewrites the three planes of an operand as one 16-byte chunk per block:
// dwords 0-2 hold the 16 FP6 codes (element j at bits 6 j .. 6 j + 5), dword 3 holds
// the scale byte.  The MFMA reads dword 3 both as the scale operand and as elements
// 16 .. 21 of the lane (which must contribute nothing): an A operand keeps its scale in
// byte 0 (bits of elements 16, 17), a B operand in byte 2 (elements 18, 19), so each
// of those products has a zero factor.  FP6 has no infinities or NaNs, so 0 * x = 0.
//   MX6: element = (M << (2 - tau - z)) / 8, scale byte = SE - 2 + z, z = (SE == 1)
//        (the top binade of E2M3 is needed for M = 15, tau = 0, which leaves SE - 2; a
//        block with SE = 1 moves its elements one binade down instead, still exact)
//   MX4: element = (M << (3 - tau)) / 8,     scale byte = SE - 1
constexpr int kFp6 = 2;  // operand format selector of the f8f6f4 MFMA: E2M3
constexpr int kScaleByteA = 0, kScaleByteB = 2;

template <int MB, bool B_OPERAND>
__global__ __launch_bounds__(256) void mx_to_fp6_kernel(const uint8_t *__restrict__ codes,
                                                        const uint8_t *__restrict__ sexp,
                                                        const uint8_t *__restrict__ mexp,
                                                        int64_t n_pairs, int rows, int row_pairs,
                                                        u32x4 *__restrict__ out)
{
    static_assert(MB == 4 || MB == 2, "MX6 or MX4");
    constexpr int CB = MB + 1;
    // The element map as a table in LDS: index = code | tau << CB | z << (CB + 1), value =
    // the FP6 code.  It spans at most 32 dwords, one per bank, so look-ups never conflict.
    __shared__ uint8_t s_map[4 << CB];
    if (threadIdx.x < (4u << CB)) {
        const uint32_t idx = threadIdx.x;
        const uint32_t mag = idx & ((1u << MB) - 1u), sign = (idx >> MB) & 1u;
        const int tau = (int)((idx >> CB) & 1u), z = (int)(idx >> (CB + 1));
        const int sh = (MB == 4 ? 2 : 3) - tau - z;
        const uint32_t u = sh >= 0 ? mag << sh : 0u;  // element = u / 8, u <= 60 (MX4 has no z)
        // u >= 8: FP32 of u has exponent field 127 + p (p = 3 .. 5) and u's next three
        // bits on top of its fraction; E2M3 wants exponent field p - 2 and those bits
        const uint32_t em = u < 8u ? u : (as_u((float)u) >> 20) - ((127u + 2u) << 3);
        s_map[idx] = (uint8_t)((sign << 5) | em);
    }
    __syncthreads();
    // Two blocks per thread; n_pairs = rows * row_pairs.  The image is tiled along K for the
    // product kernel: [K step of 4 blocks][row][4 chunks].
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= n_pairs) return;
    const int64_t row = p / row_pairs;
    const int q = (int)(p - row * row_pairs);
    u32x4 *const dst = out + (((int64_t)(q >> 1) * rows + row) * 4 + 2 * (q & 1));
    Packed<MB> pk;
    load_packed<MB>(codes, sexp, mexp, 2 * p, pk);
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int se = (int)((pk.se2 >> (8 * b)) & 0xffu);
        const int z = (MB == 4 && se == 1) ? 1 : 0;
        // exponent code 0 is never written by the quantizer (codes are 1 .. 254); it is held
        // at scale byte 0 here rather than wrapped
        const int scale = max(MB == 4 ? se - 2 + z : se - 1, 0);
        uint32_t w[3] = {0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int off = (16 * b + j) * CB;
            const int k = off >> 5;
            int sh = off & 31;
            uint32_t win = pk.c[k];
            if (sh + CB > 32) {  // the code straddles two words
                win = funnel_r(pk.c[(k + 1) % CB], pk.c[k], sh);
                sh = 0;
            }
            const uint32_t tz = (((pk.tau16 >> (8 * b + (j >> 1))) & 1u) << CB) | ((uint32_t)z << (CB + 1));
            const uint32_t c6 = s_map[((win >> sh) & ((1u << CB) - 1u)) | tz];
            const int bit = 6 * j;
            w[bit >> 5] |= c6 << (bit & 31);
            if ((bit & 31) + 6 > 32) w[(bit >> 5) + 1] |= c6 >> (32 - (bit & 31));
        }
        const u32x4 chunk = {w[0], w[1], w[2], (uint32_t)scale << (B_OPERAND ? 8 * kScaleByteB : 8 * kScaleByteA)};
        dst[b] = chunk;
    }
}

// MX4 x MX4 goes one step further.  An MX4 element is +-M 2^(SE - 127 - tau - 1) with
// M <= 3 and tau <= 1: M 2^-tau is one of 0, 0.5, 1, 1.5, 2, 3, all of which the 4-bit E2M1
// format holds (sign, 2 exponent bits, 1 fraction bit: 0, 0.5, 1, 1.5, 2, 3, 4, 6), and the
// rest is 2^(SE - 1 - 127), one scale byte per block.  At 4 bits per element a block is
// 8 bytes, so the image has two blocks per 16-byte chunk and a K step of the product
// kernel covers 256 elements at the same LDS footprint; that halves the bytes the product
// kernel moves per flop, which is what bounds the FP6 form.
//
// Scale bytes no longer ride in the chunk; they form an image of their own, laid out in the
// order the product kernel loads it: [128-row group][K step][row in group][16 bytes], the 16
// bytes being the scales of the step's 8 even blocks and then of its 8 odd blocks (a lane of
// the MFMA serves blocks of one parity).  Rows are padded to whole groups with zero scales.
constexpr int kFp4 = 4;  // operand format selector of the f8f6f4 MFMA: E2M1

__global__ __launch_bounds__(256) void mx_to_fp4_kernel(const uint8_t *__restrict__ codes,
                                                        const uint8_t *__restrict__ sexp,
                                                        const uint8_t *__restrict__ mexp,
                                                        int64_t n_pairs, int rows, int row_pairs,
                                                        int row_pairs_out, u32x4 *__restrict__ out,
                                                        uint8_t *__restrict__ scales)
{
    // index = code (sign << 2 | M) | tau << 3, value = the E2M1 code
    __shared__ uint8_t s_map[16];
    if (threadIdx.x < 16u) {
        const uint32_t idx = threadIdx.x, mag = idx & 3u, sign = (idx >> 2) & 1u, tau = idx >> 3;
        s_map[idx] = (uint8_t)((sign << 3) | (tau ? mag : 2u * mag - (mag == 3u ? 1u : 0u)));
    }
    __syncthreads();
    // One pair of blocks (one chunk) per thread; n_pairs counts the pairs of the padded image
    // (rows brought up to a multiple of 128, K to a whole K step of 8 blocks).  Both images are
    // tiled along K: chunks as [K step][row][4 chunks], scales as [K step][padded row][8 bytes].
    const int64_t po = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (po >= n_pairs) return;
    const int64_t row = po / row_pairs_out;
    const int q = (int)(po - row * row_pairs_out);
    const int64_t rows_pad = ((int64_t)rows + 127) / 128 * 128;
    uint8_t *sc = scales + (((int64_t)(q >> 2) * rows_pad + row) * 8 + (q & 3));
    u32x4 *const dst = out + (((int64_t)(q >> 2) * rows + row) * 4 + (q & 3));
    if (row >= rows || q >= row_pairs) {
        sc[0] = 0;
        sc[4] = 0;
        if (row < rows) *dst = u32x4{0u, 0u, 0u, 0u};
        return;
    }
    Packed<2> pk;
    load_packed<2>(codes, sexp, mexp, 2 * (row * row_pairs + q), pk);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const int off = 3 * j;
        const int k = off >> 5;
        int sh = off & 31;
        uint32_t win = pk.c[k];
        if (sh + 3 > 32) {  // the code straddles two words
            win = funnel_r(pk.c[(k + 1) % 3], pk.c[k], sh);
            sh = 0;
        }
        const uint32_t tau = (pk.tau16 >> (j >> 1)) & 1u;
        w[j >> 3] |= (uint32_t)s_map[((win >> sh) & 7u) | (tau << 3)] << (4 * (j & 7));
    }
    // rows with bit 4 set hold the two blocks of a chunk in swapped order: the 32 lanes of a
    // half wave (32 consecutive rows, one block each) then read 32 different 8-byte slots of LDS
    *dst = (row & 16) ? u32x4{w[2], w[3], w[0], w[1]} : u32x4{w[0], w[1], w[2], w[3]};
    // exponent code 0 is never written by the quantizer; it is held at scale byte 0
    sc[0] = (uint8_t)max((int)(pk.se2 & 0xffu) - 1, 0);
    sc[4] = (uint8_t)max((int)((pk.se2 >> 8) & 0xffu) - 1, 0);
}

// 16 bytes per lane from global memory straight into LDS: lane p's data lands at
// byte 16 p after `lds_block` (which must be the same for the whole wave).
__device__ __forceinline__ void global_to_lds16(const void *src, void *lds_block)
{
#if defined(__HIP_DEVICE_COMPILE__)  // the builtin exists only in the device pass
    __builtin_amdgcn_global_load_lds(src, lds_block, 16, 0, 0);
#else
    (void)src;
    (void)lds_block;
#endif
}

// The same tiling on operands that are already BF16 in memory, row-major ([M x K] and
// [N x K], K contiguous): the second half of the two-pass form for formats outside Table II,
// whose operands the general dequantize kernel expands.  Operands come in by direct
// global-to-LDS loads: a wave fills eight tile rows (1 KiB) per instruction, lane p
// supplying the 16 bytes that belong at byte 16 p of that block, i.e. chunk (p & 7) ^
// swizzle of row p / 8.  No staging registers and no LDS write instructions; two LDS
// stages, the loads of step kt+2 issued right after the barrier that ends step kt, and the
// fragment reads of sub-step s+1 before the MFMAs of sub-step s.  (Table II's formats use
// the ring kernel further down, which keeps more loads in flight.)
constexpr int kFmtBf16 = 0, kFmtFp6 = 1, kFmtFp4 = 2;

template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

template <int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(64 * WM * WN) void gemm_dl_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ B, int M, int N, int K,
    void *__restrict__ C, int64_t ldc, int c_bf16)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr int NW = WM * WN;
    constexpr int A_BYTES = BM * kPitch, B_BYTES = BN * kPitch, kBuf = A_BYTES + B_BYTES;
    constexpr int LA = BM / 8 / NW, LB = BN / 8 / NW;  // 8-row blocks per wave and K step
    constexpr int NSUB = kBK / 16;                     // sub-steps (fragment reads) per K step
    static_assert(LA >= 1 && LB >= 1 && BM % (8 * NW) == 0 && BN % (8 * NW) == 0 && TM % 2 == 0, "tile");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];  // [2][A | B]

    const int ntm = (M + BM - 1) / BM, ntn = (N + BN - 1) / BN, total = ntm * ntn;
    int t = blockIdx.x;
    if (total % 8 == 0) t = (t % 8) * (total / 8) + t / 8;
    int tm, tn;
    if (ntm % 8 == 0) {
        const int group = t / (8 * ntn);
        tm = group * 8 + t % 8;
        tn = (t % (8 * ntn)) / 8;
    } else {
        tm = t / ntn;
        tn = t % ntn;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    // the wave index as a scalar: everything derived from it (LDS destinations of the direct
    // loads, tile offsets) then stays out of the vector ALU
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int nk = K / kBK;

    // Vector-ALU instructions between the MFMAs of the steady-state loop cost matrix-pipe
    // issue slots, so the loop is kept nearly free of them: global addresses are a scalar base
    // that advances per K step plus a fixed 32-bit lane offset; LDS read addresses are computed
    // once per sub-step (all fragments of a lane share the swizzle, rows 32 apart, so fragment
    // i is an immediate offset) and moved between the two buffers with one add per K step.
    const uint8_t *a_base = reinterpret_cast<const uint8_t *>(A + (int64_t)m0 * K);
    const uint8_t *b_base = reinterpret_cast<const uint8_t *>(B + (int64_t)n0 * K);
    uint32_t a_off[LA], b_off[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int row = (wave * LA + i) * 8 + (lane >> 3);
        // rows past the edge of an operand repeat its last row (their products are never stored)
        a_off[i] = (uint32_t)(min(row, M - 1 - m0) * K + 8 * ((lane & 7) ^ ((row >> 1) & 7))) * 2u;
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int row = (wave * LB + i) * 8 + (lane >> 3);
        b_off[i] = (uint32_t)(min(row, N - 1 - n0) * K + 8 * ((lane & 7) ^ ((row >> 1) & 7))) * 2u;
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    auto fill = [&](uint8_t *dst) {  // one K step of both operands, then advance
#pragma unroll
        for (int i = 0; i < LA; ++i) global_to_lds16(a_base + a_off[i], dst + (wave * LA + i) * 8 * kPitch);
#pragma unroll
        for (int i = 0; i < LB; ++i)
            global_to_lds16(b_base + b_off[i], dst + A_BYTES + (wave * LB + i) * 8 * kPitch);
        a_base += kBK * 2;
        b_base += kBK * 2;
    };
    const int f_row = lane & 31, f_half = lane >> 5;
    // LDS byte addresses of this lane's fragment 0 of each sub-step, in the buffer that
    // sub-step is read from next.  A read moves its address to the other buffer: +flip for
    // the sub-steps read from cur, -flip for sub-step 0 (read ahead from nxt), and flip
    // changes sign every K step.
    const uint32_t smem_at = (uint32_t)(uintptr_t)(lds_u8 *)smem;
    uint32_t ra[NSUB], rb[NSUB];
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        const uint32_t pos = smem_at + (uint32_t)(((2 * sub + f_half) ^ ((f_row >> 1) & 7)) << 4);
        ra[sub] = (uint32_t)((wm * TM * 32 + f_row) * kPitch) + pos;
        rb[sub] = (uint32_t)(A_BYTES + (wn * TN * 32 + f_row) * kPitch) + pos;
    }
    int flip = -kBuf;  // the first reads (buffer 0) move on to buffer 1
    using Frag = i32x4;
    auto read_frags = [&](auto S, Frag (&fa)[TM], Frag (&fb)[TN]) {
        constexpr int sub = decltype(S)::value;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[i] = *reinterpret_cast<const lds_i32x4 *>((uintptr_t)(ra[sub] + i * 32 * kPitch));
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[j] = *reinterpret_cast<const lds_i32x4 *>((uintptr_t)(rb[sub] + j * 32 * kPitch));
        ra[sub] += sub == 0 ? -flip : flip;
        rb[sub] += sub == 0 ? -flip : flip;
    };
    auto mfmas = [&](const Frag (&fa)[TM], const Frag (&fb)[TN], int half) {  // half of the tiles
#pragma unroll
        for (int i = half * (TM / 2); i < (half + 1) * (TM / 2); ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, fa[i]), __builtin_bit_cast(bf16x8, fb[j]), acc[i][j], 0, 0, 0);
    };
    // Schedule of one K step (cur holds step kt, nxt is being filled with step kt+1,
    // fragment set 0 holds sub-step 0 of step kt):
    //   reads of sub-step s+1 are issued before the MFMAs of sub-step s, up to the last;
    //   then wait for everything this wave has in flight and meet the other waves:
    //   from here on nxt is complete and nobody reads cur any more (the fragments of
    //   the last sub-step are in registers), so the fill of step kt+2 into cur and the reads
    //   of sub-step 0 of step kt+1 are issued and run under the MFMAs of the last sub-step.
    static_assert(NSUB % 2 == 0, "the last sub-step must leave fragment set 0 free");
    uint8_t *cur = smem, *nxt = smem + kBuf;
    Frag fa[2][TM], fb[2][TN];
    constexpr std::integral_constant<int, 0> first{};
    fill(cur);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (nk > 1) fill(nxt);
    read_frags(first, fa[0], fb[0]);  // from buffer 0; sub-step 0 now points at buffer 1 = nxt
    flip = -flip;
    // One K step.  The last two steps have nothing left to fill or to read ahead; they are
    // peeled so that the body of the steady-state loop is one straight block.
    auto k_step = [&](auto do_fill, auto do_read) {
        static_for<NSUB - 1>([&](auto S) {
            constexpr int s = decltype(S)::value;
            mfmas(fa[s & 1], fb[s & 1], 0);
            __builtin_amdgcn_sched_barrier(0);
            read_frags(std::integral_constant<int, s + 1>{}, fa[(s + 1) & 1], fb[(s + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(fa[s & 1], fb[s & 1], 1);
            __builtin_amdgcn_sched_barrier(0);
        });
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        mfmas(fa[1], fb[1], 0);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (decltype(do_fill)::value) fill(cur);
        if constexpr (decltype(do_read)::value) read_frags(first, fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        mfmas(fa[1], fb[1], 1);
        __builtin_amdgcn_sched_barrier(0);
        flip = -flip;
        uint8_t *t2 = cur;
        cur = nxt;
        nxt = t2;
    };
    for (int kt = 0; kt + 2 < nk; ++kt) k_step(std::true_type{}, std::true_type{});
    if (nk > 1) k_step(std::false_type{}, std::true_type{});
    k_step(std::false_type{}, std::false_type{});
    store_tiles<TM, TN>(acc, C, ldc, c_bf16, M, N, m0 + wm * TM * 32, n0 + wn * TN * 32, lane,
                        m0 + BM <= M && n0 + BN <= N);
}

// Packed Table II planes -> BF16, tiled along K for the ring kernel: [K step of 32
// elements][row][64 bytes].  A workgroup covers 16 rows x 16 K steps.  Thread (row, step)
// reads the packed bits of its 32 elements (per row the 16 steps are consecutive memory) and
// expands them into LDS; then the workgroup writes the 16 KiB out in image order, where each
// K step's 16 rows are 1 KiB of consecutive memory: every store instruction of a wave
// covers whole cache lines.
template <int MB>
__global__ __launch_bounds__(256) void mx_to_bf16_tiled_kernel(const uint8_t *__restrict__ codes,
                                                               const uint8_t *__restrict__ sexp,
                                                               const uint8_t *__restrict__ mexp, int rows,
                                                               int row_pairs, u32x4 *__restrict__ out)
{
    __shared__ u32x4 s_tile[16 * 16 * 4];  // [step][row][4 chunks], chunk c of row r at c ^ ((r >> 2) & 3)
    const int r_l = threadIdx.x & 15, q_l = threadIdx.x >> 4;
    const int row0 = blockIdx.x * 16, q0 = blockIdx.y * 16;
    if (row0 + r_l < rows && q0 + q_l < row_pairs) {
        Packed<MB> pk;
        load_packed<MB>(codes, sexp, mexp, 2 * ((int64_t)(row0 + r_l) * row_pairs + q0 + q_l), pk);
        uint32_t w[16];
        unpack32<MB>(pk, w);
#pragma unroll
        for (int v = 0; v < 4; ++v)
            s_tile[(q_l * 16 + r_l) * 4 + (v ^ ((r_l >> 2) & 3))] =
                u32x4{w[4 * v], w[4 * v + 1], w[4 * v + 2], w[4 * v + 3]};
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int u = it * 256 + threadIdx.x;  // chunk u of the tile in image order
        const int q = u >> 6, r = (u >> 2) & 15, c = u & 3;
        if (row0 + r < rows && q0 + q < row_pairs)
            out[((int64_t)(q0 + q) * rows + row0 + r) * 4 + c] = s_tile[(q * 16 + r) * 4 + (c ^ ((r >> 2) & 3))];
    }
}

// The product on K-tiled images (BF16, or FP6 / FP4 blocks) with a ring of four LDS stages.
//
// With two stages the loads of step kt+1 are all that is in flight while step kt computes,
// and every barrier waits until the last of them has landed: the memory pipeline drains
// once per K step, and at 256 x 256 that drain takes about as long as the MFMAs of the
// step.  Here a stage holds 64 bytes per tile row (half as much), four stages fit the same
// LDS, and the loads of steps kt+1 .. kt+3 are in flight together: the barrier at the end
// of step kt needs only step kt+1 complete (vmcnt counts loads in order, so "at most the
// loads of two steps outstanding" says exactly that).
//
// The images are tiled along K to match: [K step][row][64 bytes], so that the 16 rows one
// wave instruction brings are 1 KiB of consecutive memory (whole cache lines).
//   BF16: 64 bytes = 32 elements = 2 sub-steps of one 32 x 32 x 16 MFMA (chunk 2 s + l / 32)
//   FP6: 64 bytes = 4 blocks = 2 sub-steps (lanes 0-31 take block 2 s, lanes 32-63 block 2 s + 1)
//   FP4: 64 bytes = 8 blocks = 4 sub-steps (chunk s, one 8-byte block per half wave), and a
//        scale image [K step][row padded to 128][8 bytes]: the step's four even-block scales,
//        then its four odd-block scales
// LDS rows are 64 bytes = a quarter of the banks: the 16 lanes served together (16
// consecutive rows) are conflict-free when chunk c of row r sits at position
// c ^ ((r >> 2) & 3).
constexpr int kRingRow = 64, kRingStages = 4;

// Wait until at most N of this wave's vector-memory loads are outstanding and all its LDS
// reads have returned, then meet the other waves.  __syncthreads() would not do: its fences
// wait for every outstanding load, which is exactly the drain the ring is there to avoid.
// The data hazards are covered by hand: a stage is read only after a barrier that every wave
// reached with that stage's loads landed, and refilled only after a barrier that every wave
// reached with its reads of that stage returned.
template <int N>
__device__ __forceinline__ void ring_barrier()
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
#endif
}

template <int WM, int WN, int TM, int TN, int FMT>
__global__ __launch_bounds__(64 * WM * WN) void gemm_ring_kernel(
    const uint8_t *__restrict__ A, const uint8_t *__restrict__ B, const uint8_t *__restrict__ SA,
    const uint8_t *__restrict__ SB, int M, int N, int nk, void *__restrict__ C, int64_t ldc, int c_bf16)
{
    constexpr bool FP6 = FMT == kFmtFp6, FP4 = FMT == kFmtFp4, BF16 = FMT == kFmtBf16;
    static_assert(FP6 || FP4 || BF16, "format");
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr int NW = WM * WN;
    constexpr int A_BYTES = BM * kRingRow, B_BYTES = BN * kRingRow, kStage = A_BYTES + B_BYTES;
    constexpr int kSStage = (BM + BN) * 8;            // FP4: scale bytes of one stage
    constexpr int LA = BM / 16 / NW, LB = BN / 16 / NW;  // 16-row blocks per wave and K step
    constexpr int kLoads = LA + LB;                   // loads per wave and K step (FP4: some waves one more)
    constexpr int NSUB = FP4 ? 4 : 2;
    constexpr int kScaleWaves = (BM + BN) / 128;      // FP4: one 128-row piece of scales per wave
    static_assert(LA >= 1 && LB >= 1 && BM % (16 * NW) == 0 && BN % (16 * NW) == 0 && TM % 2 == 0, "tile");
    static_assert((kStage & (kStage - 1)) == 0 && (kSStage & (kSStage - 1)) == 0, "ring positions wrap with a mask");
    static_assert(BM % 128 == 0 && BN % 128 == 0 && kScaleWaves <= NW, "scale pieces");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];  // [4][A | B], FP4: + [4][SA | SB]

    const int ntm = (M + BM - 1) / BM, ntn = (N + BN - 1) / BN, total = ntm * ntn;
    int t = blockIdx.x;
    if (total % 8 == 0) t = (t % 8) * (total / 8) + t / 8;
    int tm, tn;
    if (ntm % 8 == 0) {
        const int group = t / (8 * ntn);
        tm = group * 8 + t % 8;
        tn = (t % (8 * ntn)) / 8;
    } else {
        tm = t / ntn;
        tn = t % ntn;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // global side: a scalar base per operand that moves one K step (all rows x 64 bytes) at a
    // time, plus a fixed lane offset; lane p of a load brings row p / 4 of its 16-row block,
    // the chunk that belongs at position p % 4 of that row
    const uint8_t *a_base = A + (int64_t)m0 * kRingRow, *b_base = B + (int64_t)n0 * kRingRow;
    const int64_t a_step = (int64_t)M * kRingRow, b_step = (int64_t)N * kRingRow;
    uint32_t a_off[LA], b_off[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int row = (wave * LA + i) * 16 + (lane >> 2);
        // rows past the edge of an operand repeat its last row (their products are never stored)
        a_off[i] = (uint32_t)(min(row, M - 1 - m0) * kRingRow + (((lane & 3) ^ ((row >> 2) & 3)) << 4));
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int row = (wave * LB + i) * 16 + (lane >> 2);
        b_off[i] = (uint32_t)(min(row, N - 1 - n0) * kRingRow + (((lane & 3) ^ ((row >> 2) & 3)) << 4));
    }
    const uint8_t *s_base = nullptr;
    int64_t s_step = 0;
    int s_piece = 0;
    if constexpr (FP4) {
        if (wave < kScaleWaves) {
            const bool is_b = wave >= BM / 128;
            const int piece = is_b ? wave - BM / 128 : wave;
            const int rows_pad = ((is_b ? N : M) + 127) / 128 * 128;
            s_base = (is_b ? SB : SA) + ((int64_t)(is_b ? n0 : m0) + piece * 128) * 8 + lane * 16;
            s_step = (int64_t)rows_pad * 8;
            s_piece = (is_b ? BM * 8 : 0) + piece * 1024;
        }
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // ring positions (byte offsets, scalars): the stage being read and the stage being filled
    int rd = 0, wr = 0, srd = 0, swr = 0;
    auto fill = [&]() {  // one K step of both operands into stage wr, then advance
#pragma unroll
        for (int i = 0; i < LA; ++i) global_to_lds16(a_base + a_off[i], smem + wr + (wave * LA + i) * 16 * kRingRow);
#pragma unroll
        for (int i = 0; i < LB; ++i)
            global_to_lds16(b_base + b_off[i], smem + wr + A_BYTES + (wave * LB + i) * 16 * kRingRow);
        a_base += a_step;
        b_base += b_step;
        if constexpr (FP4) {
            if (wave < kScaleWaves) {
                global_to_lds16(s_base, smem + kRingStages * kStage + swr + s_piece);
                s_base += s_step;
            }
            swr = (swr + kSStage) & (kRingStages * kSStage - 1);
        }
        wr = (wr + kStage) & (kRingStages * kStage - 1);
    };

    const int f_row = lane & 31, f_half = lane >> 5;
    // A fragment is the 16 bytes of one chunk (FP4: the 8 bytes of one block).  The FP6 MFMA
    // takes six registers per operand (FP4: four), of which the upper two hold elements 22-31
    // (16-31) of the lane; those must contribute nothing.  FP6 and FP4 have no infinities or
    // NaNs, so it is enough that ONE factor of each such product is zero: B fragments keep
    // zeros there for the whole kernel (the fragment variables are eight wide and a read
    // replaces only their lower part), A fragments leave those registers undefined.
    using Frag = typename std::conditional<BF16, i32x4, i32x8>::type;
    auto read_frag = [&](uint32_t at, Frag &f, auto keep_zeros) {  // `at`: an LDS byte address
        constexpr bool Z = decltype(keep_zeros)::value;
        if constexpr (BF16) {
            f = *reinterpret_cast<const lds_i32x4 *>((uintptr_t)at);
        } else if constexpr (FP6) {
            const i32x4 v = *reinterpret_cast<const lds_i32x4 *>((uintptr_t)at);
            if constexpr (Z) {
                const i32x8 wide = __builtin_shufflevector(v, v, 0, 1, 2, 3, 0, 1, 2, 3);
                f = __builtin_shufflevector(wide, f, 0, 1, 2, 3, 12, 13, 14, 15);
            } else {
                f = __builtin_shufflevector(v, v, 0, 1, 2, 3, -1, -1, -1, -1);
            }
        } else {
            // volatile: two 8-byte reads fused into one instruction land in one register
            // tuple and would have to be copied apart again
            const i32x2 v = *reinterpret_cast<const volatile lds_i32x2 *>((uintptr_t)at);
            if constexpr (Z) {
                const i32x8 wide = __builtin_shufflevector(v, v, 0, 1, 0, 1, 0, 1, 0, 1);
                f = __builtin_shufflevector(wide, f, 0, 1, 10, 11, 12, 13, 14, 15);
            } else {
                f = __builtin_shufflevector(v, v, 0, 1, -1, -1, -1, -1, -1, -1);
            }
        }
    };
    // LDS byte addresses of this lane's fragment 0 of each sub-step within stage 0 (all
    // fragments of a lane share the swizzle, rows 32 apart: fragment i is an immediate offset)
    const uint32_t smem_at = (uint32_t)(uintptr_t)(lds_u8 *)smem;
    uint32_t ra[NSUB], rb[NSUB];
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        const int chunk = FP4 ? sub : 2 * sub + f_half, byte = FP4 ? 8 * (f_half ^ (f_row >> 4)) : 0;
        const uint32_t pos = smem_at + (uint32_t)(((chunk ^ ((f_row >> 2) & 3)) << 4) + byte);
        ra[sub] = (uint32_t)((wm * TM * 32 + f_row) * kRingRow) + pos;
        rb[sub] = (uint32_t)(A_BYTES + (wn * TN * 32 + f_row) * kRingRow) + pos;
    }
    auto read_frags = [&](auto S, int stage, Frag (&fa)[TM], Frag (&fb)[TN]) {
        constexpr int sub = decltype(S)::value;
        const uint32_t pa = ra[sub] + (uint32_t)stage, pb = rb[sub] + (uint32_t)stage;
#pragma unroll
        for (int i = 0; i < TM; ++i) read_frag(pa + i * 32 * kRingRow, fa[i], std::false_type{});
#pragma unroll
        for (int j = 0; j < TN; ++j) read_frag(pb + j * 32 * kRingRow, fb[j], std::true_type{});
    };
    // FP4: the four scale bytes of this lane's parity of blocks, sub-step s in byte s
    uint32_t sa[TM], sb[TN], sa_next[TM], sb_next[TN];
    const uint32_t sra = smem_at + kRingStages * kStage + (uint32_t)((wm * TM * 32 + f_row) * 8 + 4 * f_half);
    const uint32_t srb = smem_at + kRingStages * kStage + (uint32_t)(BM * 8 + (wn * TN * 32 + f_row) * 8 + 4 * f_half);
    auto read_scales = [&](int sstage, uint32_t (&xa)[TM], uint32_t (&xb)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i) xa[i] = *reinterpret_cast<const lds_u32 *>((uintptr_t)(sra + sstage + i * 32 * 8));
#pragma unroll
        for (int j = 0; j < TN; ++j) xb[j] = *reinterpret_cast<const lds_u32 *>((uintptr_t)(srb + sstage + j * 32 * 8));
    };
    auto mfmas = [&](auto S, const Frag (&fa)[TM], const Frag (&fb)[TN], int half) {  // half of the tiles
        constexpr int sub = decltype(S)::value;
#pragma unroll
        for (int i = half * (TM / 2); i < (half + 1) * (TM / 2); ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if constexpr (BF16) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, fa[i]), __builtin_bit_cast(bf16x8, fb[j]), acc[i][j], 0, 0, 0);
                } else if constexpr (FP6) {
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        fa[i], fb[j], acc[i][j], kFp6, kFp6, kScaleByteA, fa[i][3], kScaleByteB, fb[j][3]);
                } else {
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        fa[i], fb[j], acc[i][j], kFp4, kFp4, sub, (int)sa[i], sub, (int)sb[j]);
                }
            }
    };

    Frag fa[2][TM], fb[2][TN];
    if constexpr (!BF16) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[h][j] = i32x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
    constexpr std::integral_constant<int, 0> first{};
    constexpr std::integral_constant<int, NSUB - 1> last{};
    static_assert(NSUB % 2 == 0, "the last sub-step must leave fragment set 0 free");

    // stages 0 .. 2 go out at once; then wait for stage 0 alone
    fill();
    if (nk > 1) fill();
    if (nk > 2) fill();
    if (nk > 2) ring_barrier<2 * kLoads>();
    else if (nk > 1) ring_barrier<kLoads>();
    else ring_barrier<0>();
    read_frags(first, rd, fa[0], fb[0]);
    if constexpr (FP4) read_scales(srd, sa, sb);

    // One K step (stage rd holds step kt, fragment set 0 its sub-step 0).  AHEAD is the number
    // of later steps whose loads may still be in flight at the barrier that ends this step
    // (-1: this is the last step, no barrier); with FILL the loads of step kt+3 go out first,
    // into the stage that step kt-1 was read from (every wave is past the barrier after it).
    auto k_step = [&](auto FILL, auto AHEAD) {
        constexpr int ahead = decltype(AHEAD)::value;
        static_for<NSUB - 1>([&](auto S) {
            constexpr int s = decltype(S)::value;
            mfmas(S, fa[s & 1], fb[s & 1], 0);
            __builtin_amdgcn_sched_barrier(0);
            read_frags(std::integral_constant<int, s + 1>{}, rd, fa[(s + 1) & 1], fb[(s + 1) & 1]);
            if constexpr (decltype(FILL)::value && s == 0) fill();
            __builtin_amdgcn_sched_barrier(0);
            mfmas(S, fa[s & 1], fb[s & 1], 1);
            __builtin_amdgcn_sched_barrier(0);
        });
        const int next = (rd + kStage) & (kRingStages * kStage - 1);
        const int snext = (srd + kSStage) & (kRingStages * kSStage - 1);
        if constexpr (ahead >= 0) ring_barrier<ahead * kLoads>();
        mfmas(last, fa[1], fb[1], 0);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (ahead >= 0) {
            read_frags(first, next, fa[0], fb[0]);
            if constexpr (FP4) read_scales(snext, sa_next, sb_next);
        }
        __builtin_amdgcn_sched_barrier(0);
        mfmas(last, fa[1], fb[1], 1);
        __builtin_amdgcn_sched_barrier(0);
        rd = next;
        srd = snext;
        if constexpr (FP4 && ahead >= 0) {
#pragma unroll
            for (int i = 0; i < TM; ++i) sa[i] = sa_next[i];
#pragma unroll
            for (int j = 0; j < TN; ++j) sb[j] = sb_next[j];
        }
    };
    int kt = 0;
    for (; kt + 3 < nk; ++kt) k_step(std::true_type{}, std::integral_constant<int, 2>{});
    if (kt + 2 < nk) {
        k_step(std::false_type{}, std::integral_constant<int, 1>{});
        ++kt;
    }
    if (kt + 1 < nk) k_step(std::false_type{}, std::integral_constant<int, 0>{});
    k_step(std::false_type{}, std::integral_constant<int, -1>{});
    store_tiles<TM, TN>(acc, C, ldc, c_bf16, M, N, m0 + wm * TM * 32, n0 + wn * TN * 32, lane,
                        m0 + BM <= M && n0 + BN <= N);
}

// The product for few rows of A (M <= 64: a decoding step, a handful of tokens against a weight
// matrix): one or two MFMA tiles hold all of A's rows, so there is nothing to reuse from LDS and the
// call is a stream over B's image.  A workgroup takes 32 rows of B and all of K; its four waves
// take K steps in turn (wave w the steps w, w + 4, ...), each lane loading its fragments straight
// from the images in the MFMA's own layout (fragment = chunk 2 s + lane / 32 of row lane % 32; FP4:
// see below), so that the waves of a workgroup read B's image as 2 KiB runs.
// Plain loads: a row's 64 bytes arrive as two 32-byte halves in consecutive instructions, and the
// second must find the line the first brought (with the streaming hint the same stream takes 40 %
// longer).  The four partial tiles are added in LDS in a fixed order (the result does not depend
// on timing).  Same images, same scale-byte conventions and the same idle-half trick as
// gemm_ring_kernel.  Measured, N = K = 12288, ten launches back to back: MX6 23-27 us for M = 1
// .. 32 (5.6-6.5 TB/s of B's image) and 37 us for M = 64, MX4 (FP4 images) 16-18 and 27 us, MX9
// (BF16 images) 48-66 and 92 us; the tiled kernel takes 57 / 57 / 112 us for the same calls.
// Waves per workgroup x K steps a wave loads ahead, same order of figures for MX6 M = 1 / MX4 M = 1
// / MX9 M = 64: 4 x 2 23.1 / 16.2 / 92, 4 x 4 24.5 / 18.3 / 100, 8 x 2 25.7 / 17.3 / 97, 8 x 4 25.5
// / 17.5 / 100, 16 x 2 25.8 / 18.3 / 99, deeper or wider than that much worse (registers).  Every workgroup reads all of A again (from L2), which is what M costs; with
// four tiles (M <= 128) the tiled kernel is the faster one (48 against 55-62 us for MX6).
constexpr int kSkinnyWaves = 4, kSkinnyRows = 32, kSkinnyMaxM = 64;

template <int FMT, int TM>
__global__ __launch_bounds__(64 * kSkinnyWaves) void gemm_skinny_kernel(
    const uint8_t *__restrict__ A, const uint8_t *__restrict__ B, const uint8_t *__restrict__ SA,
    const uint8_t *__restrict__ SB, int M, int N, int nk, void *__restrict__ C, int64_t ldc, int c_bf16)
{
    constexpr bool FP6 = FMT == kFmtFp6, FP4 = FMT == kFmtFp4, BF16 = FMT == kFmtBf16;
    constexpr int NSUB = FP4 ? 4 : 2;
    __shared__ float s_red[kSkinnyWaves][16][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n0 = blockIdx.x * kSkinnyRows;
    const int f_row = lane & 31, f_half = lane >> 5;
    // rows past the edge of an operand repeat its last row (their products are never stored)
    const int rb = min(n0 + f_row, N - 1);
    const int64_t a_step = (int64_t)M * kRingRow, b_step = (int64_t)N * kRingRow;
    // A lane loads two 16-byte pieces per K step and operand.  FP6 / BF16: the fragments of the
    // two sub-steps (chunks f_half and 2 + f_half).  FP4: which of a K step's eight blocks meet in
    // which of the four MFMAs is free as long as both operands agree, so the lower half wave takes
    // blocks 0-3 (chunks 0, 1) and the upper one blocks 4-7 (chunks 2, 3): 32 consecutive bytes
    // instead of four 8-byte pieces.
    constexpr int kPiece = FP4 ? 16 : 32;  // from a lane's first piece to its second
    int ra[TM], a_at[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        ra[i] = min(32 * i + f_row, M - 1);
        a_at[i] = ra[i] * kRingRow + (FP4 ? 32 : 16) * f_half;
    }
    const int b_at = rb * kRingRow + (FP4 ? 32 : 16) * f_half;
    const int64_t sa_step = (int64_t)((M + 127) / 128 * 128) * 8, sb_step = (int64_t)((N + 127) / 128 * 128) * 8;
    // FP4: the scale bytes of blocks 4 h + s, s = 0 .. 3, out of the even blocks' and the odd blocks' words
    const uint32_t scale_sel = f_half ? 0x07030602u : 0x05010400u;

    f32x16 acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    // kAhead K steps of a wave are loaded before the first of them is multiplied (enough, with the
    // waves a CU holds, for the bytes in flight a stream needs).  What is loaded is kept as it
    // comes; the MFMA operand is put together at the multiply.
    constexpr int kAhead = 2;
    i32x4 fa[kAhead][TM][2], fb[kAhead][2];
    i32x2 sa[kAhead][TM], sb[kAhead];
    auto load = [&](int q, i32x4 (&xa)[TM][2], i32x4 (&xb)[2], i32x2 (&xsa)[TM], i32x2 &xsb) {
        const uint8_t *ap = A + q * a_step, *bp = B + q * b_step + b_at;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            xb[k] = *reinterpret_cast<const i32x4 *>(bp + k * kPiece);
#pragma unroll
            for (int i = 0; i < TM; ++i) xa[i][k] = *reinterpret_cast<const i32x4 *>(ap + a_at[i] + k * kPiece);
        }
        if constexpr (FP4) {  // a row's eight scale bytes of the step: even blocks' four, odd blocks' four
            xsb = *reinterpret_cast<const i32x2 *>(SB + q * sb_step + (int64_t)rb * 8);
#pragma unroll
            for (int i = 0; i < TM; ++i) xsa[i] = *reinterpret_cast<const i32x2 *>(SA + q * sa_step + (int64_t)ra[i] * 8);
        }
    };
    // FP4: block j (0 .. 3) of the lane's four out of its two chunks; rows with bit 4 set keep the
    // two blocks of a chunk in swapped order
    auto fp4_block = [&](const i32x4 (&x)[2], int j, bool swapped) {
        const i32x4 c = x[j >> 1];
        const bool second = ((j & 1) != 0) != swapped;
        return i32x8{second ? c[2] : c[0], second ? c[3] : c[1], 0, 0, 0, 0, 0, 0};
    };
    const bool b_swapped = (rb >> 4) & 1;
    auto multiply = [&](const i32x4 (&xa)[TM][2], const i32x4 (&xb)[2], const i32x2 (&xsa)[TM], i32x2 xsb) {
        static_for<NSUB>([&](auto S) {
            constexpr int sub = decltype(S)::value;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if constexpr (BF16) {
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xa[i][sub]),
                                                                     __builtin_bit_cast(bf16x8, xb[sub]), acc[i], 0, 0, 0);
                } else if constexpr (FP6) {  // the registers of the hardware block's idle half are zero
                    const i32x8 wa = {xa[i][sub][0], xa[i][sub][1], xa[i][sub][2], xa[i][sub][3], 0, 0, 0, 0};
                    const i32x8 wb = {xb[sub][0], xb[sub][1], xb[sub][2], xb[sub][3], 0, 0, 0, 0};
                    acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wa, wb, acc[i], kFp6, kFp6, kScaleByteA,
                                                                             wa[3], kScaleByteB, wb[3]);
                } else {
                    const i32x8 wa = fp4_block(xa[i], sub, (ra[i] >> 4) & 1), wb = fp4_block(xb, sub, b_swapped);
                    const uint32_t ka = __builtin_amdgcn_perm((uint32_t)xsa[i][1], (uint32_t)xsa[i][0], scale_sel);
                    const uint32_t kb = __builtin_amdgcn_perm((uint32_t)xsb[1], (uint32_t)xsb[0], scale_sel);
                    acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wa, wb, acc[i], kFp4, kFp4, sub, (int)ka,
                                                                             sub, (int)kb);
                }
            }
        });
    };
    for (int q = wave; q < nk; q += kSkinnyWaves * kAhead) {
#pragma unroll
        for (int u = 0; u < kAhead; ++u)
            if (q + u * kSkinnyWaves < nk) load(q + u * kSkinnyWaves, fa[u], fb[u], sa[u], sb[u]);
#pragma unroll
        for (int u = 0; u < kAhead; ++u)
            if (q + u * kSkinnyWaves < nk) multiply(fa[u], fb[u], sa[u], sb[u]);
    }
    // register r of lane l is row 8 (r / 4) + 4 (l / 32) + r % 4 of its tile of A, column l % 32
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (i > 0) __syncthreads();  // the sums of the tile before have been read
#pragma unroll
        for (int r = 0; r < 16; ++r) s_red[wave][r][lane] = acc[i][r];
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16 * 64 / (64 * kSkinnyWaves); ++k) {
            const int e = k * (64 * kSkinnyWaves) + threadIdx.x, r = e >> 6, l = e & 63;
            float v = s_red[0][r][l];
#pragma unroll
            for (int w = 1; w < kSkinnyWaves; ++w) v += s_red[w][r][l];
            const int m = 32 * i + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3), n = n0 + (l & 31);
            if (m < M && n < N) {
                if (c_bf16)
                    static_cast<uint16_t *>(C)[(int64_t)m * ldc + n] = bf16_rne(v);
                else
                    static_cast<float *>(C)[(int64_t)m * ldc + n] = v;
            }
        }
    }
}

// The same stream when the BF16 product is the one to take (MX9 takes part) and A has few rows: B is
// not rewritten as a BF16 image (2 bytes per element) but read as it is stored, in its three
// planes (9, 6 or 4 bits per element), and expanded to BF16 in registers on the way into the MFMA.
// A is the K-tiled BF16 image of its few rows.  Within 64 elements of K the lower half wave takes
// the first 32 and the upper one the last 32 (four sub-steps of 8 each): a lane's share is the two
// blocks load_packed brings, and one K step of A's image (64 bytes).
template <int MBB, int TM>
__global__ __launch_bounds__(64 * kSkinnyWaves) void gemm_skinny_planes_kernel(
    const uint8_t *__restrict__ A, const uint8_t *__restrict__ b_codes, const uint8_t *__restrict__ b_sexp,
    const uint8_t *__restrict__ b_mexp, int M, int N, int nq, void *__restrict__ C, int64_t ldc, int c_bf16)
{
    __shared__ float s_red[kSkinnyWaves][16][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n0 = blockIdx.x * kSkinnyRows;
    const int f_row = lane & 31, f_half = lane >> 5;
    // rows past the edge of an operand repeat its last row (their products are never stored)
    const int rb = min(n0 + f_row, N - 1);
    const int64_t b_blk0 = (int64_t)rb * (4 * (int64_t)nq) + 2 * f_half;  // first of the lane's block pairs
    const int64_t a_step = (int64_t)M * kRingRow;                         // one K step (32 elements) of A's image
    int a_at[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) a_at[i] = min(32 * i + f_row, M - 1) * kRingRow;
    f32x16 acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    constexpr int kAhead = 2;
    Packed<MBB> pb[kAhead];
    i32x4 fa[kAhead][TM][4];
    for (int q = wave; q < nq; q += kSkinnyWaves * kAhead) {
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int qq = q + u * kSkinnyWaves;
            if (qq < nq) {
                load_packed<MBB>(b_codes, b_sexp, b_mexp, b_blk0 + 4 * (int64_t)qq, pb[u]);
                const uint8_t *ap = A + (2 * (int64_t)qq + f_half) * a_step;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int c = 0; c < 4; ++c) fa[u][i][c] = *reinterpret_cast<const i32x4 *>(ap + a_at[i] + 16 * c);
            }
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            if (q + u * kSkinnyWaves < nq) {
                uint32_t w[16];
                if constexpr (MBB == 7)
                    unpack32_mx9(pb[u], w);
                else
                    unpack32<MBB>(pb[u], w);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const i32x4 fb = {(int)w[4 * c], (int)w[4 * c + 1], (int)w[4 * c + 2], (int)w[4 * c + 3]};
#pragma unroll
                    for (int i = 0; i < TM; ++i)
                        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[u][i][c]),
                                                                         __builtin_bit_cast(bf16x8, fb), acc[i], 0, 0, 0);
                }
            }
        }
    }
    // register r of lane l is row 8 (r / 4) + 4 (l / 32) + r % 4 of its tile of A, column l % 32
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (i > 0) __syncthreads();  // the sums of the tile before have been read
#pragma unroll
        for (int r = 0; r < 16; ++r) s_red[wave][r][lane] = acc[i][r];
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16 * 64 / (64 * kSkinnyWaves); ++k) {
            const int e = k * (64 * kSkinnyWaves) + threadIdx.x, r = e >> 6, l = e & 63;
            float v = s_red[0][r][l];
#pragma unroll
            for (int w = 1; w < kSkinnyWaves; ++w) v += s_red[w][r][l];
            const int m = 32 * i + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3), n = n0 + (l & 31);
            if (m < M && n < N) {
                if (c_bf16)
                    static_cast<uint16_t *>(C)[(int64_t)m * ldc + n] = bf16_rne(v);
                else
                    static_cast<float *>(C)[(int64_t)m * ldc + n] = v;
            }
        }
    }
}

// The same with tiles of 16 x 16 (MFMA 16 x 16 x 32): twice as many workgroups, each with half the
// expansion work -- the kernel is bound by those vector instructions, and 384 workgroups of 32 rows
// meet 256 CUs as two rounds for half of them, 768 of 16 rows as three even ones.  Lane l holds row
// l % 16 and the K group l / 16; within 128 elements of K group g takes elements 32 g .. 32 g + 31
// (again the two blocks load_packed brings, and one K step of A's image), eight per MFMA.  Both
// operands give the same elements to the same lane group, which is all the instruction asks for.
template <int MBB, int TM>
__global__ __launch_bounds__(64 * kSkinnyWaves) void gemm_skinny_planes16_kernel(
    const uint8_t *__restrict__ A, const uint8_t *__restrict__ b_codes, const uint8_t *__restrict__ b_sexp,
    const uint8_t *__restrict__ b_mexp, int M, int N, int nq, void *__restrict__ C, int64_t ldc, int c_bf16)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    __shared__ float s_red[kSkinnyWaves][TM][4][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n0 = blockIdx.x * 16;
    const int f_row = lane & 15, f_grp = lane >> 4;
    const int rb = min(n0 + f_row, N - 1);
    const int64_t b_blk0 = (int64_t)rb * (8 * (int64_t)nq) + 2 * f_grp;  // K / 16 = 8 nq blocks per row
    const int64_t a_step = (int64_t)M * kRingRow;
    int a_at[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) a_at[i] = min(16 * i + f_row, M - 1) * kRingRow;
    f32x4 acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr int kAhead = 2;
    Packed<MBB> pb[kAhead];
    i32x4 fa[kAhead][TM][4];
    for (int q = wave; q < nq; q += kSkinnyWaves * kAhead) {
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int qq = q + u * kSkinnyWaves;
            if (qq < nq) {
                load_packed<MBB>(b_codes, b_sexp, b_mexp, b_blk0 + 8 * (int64_t)qq, pb[u]);
                const uint8_t *ap = A + (4 * (int64_t)qq + f_grp) * a_step;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int c = 0; c < 4; ++c) fa[u][i][c] = *reinterpret_cast<const i32x4 *>(ap + a_at[i] + 16 * c);
            }
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            if (q + u * kSkinnyWaves < nq) {
                uint32_t w[16];
                if constexpr (MBB == 7)
                    unpack32_mx9(pb[u], w);
                else
                    unpack32<MBB>(pb[u], w);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const i32x4 fb = {(int)w[4 * c], (int)w[4 * c + 1], (int)w[4 * c + 2], (int)w[4 * c + 3]};
#pragma unroll
                    for (int i = 0; i < TM; ++i)
                        acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fa[u][i][c]),
                                                                         __builtin_bit_cast(bf16x8, fb), acc[i], 0, 0, 0);
                }
            }
        }
    }
    // register r of lane l is row 4 (l / 16) + r of its tile of A, column l % 16
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) s_red[wave][i][r][lane] = acc[i][r];
    __syncthreads();
    for (int e = threadIdx.x; e < TM * 4 * 64; e += 64 * kSkinnyWaves) {
        const int i = e >> 8, r = (e >> 6) & 3, l = e & 63;
        float v = s_red[0][i][r][l];
#pragma unroll
        for (int w = 1; w < kSkinnyWaves; ++w) v += s_red[w][i][r][l];
        const int m = 16 * i + 4 * (l >> 4) + r, n = n0 + (l & 15);
        if (m < M && n < N) {
            if (c_bf16)
                static_cast<uint16_t *>(C)[(int64_t)m * ldc + n] = bf16_rne(v);
            else
                static_cast<float *>(C)[(int64_t)m * ldc + n] = v;
        }
    }
}

template <int MBB>
int launch_skinny_planes(const uint8_t *a, const uint8_t *bc, const uint8_t *bs, const uint8_t *bm, int M, int N,
                         int nq, void *C, int64_t ldc, int c_bf16, hipStream_t s)
{
    const dim3 grid((unsigned)((N + kSkinnyRows - 1) / kSkinnyRows)), block(64 * kSkinnyWaves);
    // N = K = 12288, MX9 planes, A's expansion included: 16-row tiles 51 / 55 / 73 / 112 us for M = 1 /
    // 16 / 32 / 64, 32-row tiles 65 / 69 / 75 / 102 us
    if (nq % 2 == 0 && M <= 32) {  // K a multiple of 128
        const dim3 g16((unsigned)((N + 15) / 16));
        if (M <= 16)
            hipLaunchKernelGGL((gemm_skinny_planes16_kernel<MBB, 1>), g16, block, 0, s, a, bc, bs, bm, M, N, nq / 2, C, ldc, c_bf16);
        else
            hipLaunchKernelGGL((gemm_skinny_planes16_kernel<MBB, 2>), g16, block, 0, s, a, bc, bs, bm, M, N, nq / 2, C, ldc, c_bf16);
        return launch_status();
    }
    if (M <= 32)
        hipLaunchKernelGGL((gemm_skinny_planes_kernel<MBB, 1>), grid, block, 0, s, a, bc, bs, bm, M, N, nq, C, ldc, c_bf16);
    else
        hipLaunchKernelGGL((gemm_skinny_planes_kernel<MBB, 2>), grid, block, 0, s, a, bc, bs, bm, M, N, nq, C, ldc, c_bf16);
    return launch_status();
}

template <int FMT>
int launch_skinny(const uint8_t *a, const uint8_t *b, const uint8_t *sa, const uint8_t *sb, int M, int N, int nk,
                  void *C, int64_t ldc, int c_bf16, hipStream_t s)
{
    const dim3 grid((unsigned)((N + kSkinnyRows - 1) / kSkinnyRows)), block(64 * kSkinnyWaves);
    if (M <= 32)
        hipLaunchKernelGGL((gemm_skinny_kernel<FMT, 1>), grid, block, 0, s, a, b, sa, sb, M, N, nk, C, ldc, c_bf16);
    else
        hipLaunchKernelGGL((gemm_skinny_kernel<FMT, 2>), grid, block, 0, s, a, b, sa, sb, M, N, nk, C, ldc, c_bf16);
    return launch_status();
}

// With `dry` set the launch functions below only ask for what the kernel needs (a workgroup
// of more than 64 KiB of LDS has to be granted once per device) and launch nothing: the entry
// point calls them that way before it enqueues the image writers.
template <int WM, int WN, int TM, int TN, int FMT>
int launch_ring(const uint8_t *A, const uint8_t *B, const uint8_t *SA, const uint8_t *SB, int M, int N, int nk,
                void *C, int64_t ldc, int c_bf16, bool dry, hipStream_t s)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr size_t kLds = kRingStages * (BM + BN) * (size_t)(kRingRow + (FMT == kFmtFp4 ? 8 : 0));
    static signed char granted[kMaxDevices];
    if (kLds > 64 * 1024 &&
        !grant_dynamic_lds(reinterpret_cast<const void *>(&gemm_ring_kernel<WM, WN, TM, TN, FMT>), kLds, granted))
        return BDR_ERR_LAUNCH;
    if (dry) return BDR_OK;
    hipLaunchKernelGGL((gemm_ring_kernel<WM, WN, TM, TN, FMT>), dim3((unsigned)(((M + BM - 1) / BM) * ((N + BN - 1) / BN))),
                       dim3(64 * WM * WN), kLds, s, A, B, SA, SB, M, N, nk, C, ldc, c_bf16);
    return launch_status();
}

template <int FMT>
int gemm_ring(const void *A, const void *B, const void *SA, const void *SB, int64_t M, int64_t N, int nk, void *C,
              int64_t ldc, int c_bf16, bool dry, hipStream_t s)
{
    const uint8_t *a = (const uint8_t *)A, *b = (const uint8_t *)B, *sa = (const uint8_t *)SA, *sb = (const uint8_t *)SB;
    if (M <= kSkinnyMaxM) {  // a stream over B's image
        if (dry) return BDR_OK;
        return launch_skinny<FMT>(a, b, sa, sb, (int)M, (int)N, nk, C, ldc, c_bf16, s);
    }
    if (M % 256 == 0 && N % 256 == 0 && (M / 256) * (N / 256) >= kBigTileMin) {
        const int st = launch_ring<2, 4, 4, 2, FMT>(a, b, sa, sb, (int)M, (int)N, nk, C, ldc, c_bf16, dry, s);
        if (st != BDR_ERR_LAUNCH) return st;  // a device without 128 KiB workgroups: small tiles
    }
    return launch_ring<2, 2, 2, 2, FMT>(a, b, sa, sb, (int)M, (int)N, nk, C, ldc, c_bf16, dry, s);
}

// Two tile shapes: 256 x 256 with 8 waves (128 KiB of LDS, one workgroup per CU)
// when the device grants that much LDS to a workgroup and M, N allow it, else
// 128 x 128 with 4 waves (64 KiB).
template <int MBA, int MBB>
int launch_gemm(const uint8_t *ac, const uint8_t *as, const uint8_t *am, const uint8_t *bc,
                const uint8_t *bs, const uint8_t *bm, int M, int N, int K, void *C, int64_t ldc, int c_bf16,
                hipStream_t s)
{
    constexpr size_t kBigLds = 2 * (256 + 256) * (size_t)kPitch;
    constexpr size_t kSmallLds = 2 * (128 + 128) * (size_t)kPitch;
    static signed char granted[kMaxDevices];  // does the device allow a 128 KiB workgroup?
    const bool big_ok =
        M % 256 == 0 && N % 256 == 0 && (int64_t)(M / 256) * (N / 256) >= kBigTileMin &&
        grant_dynamic_lds(reinterpret_cast<const void *>(&mx_gemm_kernel<MBA, MBB, 2, 4, 4, 2>), kBigLds, granted);
    if (big_ok) {
        const unsigned grid = (unsigned)((M / 256) * (N / 256));
        hipLaunchKernelGGL((mx_gemm_kernel<MBA, MBB, 2, 4, 4, 2>), dim3(grid), dim3(512), kBigLds, s,
                           ac, as, am, bc, bs, bm, M, N, K, C, ldc, c_bf16);
    } else {
        const unsigned grid = (unsigned)(((M + 127) / 128) * ((N + 127) / 128));
        hipLaunchKernelGGL((mx_gemm_kernel<MBA, MBB, 2, 2, 2, 2>), dim3(grid), dim3(256), kSmallLds,
                           s, ac, as, am, bc, bs, bm, M, N, K, C, ldc, c_bf16);
    }
    return launch_status();
}

template <int MBA>
int pick_b(int mb, const uint8_t *ac, const uint8_t *as, const uint8_t *am, const uint8_t *bc,
           const uint8_t *bs, const uint8_t *bm, int M, int N, int K, void *C, int64_t ldc, int c_bf16,
           hipStream_t s)
{
    if (mb == 7) return launch_gemm<MBA, 7>(ac, as, am, bc, bs, bm, M, N, K, C, ldc, c_bf16, s);
    if (mb == 4) return launch_gemm<MBA, 4>(ac, as, am, bc, bs, bm, M, N, K, C, ldc, c_bf16, s);
    return launch_gemm<MBA, 2>(ac, as, am, bc, bs, bm, M, N, K, C, ldc, c_bf16, s);
}

template <int WM, int WN, int TM, int TN>
int launch_dl(const uint16_t *A, const uint16_t *B, int M, int N, int K, void *C, int64_t ldc, int c_bf16, bool dry,
              hipStream_t s)
{
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr size_t kLds = 2 * (BM + BN) * (size_t)kPitch;
    static signed char granted[kMaxDevices];
    if (kLds > 64 * 1024 &&
        !grant_dynamic_lds(reinterpret_cast<const void *>(&gemm_dl_kernel<WM, WN, TM, TN>), kLds, granted))
        return BDR_ERR_LAUNCH;
    if (dry) return BDR_OK;
    hipLaunchKernelGGL((gemm_dl_kernel<WM, WN, TM, TN>), dim3((unsigned)(((M + BM - 1) / BM) * ((N + BN - 1) / BN))),
                       dim3(64 * WM * WN), kLds, s, A, B, M, N, K, C, ldc, c_bf16);
    return launch_status();
}

// K = 0: one workgroup per row of C (rows on grid.x, which takes up to 2^31 - 1 workgroups;
// grid.y stops at 65535 and M may be 2^20).
__global__ void gemm_zero_kernel(void *C, int64_t ldc, int c_bf16, int N)
{
    const int64_t row = blockIdx.x;
    for (int c = threadIdx.x; c < N; c += blockDim.x) {
        if (c_bf16)
            static_cast<uint16_t *>(C)[row * ldc + c] = 0;
        else
            static_cast<float *>(C)[row * ldc + c] = 0.f;
    }
}

}  // namespace

int gemm(const bdr_format &fa, const bdr_format &fb, const void *a_codes, const void *a_sexp,
         const void *a_mexp, const void *b_codes, const void *b_sexp, const void *b_mexp,
         int64_t M, int64_t N, int64_t K, void *C, int64_t ldc, int c_bf16, hipStream_t s)
{
    if (K == 0) {  // empty sum
        hipLaunchKernelGGL(gemm_zero_kernel, dim3((unsigned)M), dim3(256), 0, s, C, ldc, c_bf16, (int)N);
        return launch_status();
    }
    const uint8_t *ac = (const uint8_t *)a_codes, *as = (const uint8_t *)a_sexp,
                  *am = (const uint8_t *)a_mexp, *bc = (const uint8_t *)b_codes,
                  *bs = (const uint8_t *)b_sexp, *bm = (const uint8_t *)b_mexp;
    if (fa.m == 7) return pick_b<7>(fb.m, ac, as, am, bc, bs, bm, (int)M, (int)N, (int)K, C, ldc, c_bf16, s);
    if (fa.m == 4) return pick_b<4>(fb.m, ac, as, am, bc, bs, bm, (int)M, (int)N, (int)K, C, ldc, c_bf16, s);
    return pick_b<2>(fb.m, ac, as, am, bc, bs, bm, (int)M, (int)N, (int)K, C, ldc, c_bf16, s);
}

// C = A * B^T for row-major BF16 A [M x K] and B [N x K] (K > 0, shapes already validated).
int gemm_bf16(const void *A, const void *B, int64_t M, int64_t N, int64_t K, void *C, int64_t ldc, int c_bf16,
              bool dry, hipStream_t s)
{
    const uint16_t *a = (const uint16_t *)A, *b = (const uint16_t *)B;
    if (M % 256 == 0 && N % 256 == 0 && (M / 256) * (N / 256) >= kBigTileMin) {
        const int st = launch_dl<2, 4, 4, 2>(a, b, (int)M, (int)N, (int)K, C, ldc, c_bf16, dry, s);
        if (st != BDR_ERR_LAUNCH) return st;  // a device without 128 KiB workgroups: small tiles
    }
    return launch_dl<2, 2, 2, 2>(a, b, (int)M, (int)N, (int)K, C, ldc, c_bf16, dry, s);
}

// C = A * B^T for K-tiled BF16 images (to_bf16_tiled) of A [M x K] and B [N x K]; K % 32 == 0.
int gemm_bf16_tiled(const void *A, const void *B, int64_t M, int64_t N, int64_t K, void *C, int64_t ldc, int c_bf16,
                    bool dry, hipStream_t s)
{
    return gemm_ring<kFmtBf16>(A, B, nullptr, nullptr, M, N, (int)(K / 32), C, ldc, c_bf16, dry, s);
}

// Whether gemm_bf16_planes takes a product of these sizes (few rows of A).
bool gemm_bf16_planes_ok(int64_t M, int64_t K) { return M >= 1 && M <= kSkinnyMaxM && K % 64 == 0; }

// C = A * B^T for the K-tiled BF16 image of A [M x K] (to_bf16_tiled) and the packed planes of B
// [N x K] in a Table II format; gemm_bf16_planes_ok(M, K).
int gemm_bf16_planes(const void *A, const bdr_format &fb, const void *b_codes, const void *b_sexp,
                     const void *b_mexp, int64_t M, int64_t N, int64_t K, void *C, int64_t ldc, int c_bf16,
                     hipStream_t s)
{
    const uint8_t *a = (const uint8_t *)A, *bc = (const uint8_t *)b_codes, *bs = (const uint8_t *)b_sexp,
                  *bm = (const uint8_t *)b_mexp;
    const int nq = (int)(K / 64);
    if (fb.m == 7) return launch_skinny_planes<7>(a, bc, bs, bm, (int)M, (int)N, nq, C, ldc, c_bf16, s);
    if (fb.m == 4) return launch_skinny_planes<4>(a, bc, bs, bm, (int)M, (int)N, nq, C, ldc, c_bf16, s);
    return launch_skinny_planes<2>(a, bc, bs, bm, (int)M, (int)N, nq, C, ldc, c_bf16, s);
}

// Packed Table II planes of a [rows x K] operand (K % 32 == 0) -> BF16, tiled along K.
int to_bf16_tiled(const bdr_format &f, const void *codes, const void *sexp, const void *mexp, int64_t rows,
                  int64_t K, void *out, hipStream_t s)
{
    if (rows == 0 || K == 0) return BDR_OK;
    const uint8_t *c = (const uint8_t *)codes, *e = (const uint8_t *)sexp, *m = (const uint8_t *)mexp;
    const int rp = (int)(K / 32);
    // rows on grid.x (up to 2^31 - 1 workgroups), K steps on grid.y (K <= 2^20: at most 2048)
    const dim3 grid((unsigned)((rows + 15) / 16), (unsigned)((rp + 15) / 16)), block(256);
    u32x4 *o = (u32x4 *)out;
    if (f.m == 7) hipLaunchKernelGGL((mx_to_bf16_tiled_kernel<7>), grid, block, 0, s, c, e, m, (int)rows, rp, o);
    else if (f.m == 4) hipLaunchKernelGGL((mx_to_bf16_tiled_kernel<4>), grid, block, 0, s, c, e, m, (int)rows, rp, o);
    else hipLaunchKernelGGL((mx_to_bf16_tiled_kernel<2>), grid, block, 0, s, c, e, m, (int)rows, rp, o);
    return launch_status();
}

// C = A * B^T for FP6 block images (to_fp6) of A [M x K] and B [N x K]; K % 64 == 0.
int gemm_fp6(const void *A, const void *B, int64_t M, int64_t N, int64_t K, void *C, int64_t ldc, int c_bf16,
             bool dry, hipStream_t s)
{
    return gemm_ring<kFmtFp6>(A, B, nullptr, nullptr, M, N, (int)(K / 64), C, ldc, c_bf16, dry, s);
}

// Packed MX6 or MX4 planes of a [rows x K] operand (K % 64 == 0) -> rows x K / 16 chunks of
// 16 bytes, tiled along K as the product kernel reads them.
int to_fp6(const bdr_format &f, const void *codes, const void *sexp, const void *mexp,
           int64_t rows, int64_t K, void *out, bool b_operand, hipStream_t s)
{
    if (rows == 0 || K == 0) return BDR_OK;
    const uint8_t *c = (const uint8_t *)codes, *e = (const uint8_t *)sexp, *m = (const uint8_t *)mexp;
    const int rp = (int)(K / 32);
    const int64_t pairs = rows * rp;
    const dim3 grid((unsigned)((pairs + 255) / 256)), block(256);
    u32x4 *o = (u32x4 *)out;
    if (f.m == 4) {
        if (b_operand) hipLaunchKernelGGL((mx_to_fp6_kernel<4, true>), grid, block, 0, s, c, e, m, pairs, (int)rows, rp, o);
        else hipLaunchKernelGGL((mx_to_fp6_kernel<4, false>), grid, block, 0, s, c, e, m, pairs, (int)rows, rp, o);
    } else {
        if (b_operand) hipLaunchKernelGGL((mx_to_fp6_kernel<2, true>), grid, block, 0, s, c, e, m, pairs, (int)rows, rp, o);
        else hipLaunchKernelGGL((mx_to_fp6_kernel<2, false>), grid, block, 0, s, c, e, m, pairs, (int)rows, rp, o);
    }
    return launch_status();
}

// The scale image of an FP4 operand: rows padded to whole 128-row groups, 1 byte per block.
size_t fp4_scale_bytes(int64_t rows, int64_t K_out)
{
    return (size_t)((rows + 127) / 128 * 128) * (size_t)(K_out / 16);
}

// C = A * B^T for FP4 block images (to_fp4) of A [M x K] and B [N x K]; K % 128 == 0.
int gemm_fp4(const void *A, const void *SA, const void *B, const void *SB, int64_t M, int64_t N, int64_t K,
             void *C, int64_t ldc, int c_bf16, bool dry, hipStream_t s)
{
    return gemm_ring<kFmtFp4>(A, B, SA, SB, M, N, (int)(K / 128), C, ldc, c_bf16, dry, s);
}

// Packed MX4 planes of a [rows x K] operand (K % 32 == 0) -> rows x K_out / 32 chunks of 16
// bytes at `out` and fp4_scale_bytes(rows, K_out) scale bytes at `scales`, both tiled along K;
// K_out >= K a multiple of 128, blocks past K are zero.
int to_fp4(const void *codes, const void *sexp, const void *mexp, int64_t rows, int64_t K, int64_t K_out,
           void *out, void *scales, hipStream_t s)
{
    if (rows == 0 || K_out == 0) return BDR_OK;
    const int rp = (int)(K / 32), rpo = (int)(K_out / 32);
    const int64_t pairs = (rows + 127) / 128 * 128 * rpo;
    hipLaunchKernelGGL(mx_to_fp4_kernel, dim3((unsigned)((pairs + 255) / 256)), dim3(256), 0, s,
                       (const uint8_t *)codes, (const uint8_t *)sexp, (const uint8_t *)mexp, pairs, (int)rows, rp,
                       rpo, (u32x4 *)out, (uint8_t *)scales);
    return launch_status();
}

}  // namespace bdr
