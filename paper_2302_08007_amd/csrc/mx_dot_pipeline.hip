// Bit-true model of the dot-product pipeline the paper outlines for BDR formats
// (Sec. IV-B, "Dot Product Architecture", and the caption of the pipeline figure): the
// Hadamard product of each block of k1 elements is reduced to one integer, sub-blocks being
// shifted right by their microexponents on the way; the r / k1 block results of a pass are
// aligned to the largest exponent and added in a fixed-point word of f bits.  mx_gemm adds
// the same exact products in FP32 instead; this kernel exists to measure what that changes.
//
// What is computed, for every entry of C = A B^T and every pass of r elements of K
// (A, B in Table II's formats: k1 16, k2 2, one microexponent bit):
//   T_b   = sum over the 8 sub-blocks j of block b of
//           (Ma_2j Mb_2j + Ma_2j+1 Mb_2j+1) 2^(2 - tau_a[j] - tau_b[j])      exact integer
//   e_b   = SEa_b + SEb_b,  e_max = max over the blocks of the pass
//   U_b   = floor(T_b 2^(g - (e_max - e_b))),  g = f - 1 - W,  W = ma + mb + 6
//   pass  = (sum_b U_b) 2^(e_max - 254 - (ma - 1) - (mb - 1) - 2 - g), rounded once to FP32
//   C     = the passes added in FP32 in order of increasing k
//
// How: each operand is first rewritten (by the row-wise dequantize kernel with the exponent
// plane replaced by a constant) as BF16 integers Ma 2^(1 - tau_a + max(g, 0)) and
// Mb 2^(1 - tau_b); a 32x32x16 BF16 MFMA on one block of each with a zero accumulator then
// yields T_b 2^max(g, 0) for 32 x 32 entries at once, exactly (products of two <= 9-bit
// integers, 16 of them, stay below 2^24 units).  The rest is per entry on the vector ALUs:
// the exponent sums from the two exponent planes (two entries per instruction, as packed
// 16-bit integers), a first walk over the pass for e_max, a second one that converts the
// block results to integers, shifts them right (arithmetic shift = floor) by
// e_max - e_b + max(-g, 0) and adds them into integer accumulators.
#include "bdr_device.hpp"
#include "bdr_internal.hpp"

namespace bdr {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// Workgroup tile of C: 4 waves as 2 x 2, each kTJ MFMA tiles of 32 x 32 side by side.  One
// tile per wave keeps a lane under 128 registers, so that several waves share a SIMD and
// fill each other's waits (the kernel is bound by vector-ALU issue; with two tiles per wave
// and one wave per SIMD it ran a quarter slower).
constexpr int kTJ = 1;
constexpr int kPM = 64, kPN = 2 * 32 * kTJ;
constexpr int kBChunks = kPN * 8 / 256;  // 16-byte chunks of the B tile a thread brings in per K step
constexpr int kPThreads = 256;
constexpr int kStepBytes = 128;     // one K step: 64 BF16 = 4 blocks per row
constexpr int kFoldSteps = 16;      // K steps between folds of the 32-bit partial sums
constexpr int kMaxDrop = 31;        // a shift by the width of the word or more drops everything

// 16-byte chunk c of tile row r, placed so that the 16 lanes served together by a 16-byte
// read (16 consecutive rows, one chunk) touch every bank once.
__device__ __forceinline__ int tile_chunk(int row, int chunk)
{
    return row * kStepBytes + ((chunk ^ ((row >> 1) & 7)) << 4);
}

struct Staged {  // what a thread brings in for one K step
    u32x4 a[2], b[kBChunks];
    uint32_t se;
};

// One workgroup computes a kPM x kPN tile of C.  WIDE: passes longer than 1024 elements, whose
// sums may need more than 32 bits (64 blocks of f - 1 <= 25 magnitude bits fit 31).
template <bool WIDE>
__global__ __launch_bounds__(kPThreads, 2) void dot_pipeline_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ B,
    const uint8_t *__restrict__ sea, const uint8_t *__restrict__ seb, int M, int N, int K, int r,
    int xoff, int extra, float *__restrict__ C, int64_t ldc)
{
    __shared__ __attribute__((aligned(16))) uint8_t s_a[kPM * kStepBytes];
    __shared__ __attribute__((aligned(16))) uint8_t s_b[kPN * kStepBytes];
    __shared__ uint32_t s_se[kPM + kPN];  // the 4 exponent bytes of every tile row for this K step

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int ntn = (N + kPN - 1) / kPN;
    const int m0 = (int)(blockIdx.x / ntn) * kPM, n0 = (int)(blockIdx.x % ntn) * kPN;
    const int64_t kb = K >> 4;  // blocks per operand row = bytes per row of an exponent plane

    // --- what this thread fetches per K step (rows past the edge repeat the last row; their
    // entries are never stored)
    const uint16_t *ap[2], *bp[kBChunks];
    int a_lds[2], b_lds[kBChunks];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = tid + i * kPThreads, row = c >> 3, ch = c & 7;
        ap[i] = A + (int64_t)min(m0 + row, M - 1) * K + 8 * ch;
        a_lds[i] = tile_chunk(row, ch);
    }
#pragma unroll
    for (int i = 0; i < kBChunks; ++i) {
        const int c = tid + i * kPThreads, row = c >> 3, ch = c & 7;
        bp[i] = B + (int64_t)min(n0 + row, N - 1) * K + 8 * ch;
        b_lds[i] = tile_chunk(row, ch);
    }
    const uint8_t *sp = nullptr;  // threads 0 .. kPM - 1: an A row, the next kPN: a B row
    if (tid < kPM)
        sp = sea + (int64_t)min(m0 + tid, M - 1) * kb;
    else if (tid < kPM + kPN)
        sp = seb + (int64_t)min(n0 + tid - kPM, N - 1) * kb;

    auto fetch = [&](int kstep, bool tiles, Staged &st) {
        if (tiles) {
#pragma unroll
            for (int i = 0; i < 2; ++i) st.a[i] = *reinterpret_cast<const u32x4 *>(ap[i] + (int64_t)kstep * 64);
#pragma unroll
            for (int i = 0; i < kBChunks; ++i) st.b[i] = *reinterpret_cast<const u32x4 *>(bp[i] + (int64_t)kstep * 64);
        }
        st.se = sp ? *reinterpret_cast<const uint32_t *>(sp + 4 * (int64_t)kstep) : 0u;
    };
    auto commit = [&](bool tiles, const Staged &st) {
        if (tiles) {
#pragma unroll
            for (int i = 0; i < 2; ++i) *reinterpret_cast<u32x4 *>(s_a + a_lds[i]) = st.a[i];
#pragma unroll
            for (int i = 0; i < kBChunks; ++i) *reinterpret_cast<u32x4 *>(s_b + b_lds[i]) = st.b[i];
        }
        if (tid < kPM + kPN) s_se[tid] = st.se;
    };

    // --- the lane's entries: for MFMA tile tj (columns 32 tj ..), accumulator register e is
    // row 8 (e / 4) + 4 (lane / 32) + e % 4, column lane % 32
    const int f_row = lane & 31, f_half = lane >> 5;
    const int se_row0 = 32 * wm + 4 * f_half;           // + 8 (e / 4) + e % 4
    const int se_col0 = kPM + 32 * kTJ * wn + f_row;    // + 32 tj
    auto exps_of_step = [&](uint32_t (&ea)[16], uint32_t (&eb)[kTJ]) {
#pragma unroll
        for (int e = 0; e < 16; ++e) ea[e] = s_se[se_row0 + 8 * (e >> 2) + (e & 3)];
#pragma unroll
        for (int tj = 0; tj < kTJ; ++tj) eb[tj] = s_se[se_col0 + 32 * tj];
    };

    // Exponent sums are at most 508 and fit 16 bits: entries e and e + 1 of an MFMA tile
    // (rows r and r + 1 of one column) are handled as one packed pair.
    // pair p of block blk: byte blk of ea[2p] in the low half, of ea[2p + 1] in the high half
    auto a_pairs = [&](const uint32_t (&ea)[16], int blk, u16x2 (&ap2)[8]) {
#pragma unroll
        for (int p = 0; p < 8; ++p)
            ap2[p] = __builtin_bit_cast(
                u16x2, __builtin_amdgcn_perm(ea[2 * p + 1], ea[2 * p], 0x0c000c00u | (uint32_t)blk |
                                                                           ((uint32_t)(4 + blk) << 16)));
    };
    auto b_pair = [&](uint32_t eb, int blk) {  // byte blk of eb in both halves
        return __builtin_bit_cast(u16x2, __builtin_amdgcn_perm(eb, eb, 0x0c000c00u | (uint32_t)blk |
                                                                           ((uint32_t)blk << 16)));
    };
    const u16x2 extra2 = {(unsigned short)extra, (unsigned short)extra};
    const u16x2 cap2 = {(unsigned short)kMaxDrop, (unsigned short)kMaxDrop};

    // A pass is two walks over its K steps, each with the next step's data on its way from
    // memory while the current one is computed.  (One loop over all walks of all passes, with
    // the fetch running across their boundaries, was tried: the branch inside it cost more
    // than the exposed fetches it removed.)
    float cacc[kTJ][16];
    const int n_pass = K / r, steps = r / 64;
    for (int pass = 0; pass < n_pass; ++pass) {
        const int step0 = pass * steps;
        Staged st;

        // ---- first walk: the largest exponent sum of the pass, per entry
        u16x2 emax[kTJ][8];
#pragma unroll
        for (int tj = 0; tj < kTJ; ++tj)
#pragma unroll
            for (int p = 0; p < 8; ++p) emax[tj][p] = u16x2{0, 0};
        fetch(step0, false, st);
        __syncthreads();  // everybody is done with the previous contents of the staging area
        commit(false, st);
        __syncthreads();
        for (int s = 0; s < steps; ++s) {
            if (s + 1 < steps) fetch(step0 + s + 1, false, st);
            uint32_t ea[16], eb[kTJ];
            exps_of_step(ea, eb);
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) {
                u16x2 ap2[8];
                a_pairs(ea, blk, ap2);
#pragma unroll
                for (int tj = 0; tj < kTJ; ++tj) {
                    const u16x2 bp2 = b_pair(eb[tj], blk);
#pragma unroll
                    for (int p = 0; p < 8; ++p)
                        emax[tj][p] = __builtin_elementwise_max(emax[tj][p], (u16x2)(ap2[p] + bp2));
                }
            }
            __syncthreads();
            if (s + 1 < steps) commit(false, st);
            __syncthreads();
        }

        // ---- second walk: block products, aligned to e_max, dropped into the word and added
        // shift of block b = (e_max + extra) - e_b, held at 31
        u16x2 top[kTJ][8];
        int part[kTJ][16];
        int64_t total[WIDE ? kTJ : 1][WIDE ? 16 : 1];
#pragma unroll
        for (int tj = 0; tj < kTJ; ++tj) {
#pragma unroll
            for (int p = 0; p < 8; ++p) top[tj][p] = emax[tj][p] + extra2;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                part[tj][e] = 0;
                if (WIDE) total[tj][WIDE ? e : 0] = 0;
            }
        }
        fetch(step0, true, st);
        commit(true, st);  // the loop above ended on a barrier
        __syncthreads();
        for (int s = 0; s < steps; ++s) {
            if (s + 1 < steps) fetch(step0 + s + 1, true, st);
            uint32_t ea[16], eb[kTJ];
            exps_of_step(ea, eb);
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) {
                const bf16x8 fa = *reinterpret_cast<const bf16x8 *>(
                    s_a + tile_chunk(32 * wm + f_row, 2 * blk + f_half));
                u16x2 ap2[8];
                a_pairs(ea, blk, ap2);
#pragma unroll
                for (int tj = 0; tj < kTJ; ++tj) {
                    const bf16x8 fb = *reinterpret_cast<const bf16x8 *>(
                        s_b + tile_chunk(32 * kTJ * wn + 32 * tj + f_row, 2 * blk + f_half));
                    f32x16 t;
#pragma unroll
                    for (int e = 0; e < 16; ++e) t[e] = 0.f;
                    t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, t, 0, 0, 0);  // T_b 2^max(g, 0), exact
                    const u16x2 bp2 = b_pair(eb[tj], blk);
#pragma unroll
                    for (int p = 0; p < 8; ++p) {
                        const u16x2 drop = __builtin_elementwise_min((u16x2)(top[tj][p] - (u16x2)(ap2[p] + bp2)), cap2);
                        part[tj][2 * p] += (int)t[2 * p] >> (int)drop.x;          // arithmetic: floor
                        part[tj][2 * p + 1] += (int)t[2 * p + 1] >> (int)drop.y;
                    }
                }
            }
            if (WIDE && ((s + 1) % kFoldSteps == 0 || s + 1 == steps)) {
#pragma unroll
                for (int tj = 0; tj < kTJ; ++tj)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        total[tj][WIDE ? e : 0] += part[tj][e];
                        part[tj][e] = 0;
                    }
            }
            __syncthreads();
            if (s + 1 < steps) commit(true, st);
            __syncthreads();
        }

        // ---- the pass's value, rounded once to FP32, and the FP32 sum over the passes
#pragma unroll
        for (int tj = 0; tj < kTJ; ++tj)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int em = e & 1 ? (int)emax[tj][e >> 1].y : (int)emax[tj][e >> 1].x;
                const float sum = WIDE ? (float)total[tj][WIDE ? e : 0] : (float)part[tj][e];
                const float v = __builtin_ldexpf(sum, em + xoff);
                cacc[tj][e] = pass == 0 ? v : cacc[tj][e] + v;
            }
    }

#pragma unroll
    for (int tj = 0; tj < kTJ; ++tj) {
        const int col = n0 + 32 * kTJ * wn + 32 * tj + f_row;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = m0 + se_row0 + 8 * (e >> 2) + (e & 3);
            if (row < M && col < N) C[(int64_t)row * ldc + col] = cacc[tj][e];
        }
    }
}

}  // namespace

// Shapes and formats were validated by the caller: Table II formats, K % 64 == 0, r % 64 == 0,
// K % r == 0, K > 0, 2 <= f_bits <= 26.  workspace: (M + N) * K BF16 values, each operand
// rounded up to 256 bytes.
int dot_pipeline(const bdr_format &fa, const bdr_format &fb, const void *a_codes, const void *a_sexp,
                 const void *a_mexp, const void *b_codes, const void *b_sexp, const void *b_mexp,
                 int64_t M, int64_t N, int64_t K, int64_t r, int f_bits, float *C, int64_t ldc,
                 void *workspace, hipStream_t s)
{
    const int W = fa.m + fb.m + 4 + 2;  // magnitude bits of a block result: ma + mb + log2 16 + 2 beta
    const int g = f_bits - 1 - W;
    const int g_img = g > 0 ? g : 0, extra = g < 0 ? -g : 0;  // guard bits go into the image, missing ones into the shift
    char *wa = static_cast<char *>(workspace);
    char *wb = wa + (((size_t)M * (size_t)K * 2 + 255) & ~(size_t)255);
    // Ma 2^(1 - tau + g_img) and Mb 2^(1 - tau): the element value with exponent code 127 + m (+ g_img)
    int st = dequantize_row_fixed_exponent(fa, a_codes, a_mexp, M, K, wa, 127 + fa.m + g_img, s);
    if (st) return st;
    st = dequantize_row_fixed_exponent(fb, b_codes, b_mexp, N, K, wb, 127 + fb.m, s);
    if (st) return st;
    const int xoff = -254 - (fa.m - 1) - (fb.m - 1) - 2 - g;
    const unsigned grid = (unsigned)(((M + kPM - 1) / kPM) * ((N + kPN - 1) / kPN));
    if (r > 1024)
        hipLaunchKernelGGL(dot_pipeline_kernel<true>, dim3(grid), dim3(kPThreads), 0, s, (const uint16_t *)wa,
                           (const uint16_t *)wb, (const uint8_t *)a_sexp, (const uint8_t *)b_sexp, (int)M,
                           (int)N, (int)K, (int)r, xoff, extra, C, ldc);
    else
        hipLaunchKernelGGL(dot_pipeline_kernel<false>, dim3(grid), dim3(kPThreads), 0, s, (const uint16_t *)wa,
                           (const uint16_t *)wb, (const uint8_t *)a_sexp, (const uint8_t *)b_sexp, (int)M,
                           (int)N, (int)K, (int)r, xoff, extra, C, ldc);
    return launch_status();
}

}  // namespace bdr
