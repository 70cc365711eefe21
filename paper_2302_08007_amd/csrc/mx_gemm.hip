// C = Ahat * Bhat^T on MX-quantized operands (Sec. V: both inputs of a tensor
// operation are MX-quantized along the reduction dimension).
//
// A is the packed image of an [M x K] tensor, B of an [N x K] tensor, both
// blocked along K.  A workgroup owns a 128 x 128 tile of C and walks K in steps
// of 64: every thread pulls the packed bits of 32 elements of A and 32 of B
// (two blocks each) from global memory, expands them exactly to BF16 (a BF16 has
// 8 significant bits, an MX element at most 7, and the scale is a power of two),
// and writes them to LDS; the four waves then feed 32x32x16 BF16 MFMAs from LDS
// and accumulate in FP32.  Global loads for the next K step are issued before the
// MFMAs of the current one, and LDS is double buffered, so one barrier per step.
//
// This is not the dot-product engine of Sec. IV-B (integer Hadamard tree with a
// conditional shift and fixed-point accumulation): that design targets a custom
// datapath.  On gfx950 the matrix cores take BF16, so the operands are brought to
// BF16 and the hardware does the rest.
#include "bdr_device.hpp"
#include "bdr_internal.hpp"

namespace bdr {

namespace {

constexpr int kBM = 128, kBN = 128, kBK = 64;
constexpr int kGemmThreads = 256;
constexpr int kPitch = kBK * 2;  // bytes per LDS row: 64 BF16 = eight 16-byte chunks
constexpr int kOperandBytes = kBM * kPitch;
// LDS rows are 128 bytes, so the same chunk of consecutive rows would sit on the
// same banks.  Chunk c of row r is stored at position c ^ (r & 7): eight
// consecutive rows then spread one chunk index over all 32 banks.
__device__ __forceinline__ int lds_chunk(int row, int chunk)
{
    return row * kPitch + ((chunk ^ (row & 7)) << 4);
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x3_a4 __attribute__((ext_vector_type(3), aligned(4)));
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));

// The packed bits one thread needs for 32 consecutive elements (two blocks) of a row.
template <int MB>
struct Packed {
    uint32_t c[MB + 1];  // 32 codes x (MB+1) bits = MB+1 dwords
    uint32_t se2, tau16; // two exponent bytes, two microexponent bytes
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

// Expand the 32 elements to BF16 and store them as chunks 4*half .. 4*half+3 of
// LDS row `row` of the operand tile at `base`.
template <int MB>
__device__ __forceinline__ void unpack_to_lds(const Packed<MB> &p, uint8_t *base, int row, int half)
{
    constexpr int CB = MB + 1;
    constexpr uint32_t CMASK = (1u << CB) - 1u, MMASK = (1u << MB) - 1u;
    uint32_t out[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {  // pair j: elements 2j, 2j+1, one microexponent bit
        const int blk = j >> 3;
        const int se = (int)((p.se2 >> (8 * blk)) & 0xffu);
        const int q = se - 127 - (MB - 1) - (int)((p.tau16 >> j) & 1u);
        uint32_t h[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int off = (2 * j + e) * CB;
            uint32_t c = p.c[off >> 5] >> (off & 31);
            if constexpr (CB != 8)
                if ((off & 31) + CB > 32) c |= p.c[((off >> 5) + 1) % CB] << (32 - (off & 31));
            c &= CMASK;
            h[e] = as_u(__builtin_ldexpf((float)(c & MMASK), q)) | ((c >> MB) << 31);
        }
        out[j] = (h[0] >> 16) | (h[1] & 0xffff0000u);  // exact: the low halves are zero
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const u32x4 w = {out[4 * v], out[4 * v + 1], out[4 * v + 2], out[4 * v + 3]};
        *reinterpret_cast<u32x4 *>(base + lds_chunk(row, 4 * half + v)) = w;
    }
}

template <int MBA, int MBB>
__global__ __launch_bounds__(kGemmThreads) void mx_gemm_kernel(
    const uint8_t *__restrict__ a_codes, const uint8_t *__restrict__ a_sexp,
    const uint8_t *__restrict__ a_mexp, const uint8_t *__restrict__ b_codes,
    const uint8_t *__restrict__ b_sexp, const uint8_t *__restrict__ b_mexp, int M, int N, int K,
    float *__restrict__ C, int64_t ldc)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];  // [2][A | B]

    // Tile order: workgroup ids go round-robin over the 8 XCDs, each with its own
    // L2, so give every XCD a contiguous range of tiles and walk that range in
    // groups of 8 tile rows per tile column to keep the operands of a group hot.
    const int ntm = M / kBM, ntn = N / kBN, total = ntm * ntn;
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
    const int m0 = tm * kBM, n0 = tn * kBN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // unpack role: row tid/2 of the tile, elements 32*(tid&1) .. +31 of the K step
    const int urow = tid >> 1, uhalf = tid & 1;
    const int64_t kblocks = K >> 4;
    int64_t a_blk = (int64_t)(m0 + urow) * kblocks + 2 * uhalf;
    int64_t b_blk = (int64_t)(n0 + urow) * kblocks + 2 * uhalf;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    Packed<MBA> pa;
    Packed<MBB> pb;
    const int nk = K / kBK;
    if (nk > 0) {
        load_packed<MBA>(a_codes, a_sexp, a_mexp, a_blk, pa);
        load_packed<MBB>(b_codes, b_sexp, b_mexp, b_blk, pb);
        unpack_to_lds<MBA>(pa, smem, urow, uhalf);
        unpack_to_lds<MBB>(pb, smem + kOperandBytes, urow, uhalf);
    }
    __syncthreads();

    // fragment addresses: lane l feeds row l % 32, k offset 8 * (l / 32) of a 32 x 16 slab
    const int f_row = lane & 31, f_half = lane >> 5;
    for (int kt = 0; kt < nk; ++kt) {
        const uint8_t *cur = smem + (kt & 1) * (2 * kOperandBytes);
        uint8_t *nxt = smem + ((kt + 1) & 1) * (2 * kOperandBytes);
        const bool more = kt + 1 < nk;
        if (more) {
            a_blk += 4;
            b_blk += 4;
            load_packed<MBA>(a_codes, a_sexp, a_mexp, a_blk, pa);
            load_packed<MBB>(b_codes, b_sexp, b_mexp, b_blk, pb);
        }
#pragma unroll
        for (int s = 0; s < kBK / 16; ++s) {
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[i] = *reinterpret_cast<const bf16x8 *>(
                    cur + lds_chunk(wm * 64 + i * 32 + f_row, 2 * s + f_half));
                fb[i] = *reinterpret_cast<const bf16x8 *>(
                    cur + kOperandBytes + lds_chunk(wn * 64 + i * 32 + f_row, 2 * s + f_half));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            unpack_to_lds<MBA>(pa, nxt, urow, uhalf);
            unpack_to_lds<MBB>(pb, nxt + kOperandBytes, urow, uhalf);
        }
        __syncthreads();
    }

    // 32 x 32 accumulator: register r of lane l is row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn * 64 + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                C[(int64_t)row * ldc + col] = acc[i][j][r];
            }
        }
}

template <int MBA, int MBB>
void launch_gemm(const uint8_t *ac, const uint8_t *as, const uint8_t *am, const uint8_t *bc,
                 const uint8_t *bs, const uint8_t *bm, int M, int N, int K, float *C, int64_t ldc,
                 hipStream_t s)
{
    const unsigned grid = (unsigned)((M / kBM) * (N / kBN));
    const size_t lds = 4 * (size_t)kOperandBytes;
    hipLaunchKernelGGL((mx_gemm_kernel<MBA, MBB>), dim3(grid), dim3(kGemmThreads), lds, s, ac, as,
                       am, bc, bs, bm, M, N, K, C, ldc);
}

template <int MBA>
void pick_b(int mb, const uint8_t *ac, const uint8_t *as, const uint8_t *am, const uint8_t *bc,
            const uint8_t *bs, const uint8_t *bm, int M, int N, int K, float *C, int64_t ldc,
            hipStream_t s)
{
    if (mb == 7)
        launch_gemm<MBA, 7>(ac, as, am, bc, bs, bm, M, N, K, C, ldc, s);
    else if (mb == 4)
        launch_gemm<MBA, 4>(ac, as, am, bc, bs, bm, M, N, K, C, ldc, s);
    else
        launch_gemm<MBA, 2>(ac, as, am, bc, bs, bm, M, N, K, C, ldc, s);
}

__global__ void gemm_zero_kernel(float *C, int64_t ldc, int N)
{
    const int64_t row = blockIdx.y;
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < N; c += gridDim.x * blockDim.x)
        C[row * ldc + c] = 0.f;
}

}  // namespace

int gemm(const bdr_format &fa, const bdr_format &fb, const void *a_codes, const void *a_sexp,
         const void *a_mexp, const void *b_codes, const void *b_sexp, const void *b_mexp,
         int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, hipStream_t s)
{
    if (K == 0) {  // empty sum
        hipLaunchKernelGGL(gemm_zero_kernel, dim3(4, (unsigned)M), dim3(256), 0, s, C, ldc, (int)N);
        return launch_status();
    }
    const uint8_t *ac = (const uint8_t *)a_codes, *as = (const uint8_t *)a_sexp,
                  *am = (const uint8_t *)a_mexp, *bc = (const uint8_t *)b_codes,
                  *bs = (const uint8_t *)b_sexp, *bm = (const uint8_t *)b_mexp;
    if (fa.m == 7)
        pick_b<7>(fb.m, ac, as, am, bc, bs, bm, (int)M, (int)N, (int)K, C, ldc, s);
    else if (fa.m == 4)
        pick_b<4>(fb.m, ac, as, am, bc, bs, bm, (int)M, (int)N, (int)K, C, ldc, s);
    else
        pick_b<2>(fb.m, ac, as, am, bc, bs, bm, (int)M, (int)N, (int)K, C, ldc, s);
    return launch_status();
}

}  // namespace bdr
