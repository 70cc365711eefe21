// Column-wise (blocks down the columns) quantize, dequantize and fused round
// trip, staged through LDS: kernels for the Table II formats, and further down one
// kernel that takes any format tuple at run time.
//
// MX is a directional format: a tensor must be quantized along the reduction
// axis, and quantizing does not commute with transposing (Sec. V, "Training").
// The result here is defined as the row-wise result on the transposed tensor,
// plane indices included, but the transpose is never materialized: a workgroup
// brings a 128-row tile (64 FP32 or 128 BF16 columns, 32 KiB) into LDS with
// row-contiguous 16-byte loads,
// each lane then reads one 16-row block of one column out of LDS, quantizes it
// entirely in registers (the block is in one lane, so no cross-lane reduction is
// needed), and the eight lanes that hold the eight consecutive blocks of one
// column write a contiguous run of the packed planes.
//
// LDS layout: row-major 16-byte chunks, chunk k of row r stored at position
// k ^ swz(r) where swz depends only on the block index r / 16.  Lanes of a wave
// read the same row offset of eight different blocks; the XOR puts those on
// different banks.
#include "bdr_device.hpp"
#include "bdr_internal.hpp"

namespace bdr {

namespace {

constexpr int kTR = 128;              // tile rows = kBPT blocks of 16 (64-row tiles measured slower)
constexpr int kBPT = kTR / 16;        // blocks per tile column (a power of two <= 8)
constexpr int kCPW = 64 / kBPT;       // columns a wave takes per pass
constexpr int kColThreads = 256;
// Column tiles an XCD sweeps before it moves down one row tile.  BF16 8192 x 12288, MX9 / MX6 / MX4
// quantize in microseconds: 2, 4, 8: 66 / 72 / 63; 16: 60 / 65 / 59; 32: 64 / 76 / 62; the whole row (96):
// 77 / 126 / 76.  Dequantize and the fused round trip do not depend on it.
constexpr uint32_t kColRun = 16;

typedef uint32_t u32x3_a4 __attribute__((ext_vector_type(3), aligned(4)));

template <typename T>
struct TileGeom;
template <>
struct TileGeom<uint16_t> {
    static constexpr int kTC = 128;              // tile columns: 256-byte row segments, 32 KiB tile
    static constexpr int kEPC = 8;               // elements per 16-byte chunk
    static constexpr int kChunks = kTC / kEPC;   // chunks per tile row
    __device__ static int swz(int r) { return (r >> 4) & 7; }
};
template <>
struct TileGeom<float> {
    static constexpr int kTC = 64;
    static constexpr int kEPC = 4;
    static constexpr int kChunks = kTC / kEPC;
    __device__ static int swz(int r) { return ((r >> 4) & 7) << 1; }
};

// byte offset of element (r, c) of the tile in LDS
template <typename T>
__device__ __forceinline__ int lds_off(int r, int c)
{
    typedef TileGeom<T> G;
    const int k = c / G::kEPC, e = c % G::kEPC;
    return (r * G::kChunks + (k ^ G::swz(r))) * 16 + e * (int)sizeof(T);
}

template <typename T, int THREADS = kColThreads>
__device__ __forceinline__ void tile_load(const T *__restrict__ x, int64_t ld, int64_t r0,
                                          int64_t c0, uint8_t *tile)
{
    typedef TileGeom<T> G;
    constexpr int kTotal = kTR * G::kChunks;
    static_assert(kTotal % THREADS == 0, "whole passes");
#pragma unroll
    for (int j = 0; j < kTotal / THREADS; ++j) {
        const int q = threadIdx.x + j * THREADS;
        const int r = q / G::kChunks, k = q % G::kChunks;
        const u32x4 v = ldg<true>(
            reinterpret_cast<const u32x4 *>(x + (r0 + r) * ld + c0 + k * G::kEPC));
        *reinterpret_cast<u32x4 *>(tile + (r * G::kChunks + (k ^ G::swz(r))) * 16) = v;
    }
}

template <typename T, int THREADS = kColThreads>
__device__ __forceinline__ void tile_store(T *__restrict__ y, int64_t ld, int64_t r0, int64_t c0,
                                           const uint8_t *tile)
{
    typedef TileGeom<T> G;
    constexpr int kTotal = kTR * G::kChunks;
    static_assert(kTotal % THREADS == 0, "whole passes");
#pragma unroll
    for (int j = 0; j < kTotal / THREADS; ++j) {
        const int q = threadIdx.x + j * THREADS;
        const int r = q / G::kChunks, k = q % G::kChunks;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(tile + (r * G::kChunks + (k ^ G::swz(r))) * 16);
        stg<true>(v, reinterpret_cast<u32x4 *>(y + (r0 + r) * ld + c0 + k * G::kEPC));
    }
}

__device__ __forceinline__ uint32_t lds_get(const uint8_t *tile, int off, float)
{
    return *reinterpret_cast<const uint32_t *>(tile + off);
}
__device__ __forceinline__ uint32_t lds_get(const uint8_t *tile, int off, uint16_t)
{
    return (uint32_t)*reinterpret_cast<const uint16_t *>(tile + off) << 16;
}
__device__ __forceinline__ void lds_put(uint8_t *tile, int off, uint32_t bits, float)
{
    *reinterpret_cast<uint32_t *>(tile + off) = bits;
}
__device__ __forceinline__ void lds_put(uint8_t *tile, int off, uint32_t bits, uint16_t)
{
    *reinterpret_cast<uint16_t *>(tile + off) = (uint16_t)(bits >> 16);
}

// Quantize one whole block held by one lane (no cross-lane step).
// w: the 16 codes packed little-endian, (MB+1) bits each.  yb only when DEQ.
template <int MB, bool DEQ>
__device__ __forceinline__ void mx_quant16(const uint32_t (&xb)[16], uint32_t (&w)[4],
                                           uint32_t &se, uint32_t &tau8, uint32_t (&yb)[16])
{
    constexpr int NW = MxWords<MB, 8>::kN;
    uint32_t ww[NW];
    mx_quant_lane<MB, 8, 0, DEQ>(xb, ww, se, tau8, yb);
#pragma unroll
    for (int k = 0; k < 4; ++k) w[k] = k < NW ? ww[k < NW ? k : 0] : 0u;
}

template <int MB>
__device__ __forceinline__ void mx_dequant16(const uint32_t (&w)[4], uint32_t se, uint32_t tau8,
                                             uint32_t (&yb)[16])
{
    constexpr int CB = MB + 1;
    constexpr uint32_t CMASK = (1u << CB) - 1u, MMASK = (1u << MB) - 1u;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int off = i * CB;
        uint32_t c = w[off >> 5] >> (off & 31);
        if ((off & 31) + CB > 32) c |= w[(off >> 5) + 1] << (32 - (off & 31));
        c &= CMASK;
        const int q = (int)se - 127 - (int)((tau8 >> (i >> 1)) & 1u) - (MB - 1);
        yb[i] = as_u(__builtin_ldexpf((float)(c & MMASK), q)) | ((c >> MB) << 31);
    }
}

// Packed codes of one block <-> global memory.  blk: block index in the codes
// plane.  Lanes 2p and 2p+1 hold blocks 2p and 2p+1 (blk parity = lane parity);
// for 5- and 3-bit codes a block is 10 or 6 bytes, so a pair of lanes shares its
// middle dword and exchanges 16 bits through DPP.
template <int MB>
__device__ __forceinline__ void codes_store(uint8_t *codes, int64_t blk, const uint32_t (&w)[4])
{
    constexpr int CB = MB + 1;
    const bool odd = blk & 1;
    if (CB == 8) {
        u32x4 v = {w[0], w[1], w[2], w[3]};
        stg<true>(v, reinterpret_cast<u32x4 *>(codes + 16 * blk));
    } else if (CB == 5) {
        const uint32_t ow0 = dpp<kQuadXor1>(w[0]);
        uint8_t *pb = codes + 20 * (blk >> 1);
        if (!odd) {
            u32x3_a4 v = {w[0], w[1], w[2] | (ow0 << 16)};
            *reinterpret_cast<u32x3_a4 *>(pb) = v;
        } else {
            store_pair_a4((w[0] >> 16) | (w[1] << 16), (w[1] >> 16) | (w[2] << 16), pb + 12);
        }
    } else {
        const uint32_t ow0 = dpp<kQuadXor1>(w[0]);
        uint8_t *pb = codes + 12 * (blk >> 1);
        if (!odd)
            store_pair_a4(w[0], w[1] | (ow0 << 16), pb);
        else
            *reinterpret_cast<uint32_t *>(pb + 8) = (w[0] >> 16) | (w[1] << 16);
    }
}

template <int MB>
__device__ __forceinline__ void codes_load(const uint8_t *codes, int64_t blk, uint32_t (&w)[4])
{
    constexpr int CB = MB + 1;
    const uint32_t s = 16u * (uint32_t)(blk & 1);
    w[0] = w[1] = w[2] = w[3] = 0;
    if (CB == 8) {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(codes + 16 * blk);
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    } else if (CB == 5) {
        // even block: dwords 0-2 of the pair's five; odd block: dwords 2-4, 16 bits in
        const u32x3_a4 v = *reinterpret_cast<const u32x3_a4 *>(codes + 20 * (blk >> 1) + 8 * (blk & 1));
        w[0] = funnel_r(v.y, v.x, s);
        w[1] = funnel_r(v.z, v.y, s);
        w[2] = (v.z >> s) & 0xffffu;
    } else {
        uint32_t v0, v1;
        load_pair_a4(codes + 12 * (blk >> 1) + 4 * (blk & 1), v0, v1);
        w[0] = funnel_r(v1, v0, s);
        w[1] = (v1 >> s) & 0xffffu;
    }
}

// Which tile a workgroup takes.  Tiles that follow each other down a column write adjacent
// runs of the planes (8 blocks each: 48 to 128 bytes of codes, 8 bytes of exponents), so a
// 64-byte line is shared by several workgroups.  Workgroups are dealt to the 8 XCDs round
// robin by their linear index; the index is remapped so that an XCD owns a band of
// consecutive row tiles and walks it in chunks of kColRun column tiles: row neighbours of a
// tile follow within kColRun workgroups on the same XCD, whose L2 then sees whole lines
// before it writes them back, while the tiles in flight still cover several KiB of every
// row they read.  With ALONG_ROWS (no plane is written) tiles simply follow each other along
// the rows of the tensor, so that the tiles in flight cover whole rows (measured: a 2-D tile
// copy runs 12 % faster this way than walking down the columns first); row neighbours then
// meet on one XCD whenever the number of column tiles is a multiple of 8, which keeps the
// plane lines they share in one L2.
template <bool ALONG_ROWS>
__device__ __forceinline__ void tile_of(uint32_t &tx, uint32_t &ty)
{
    const uint32_t gx = gridDim.x, lin = blockIdx.x + gx * blockIdx.y;
    tx = blockIdx.x;
    ty = blockIdx.y;
    if (ALONG_ROWS) {
        ty = lin % gridDim.y;
        tx = lin / gridDim.y;
    } else if (gx % 8 == 0) {
        const uint32_t per = gx / 8, xcd = lin % 8, j = lin / 8;
        uint32_t cw = kColRun;
        while (gridDim.y % cw) cw >>= 1;
        const uint32_t chunk = j / (per * cw), rem = j % (per * cw);
        tx = xcd * per + rem / cw;
        ty = chunk * cw + rem % cw;
    }
}

// Threads per tile.  Quantize runs fastest with one lane per block of the tile (BF16 8192 x
// 12288, MX9 / MX6 / MX4 in microseconds: 256 threads 65 / 73 / 66, 512: 62 / 72 / 64, 1024: 59 /
// 66 / 59); dequantize and the fused round trip, which end in the store of the tile, do not
// gain (48 / 42 / 39 -> 48 / 43 / 40 and 72 -> 74) and stay at 256.
template <typename T, int MODE>
constexpr int col_threads()
{
    return MODE == 0 ? kTR / 16 * TileGeom<T>::kTC : kColThreads;
}

// MODE 0 quantize (x -> planes), 1 dequantize (planes -> y), 2 fused (x -> y).
template <int MB, typename T, int MODE>
__global__ __launch_bounds__((col_threads<T, MODE>())) void mx_col_kernel(
    const T *x, T *y, uint8_t *__restrict__ codes, uint8_t *__restrict__ sexp,
    uint8_t *__restrict__ mexp, int64_t rows, int64_t ld)
{
    constexpr int kTC = TileGeom<T>::kTC;
    constexpr int THREADS = col_threads<T, MODE>(), kWaves = THREADS / 64;
    __shared__ __attribute__((aligned(16))) uint8_t tile[kTR * kTC * sizeof(T)];
    uint32_t tx, ty;
    tile_of<MODE != 0>(tx, ty);
    const int64_t r0 = (int64_t)tx * kTR;
    const int64_t c0 = (int64_t)ty * kTC;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = lane & (kBPT - 1), cl = lane / kBPT;
    const int64_t blocks_per_col = rows >> 4;

    if (MODE != 1) {
        tile_load<T, THREADS>(x, ld, r0, c0, tile);
        __syncthreads();
    }
#pragma unroll
    for (int it = 0; it < kTC / (kWaves * kCPW); ++it) {
        const int c = kCPW * (wave + kWaves * it) + cl;  // column inside the tile
        const int64_t blk = (c0 + c) * blocks_per_col + (r0 >> 4) + b;
        uint32_t xb[16], yb[16], w[4], se, tau8;
        if (MODE != 1) {
#pragma unroll
            for (int i = 0; i < 16; ++i) xb[i] = lds_get(tile, lds_off<T>(16 * b + i, c), T());
            mx_quant16<MB, MODE == 2>(xb, w, se, tau8, yb);
        }
        if (MODE == 0) {
            codes_store<MB>(codes, blk, w);
            sexp[blk] = (uint8_t)se;
            mexp[blk] = (uint8_t)tau8;
        }
        if (MODE == 1) {
            codes_load<MB>(codes, blk, w);
            mx_dequant16<MB>(w, sexp[blk], mexp[blk], yb);
        }
        if (MODE != 0) {
#pragma unroll
            for (int i = 0; i < 16; ++i) lds_put(tile, lds_off<T>(16 * b + i, c), yb[i], T());
        }
    }
    if (MODE != 0) {
        __syncthreads();
        tile_store<T, THREADS>(y, ld, r0, c0, tile);
    }
}

// Column blocks quantized straight into an operand image of the product kernel (see
// mx_quantize_operand_row_kernel): the operand is the transpose, so its rows are the tensor's
// columns and its K index the tensor's row.  The same tile, the same lane per block; a tile gives
// every one of its columns eight blocks, i.e. whole 64-byte pieces in two (FP6) or four (BF16) K
// steps, and the columns of a tile follow each other in the image, so a tile writes runs of
// 64 bytes x its columns: no partial lines, no neighbours to wait for.
constexpr int kOperandFp6B = 1, kOperandBf16 = 2, kOperandFp4 = 3;  // (0: FP6, A operand)

template <int MB, typename T, int KIND>
__global__ __launch_bounds__((col_threads<T, 0>())) void mx_col_operand_kernel(
    const T *x, u32x4 *__restrict__ out, int64_t cols, int64_t ld, uint8_t *__restrict__ scales)
{
    constexpr int kTC = TileGeom<T>::kTC;
    constexpr int THREADS = col_threads<T, 0>();
    __shared__ __attribute__((aligned(16))) uint8_t tile[kTR * kTC * sizeof(T)];
    uint32_t tx, ty;
    tile_of<true>(tx, ty);
    const int64_t r0 = (int64_t)tx * kTR, c0 = (int64_t)ty * kTC;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = lane & (kBPT - 1), c = kCPW * wave + lane / kBPT;  // one pass: THREADS = kBPT * kTC
    static_assert(THREADS == kBPT * kTC, "one lane per block of the tile");
    constexpr bool kFp6 = KIND == 0 || KIND == kOperandFp6B;
    __shared__ uint8_t s_map[kFp6 ? 128 : 1];
    if constexpr (kFp6) fp6_map_fill<MB>(s_map);
    tile_load<T, THREADS>(x, ld, r0, c0, tile);
    __syncthreads();
    uint32_t xb[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) xb[i] = lds_get(tile, lds_off<T>(16 * b + i, c), T());
    if constexpr (KIND == kOperandFp4) {
        // The tile's 128 rows are one K step of the FP4 image, a column's eight lanes hold its
        // eight blocks: 8 bytes of codes each (64 contiguous bytes per column; columns with bit 4
        // set keep the two blocks of a chunk in swapped order), and the eight scale bytes, gathered
        // by three DPP steps into the even blocks' word (lane 0) and the odd blocks' (lane 1).
        static_assert(MB == 2 && kBPT == 8, "MX4, eight blocks per K step");
        uint32_t w0, w1, scale;
        mx_quant_fp4_block(xb, w0, w1, scale);
        const int64_t col = c0 + c, step = tx;
        const int half = (b & 1) ^ (int)((col >> 4) & 1);
        stg<true>(u32x2{w0, w1}, reinterpret_cast<u32x2 *>(reinterpret_cast<uint8_t *>(out) +
                                                           ((step * cols + col) * 4 + (b >> 1)) * 16 + 8 * half));
        uint32_t sw = scale << (8 * (b >> 1));
        sw |= dpp<kQuadXor2>(sw);
        sw |= dpp<kQuadXor1>(dpp<kQuadXor2>(dpp<kRowHalfMirror>(sw)));  // lane b ^ 4
        if (b < 2) *reinterpret_cast<uint32_t *>(scales + (step * cols + col) * 8 + 4 * b) = sw;
    } else if constexpr (KIND != kOperandBf16) {
        // four lanes write one 64-byte piece, a wave 512 contiguous bytes in each of two K steps
        const int64_t kb = (r0 >> 4) + b;
        const u32x4 chunk = mx_quant_fp6_block<MB, KIND == kOperandFp6B>(xb, s_map);
        stg<true>(chunk, out + (((kb >> 2) * cols + (c0 + c)) * 4 + (kb & 3)));
    } else {
        // A lane's two chunks would leave as 16-byte pieces 32 bytes apart (86 us for 8192 x 12288
        // BF16).  The tile's part of the image (four K steps x kTC columns x 64 bytes, never more
        // than the tile itself) is put together in the tile's own LDS instead and leaves as whole
        // runs of kTC x 64 bytes, a wave writing 1 KiB in a row per store (73 us).  For the FP6
        // image the same detour costs more than it saves (67 -> 71-74 us).
        constexpr int kSteps = kTR / 32;
        static_assert(kSteps * kTC * 64 <= (int)sizeof(tile), "the image of a tile fits in the tile");
        static_assert((kSteps * kTC * 4) % THREADS == 0, "whole passes");
        u32x4 *img = reinterpret_cast<u32x4 *>(tile);
        u32x4 v0, v1;
        mx_quant_bf16_block<MB>(xb, v0, v1);
        __syncthreads();  // every lane has its block in registers
        img[((b >> 1) * kTC + c) * 4 + 2 * (b & 1)] = v0;
        img[((b >> 1) * kTC + c) * 4 + 2 * (b & 1) + 1] = v1;
        __syncthreads();
        const int64_t step0 = r0 / 32;
#pragma unroll
        for (int i = threadIdx.x; i < kSteps * kTC * 4; i += THREADS) {
            const int st = i / (kTC * 4), w = i % (kTC * 4);
            stg<true>(img[i], out + (((step0 + st) * cols + c0) * 4 + w));
        }
    }
}

template <int MB, typename T>
void launch_operand_col(int kind, dim3 grid, hipStream_t s, const T *x, u32x4 *o, int64_t cols, int64_t ld,
                        uint8_t *scales)
{
    const dim3 block(col_threads<T, 0>());
    if (kind == kOperandBf16)
        hipLaunchKernelGGL((mx_col_operand_kernel<MB, T, kOperandBf16>), grid, block, 0, s, x, o, cols, ld, scales);
    else if constexpr (MB <= 4) {
        if (kind == kOperandFp6B)
            hipLaunchKernelGGL((mx_col_operand_kernel<MB, T, kOperandFp6B>), grid, block, 0, s, x, o, cols, ld, scales);
        else if (kind == 0)
            hipLaunchKernelGGL((mx_col_operand_kernel<MB, T, 0>), grid, block, 0, s, x, o, cols, ld, scales);
        else if constexpr (MB == 2)
            hipLaunchKernelGGL((mx_col_operand_kernel<2, T, kOperandFp4>), grid, block, 0, s, x, o, cols, ld, scales);
    }
}

template <typename T>
int quantize_operand_col_t(const bdr_format &f, const T *x, int64_t rows, int64_t cols, int64_t ld, void *out,
                           int kind, hipStream_t s)
{
    const dim3 grid((unsigned)(rows / kTR), (unsigned)(cols / TileGeom<T>::kTC));
    u32x4 *o = (u32x4 *)out;
    // FP4 kind: the scale image follows the chunks (the operand is [cols x rows]: half a byte per element)
    uint8_t *scales = kind == kOperandFp4 ? (uint8_t *)out + cols * (rows / 2) : nullptr;
    if (f.m == 7)
        launch_operand_col<7, T>(kind, grid, s, x, o, cols, ld, scales);
    else if (f.m == 4)
        launch_operand_col<4, T>(kind, grid, s, x, o, cols, ld, scales);
    else
        launch_operand_col<2, T>(kind, grid, s, x, o, cols, ld, scales);
    return launch_status();
}

template <int MB, typename T>
void launch_col(int mode, const T *x, T *y, uint8_t *codes, uint8_t *sexp, uint8_t *mexp,
                int64_t rows, int64_t cols, int64_t ld, hipStream_t s)
{
    const dim3 grid((unsigned)(rows / kTR), (unsigned)(cols / TileGeom<T>::kTC));
    if (mode == 0)
        hipLaunchKernelGGL((mx_col_kernel<MB, T, 0>), grid, dim3(col_threads<T, 0>()), 0, s, x, y, codes, sexp, mexp, rows, ld);
    else if (mode == 1)
        hipLaunchKernelGGL((mx_col_kernel<MB, T, 1>), grid, dim3(col_threads<T, 1>()), 0, s, x, y, codes, sexp, mexp, rows, ld);
    else
        hipLaunchKernelGGL((mx_col_kernel<MB, T, 2>), grid, dim3(col_threads<T, 2>()), 0, s, x, y, codes, sexp, mexp, rows, ld);
}

template <typename T>
int col_dispatch(int mode, const bdr_format &f, const T *x, T *y, uint8_t *codes, uint8_t *sexp,
                 uint8_t *mexp, int64_t rows, int64_t cols, int64_t ld, hipStream_t s)
{
    if (f.m == 7)
        launch_col<7, T>(mode, x, y, codes, sexp, mexp, rows, cols, ld, s);
    else if (f.m == 4)
        launch_col<4, T>(mode, x, y, codes, sexp, mexp, rows, cols, ld, s);
    else
        launch_col<2, T>(mode, x, y, codes, sexp, mexp, rows, cols, ld, s);
    return launch_status();
}

// ---- any format tuple with 8 <= k1 <= 128 on the same tiles
//
// The same staging (row-contiguous loads of a 128-row tile into LDS, one lane per block of
// one column), with the tuple at run time: a lane walks its block in LDS three times (block
// maximum; per sub-block its maximum; per element the code), packs the codes of its block
// (a whole number of bytes, since k1 is a multiple of 8) into a staging area in LDS, and the
// workgroup then writes each column's run of the three planes with consecutive lanes.  The
// microexponent stream of a column gets (128 / k2) d2 bits per tile; where that is not a
// whole number of bytes the workgroup walks rt = 2, 4 or 8 tiles down the column and writes
// the stream once at the end.  Dequantize and the fused round trip use the same walk.
// smallest number of tiles (1, 2, 4, 8) down a column whose microexponent bits fill whole bytes
__host__ __device__ constexpr int tiles_for_whole_bytes(const GenFmt &f)
{
    for (int rt = 1; rt < 8; rt *= 2)
        if (rt * (kTR / f.k2) * f.d2 % 8 == 0) return rt;
    return 8;
}

constexpr int kGenCodesMax = 16 * 9 + 4;  // bytes per tile column: 128 codes of up to 9 bits (+ read-ahead)
constexpr int kGenSexpMax = 16;           // 128 / k1 with k1 >= 8
constexpr int kGenMexpMax = 48 + 4;       // (128 / k2) d2 / 8 with k2 = 1, d2 = 3 (taller bands have larger k2) + read-ahead

// SPEC >= 0: the tuple is entry SPEC of the table of formats the general kernels are compiled for
// (hot_format), so the walks unroll and the shifts are immediates; SPEC < 0: tuple at run time.
template <typename T, int MODE, int SPEC = -1>
__global__ __launch_bounds__(kColThreads) void generic_col_tiled_kernel(
    GenFmt f_arg, int rt_arg, const T *x, T *y, uint8_t *__restrict__ codes, uint8_t *__restrict__ sexp,
    uint8_t *__restrict__ mexp, int64_t rows, int64_t ld)
{
    const GenFmt f = SPEC >= 0 ? hot_format(SPEC >= 0 ? SPEC : 0) : f_arg;
    const int rt = SPEC >= 0 ? tiles_for_whole_bytes(hot_format(SPEC >= 0 ? SPEC : 0)) : rt_arg;
    constexpr int kTC = TileGeom<T>::kTC;
    __shared__ __attribute__((aligned(16))) uint8_t tile[kTR * kTC * sizeof(T)];
    __shared__ uint32_t s_codes[MODE == 2 ? 1 : kTC * kGenCodesMax / 4];
    __shared__ uint8_t s_sexp[MODE == 2 ? 1 : kTC * kGenSexpMax];
    __shared__ uint32_t s_mexp[MODE == 2 ? 1 : kTC * kGenMexpMax / 4];
    uint8_t *const lc = reinterpret_cast<uint8_t *>(s_codes);
    uint8_t *const lm = reinterpret_cast<uint8_t *>(s_mexp);

    const int cb = f.m + 1, lk1 = __builtin_ctz(f.k1), lk2 = __builtin_ctz(f.k2);
    const int nb = kTR >> lk1, lnb = __builtin_ctz(nb);  // blocks per tile column
    const int nsub = f.k1 >> lk2;                        // sub-blocks per block
    const int beta = (1 << f.d2) - 1;
    const float top = (float)((1u << f.m) - 1u);
    const uint32_t cmask = (1u << cb) - 1u, mmask = (1u << f.m) - 1u;
    const int mbytes = rt * (kTR >> lk2) * f.d2 / 8;     // microexponent bytes per column and band
    uint32_t tx, ty;
    tile_of<MODE != 0>(tx, ty);
    const int64_t band0 = (int64_t)tx * rt * kTR, c0 = (int64_t)ty * kTC;
    const int tid = threadIdx.x;

    if (MODE != 2 && f.d2 > 0) {
        if (MODE == 0) {
            for (int i = tid; i < kTC * kGenMexpMax / 4; i += kColThreads) s_mexp[i] = 0;
        } else {
            for (int i = tid; i < kTC * mbytes; i += kColThreads) {
                const int c = i / mbytes, b = i - c * mbytes;
                lm[c * kGenMexpMax + b] = mexp[((((c0 + c) * rows + band0) >> lk2) * f.d2 >> 3) + b];
            }
        }
    }
    for (int it = 0; it < rt; ++it) {
        const int64_t r0 = band0 + (int64_t)it * kTR;
        if (MODE != 1) tile_load(x, ld, r0, c0, tile);
        if (MODE == 1) {
            for (int i = tid; i < kTC * 4 * cb; i += kColThreads) {
                const int c = i / (4 * cb), w = i - c * 4 * cb;
                s_codes[c * (kGenCodesMax / 4) + w] =
                    reinterpret_cast<const uint32_t *>(codes + (((c0 + c) * rows + r0) * cb >> 3))[w];
            }
            for (int i = tid; i < kTC * nb; i += kColThreads) {
                const int c = i >> lnb, b = i & (nb - 1);
                s_sexp[c * kGenSexpMax + b] = sexp[(((c0 + c) * rows + r0) >> lk1) + b];
            }
        }
        __syncthreads();
        for (int q = tid; q < kTC * nb; q += kColThreads) {
            const int c = q >> lnb, b = q & (nb - 1), rbase = b << lk1;
            int mpos = ((it * kTR + rbase) >> lk2) * f.d2;  // bit of this block's first field in the column's stream
            if (MODE != 1) {
                uint32_t bm = 0;
                for (int i = 0; i < f.k1; ++i)
                    bm = umax(bm, clamp_mag(lds_get(tile, lds_off<T>(rbase + i, c), T()) & kAbsMask));
                const int se = (int)(bm >> 23);
                uint64_t acc = 0;
                int nbits = 0;
                uint8_t *cp = lc + c * kGenCodesMax + (rbase * cb >> 3);
                for (int j = 0; j < nsub; ++j) {
                    const int e0 = rbase + (j << lk2);
                    uint32_t sm = 0;
                    for (int e = 0; e < f.k2; ++e)
                        sm = umax(sm, clamp_mag(lds_get(tile, lds_off<T>(e0 + e, c), T()) & kAbsMask));
                    int t = se - (int)(sm >> 23);
                    t = t < beta ? t : beta;
                    const int sh = (f.m - 1) + 127 - se + t;
                    if (MODE == 0 && f.d2 > 0) {
                        uint32_t *mw = s_mexp + c * (kGenMexpMax / 4) + (mpos >> 5);
                        atomicOr(mw, (uint32_t)t << (mpos & 31));
                        if ((mpos & 31) + f.d2 > 32) atomicOr(mw + 1, (uint32_t)t >> (32 - (mpos & 31)));
                        mpos += f.d2;
                    }
                    for (int e = 0; e < f.k2; ++e) {
                        const int off = lds_off<T>(e0 + e, c);
                        const uint32_t xb = lds_get(tile, off, T());
                        const float mf = gen_round(__builtin_fabsf(as_f(xb)), sh, top, f.rounding);
                        if (MODE == 0) {
                            acc |= (uint64_t)((uint32_t)mf | ((xb >> 31) << f.m)) << nbits;
                            nbits += cb;
                            while (nbits >= 8) {
                                *cp++ = (uint8_t)acc;
                                acc >>= 8;
                                nbits -= 8;
                            }
                        } else {
                            lds_put(tile, off, as_u(__builtin_ldexpf(mf, -sh)) | (xb & 0x80000000u), T());
                        }
                    }
                }
                if (MODE == 0) s_sexp[c * kGenSexpMax + b] = (uint8_t)se;
            } else {
                const int se = s_sexp[c * kGenSexpMax + b];
                const uint8_t *cp = lc + c * kGenCodesMax;
                const uint8_t *mp = lm + c * kGenMexpMax;
                for (int j = 0; j < nsub; ++j) {
                    int tau = 0;
                    if (f.d2 > 0) {
                        const int byte = mpos >> 3;  // a field of up to 3 bits spans at most two bytes
                        tau = (int)((((uint32_t)mp[byte] | ((uint32_t)mp[byte + 1] << 8)) >> (mpos & 7)) & (uint32_t)beta);
                        mpos += f.d2;
                    }
                    const int qe = se - 127 - tau - (f.m - 1);
                    const int e0 = rbase + (j << lk2);
                    for (int e = 0; e < f.k2; ++e) {
                        const int bit = (e0 + e) * cb, byte = bit >> 3;  // up to 9 bits from bit 0 .. 7: two bytes
                        const uint32_t cd = ((((uint32_t)cp[byte] | ((uint32_t)cp[byte + 1] << 8)) >> (bit & 7))) & cmask;
                        lds_put(tile, lds_off<T>(e0 + e, c),
                                as_u(__builtin_ldexpf((float)(cd & mmask), qe)) | ((cd >> f.m) << 31), T());
                    }
                }
            }
        }
        __syncthreads();
        if (MODE == 0) {
            for (int i = tid; i < kTC * 4 * cb; i += kColThreads) {
                const int c = i / (4 * cb), w = i - c * 4 * cb;
                reinterpret_cast<uint32_t *>(codes + (((c0 + c) * rows + r0) * cb >> 3))[w] =
                    s_codes[c * (kGenCodesMax / 4) + w];
            }
            for (int i = tid; i < kTC * nb; i += kColThreads) {
                const int c = i >> lnb, b = i & (nb - 1);
                sexp[(((c0 + c) * rows + r0) >> lk1) + b] = s_sexp[c * kGenSexpMax + b];
            }
        } else {
            tile_store(y, ld, r0, c0, tile);
        }
        if (it + 1 < rt) __syncthreads();  // the tile and the staging areas are reused
    }
    if (MODE == 0 && f.d2 > 0) {
        for (int i = tid; i < kTC * mbytes; i += kColThreads) {
            const int c = i / mbytes, b = i - c * mbytes;
            mexp[((((c0 + c) * rows + band0) >> lk2) * f.d2 >> 3) + b] = lm[c * kGenMexpMax + b];
        }
    }
}

// Tiles walked per workgroup so that a column's microexponent bits come to whole bytes, or 0
// when this kernel does not take the case.
int generic_tiled_rt(const bdr_format &f, int64_t rows, int64_t cols, int tc)
{
    if (f.k1 < 8 || f.k1 > kTR || rows % kTR != 0 || cols % tc != 0 || cols / tc > 65535) return 0;
    for (int rt = 1; rt <= 8; rt *= 2) {
        if (rows % ((int64_t)rt * kTR) != 0) return 0;
        const int bits = rt * (kTR / f.k2) * f.d2;
        if (bits % 8 == 0 && bits / 8 <= kGenMexpMax - 4) return rt;
    }
    return 0;
}

// Compiled-in tuples: launch the kernel of table entry `spec` (rt must be what the kernel
// derives for itself: tiles_for_whole_bytes of the entry).
template <typename T, int MODE, int SP = 0>
void launch_generic_tiled_hot(int spec, dim3 grid, hipStream_t s, const GenFmt &g, int rt, const T *x, T *y,
                              uint8_t *codes, uint8_t *sexp, uint8_t *mexp, int64_t rows, int64_t ld)
{
    if constexpr (SP < kHotCount) {
        if (spec != SP)
            return launch_generic_tiled_hot<T, MODE, SP + 1>(spec, grid, s, g, rt, x, y, codes, sexp, mexp, rows, ld);
        hipLaunchKernelGGL((generic_col_tiled_kernel<T, MODE, SP>), grid, dim3(kColThreads), 0, s, g, rt, x, y,
                           codes, sexp, mexp, rows, ld);
    }
}

template <typename T>
int generic_tiled(int mode, const bdr_format &f, int rt, const T *x, T *y, uint8_t *codes, uint8_t *sexp,
                  uint8_t *mexp, int64_t rows, int64_t cols, int64_t ld, hipStream_t s)
{
    const GenFmt g{f.k1, f.k2, f.d2, f.m, f.rounding};
    const dim3 grid((unsigned)(rows / ((int64_t)rt * kTR)), (unsigned)(cols / TileGeom<T>::kTC)), block(kColThreads);
    bdr_format fr = f;
    if (mode == 1) fr.rounding = BDR_RNE;  // reading an image does not depend on how it was rounded
    const int spec = hot_index(fr);
    if (spec >= 0 && rt == tiles_for_whole_bytes(hot_format(spec))) {
        if (mode == 0)
            launch_generic_tiled_hot<T, 0>(spec, grid, s, g, rt, x, y, codes, sexp, mexp, rows, ld);
        else if (mode == 1)
            launch_generic_tiled_hot<T, 1>(spec, grid, s, g, rt, x, y, codes, sexp, mexp, rows, ld);
        else
            launch_generic_tiled_hot<T, 2>(spec, grid, s, g, rt, x, y, codes, sexp, mexp, rows, ld);
        return launch_status();
    }
    if (mode == 0)
        hipLaunchKernelGGL((generic_col_tiled_kernel<T, 0>), grid, block, 0, s, g, rt, x, y, codes, sexp, mexp, rows, ld);
    else if (mode == 1)
        hipLaunchKernelGGL((generic_col_tiled_kernel<T, 1>), grid, block, 0, s, g, rt, x, y, codes, sexp, mexp, rows, ld);
    else
        hipLaunchKernelGGL((generic_col_tiled_kernel<T, 2>), grid, block, 0, s, g, rt, x, y, codes, sexp, mexp, rows, ld);
    return launch_status();
}

// The tiled kernels need whole tiles and a grid the hardware accepts.
bool tiled_ok(int mode, const bdr_format &f, int64_t rows, int64_t cols, int tc)
{
    // dequantize (mode 1) only reads the image: the rounding rule plays no part
    return (mode == 1 ? is_mx_layout(f) : is_mx(f)) && rows % kTR == 0 && cols % tc == 0 && cols / tc <= 65535;
}

int col_any(int mode, const bdr_format &f, const void *x, void *y, int dtype, int64_t rows,
            int64_t cols, int64_t ld, void *codes, void *sexp, void *mexp, hipStream_t s)
{
    const int tc = dtype == BDR_F32 ? TileGeom<float>::kTC : TileGeom<uint16_t>::kTC;
    if (!tiled_ok(mode, f, rows, cols, tc)) {
        const int rt = generic_tiled_rt(f, rows, cols, tc);
        if (rt == 0) return generic_col(mode, f, x, y, dtype, rows, cols, ld, codes, sexp, mexp, s);
        if (dtype == BDR_F32)
            return generic_tiled(mode, f, rt, (const float *)x, (float *)y, (uint8_t *)codes, (uint8_t *)sexp,
                                 (uint8_t *)mexp, rows, cols, ld, s);
        return generic_tiled(mode, f, rt, (const uint16_t *)x, (uint16_t *)y, (uint8_t *)codes, (uint8_t *)sexp,
                             (uint8_t *)mexp, rows, cols, ld, s);
    }
    if (dtype == BDR_F32)
        return col_dispatch(mode, f, (const float *)x, (float *)y, (uint8_t *)codes,
                            (uint8_t *)sexp, (uint8_t *)mexp, rows, cols, ld, s);
    return col_dispatch(mode, f, (const uint16_t *)x, (uint16_t *)y, (uint8_t *)codes,
                        (uint8_t *)sexp, (uint8_t *)mexp, rows, cols, ld, s);
}

}  // namespace

// x [rows x cols] with blocks down the columns (K = rows): rows a multiple of 128, cols of the
// tile width (64 FP32 / 128 BF16 columns).  false: the shape is not made of whole tiles (the
// caller reports it).
bool quantize_operand_col_ok(int dtype, int64_t rows, int64_t cols)
{
    const int tc = dtype == BDR_F32 ? TileGeom<float>::kTC : TileGeom<uint16_t>::kTC;
    return rows % kTR == 0 && cols % tc == 0 && cols / tc <= 65535;
}

int quantize_operand_col(const bdr_format &f, const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld,
                         void *out, int kind, hipStream_t s)
{
    if (dtype == BDR_F32) return quantize_operand_col_t(f, (const float *)x, rows, cols, ld, out, kind, s);
    return quantize_operand_col_t(f, (const uint16_t *)x, rows, cols, ld, out, kind, s);
}

int quantize_col(const bdr_format &f, const void *x, int dtype, int64_t rows, int64_t cols,
                 int64_t ld, void *codes, void *sexp, void *mexp, hipStream_t s)
{
    return col_any(0, f, x, nullptr, dtype, rows, cols, ld, codes, sexp, mexp, s);
}

int dequantize_col(const bdr_format &f, const void *codes, const void *sexp, const void *mexp,
                   int64_t rows, int64_t cols, void *y, int dtype, int64_t ld, hipStream_t s)
{
    return col_any(1, f, nullptr, y, dtype, rows, cols, ld, const_cast<void *>(codes),
                   const_cast<void *>(sexp), const_cast<void *>(mexp), s);
}

int qdq_col(const bdr_format &f, const void *x, void *y, int dtype, int64_t rows, int64_t cols,
            int64_t ld, hipStream_t s)
{
    return col_any(2, f, x, y, dtype, rows, cols, ld, nullptr, nullptr, nullptr, s);
}

}  // namespace bdr
