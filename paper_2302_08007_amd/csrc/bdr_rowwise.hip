// Row-wise (blocks along the contiguous axis) quantize, dequantize and fused
// round trip.
//
// Two families of kernels:
//   mx_*      the Table II formats (k1 16, k2 2, d2 1, nearest-even), m in {7,4,2}.
//             One lane owns 8 consecutive elements (four sub-blocks, half a
//             block); the two lanes of a block meet through one DPP quad
//             permute.  HBM bound: every byte is read once and written once;
//             FP32 tensors move as fully contiguous 1 KiB wave rows staged
//             through wave-private LDS (wave_load512 / wave_store512).
//   generic_* any format the library accepts, parameters at run time.
//
// Quantization follows Sec. IX of the paper: the shared exponent is the exponent
// of the block maximum (Eq. "max_exp"), a sub-block is shifted down by
// tau = min(2^d2 - 1, E - E_sub) (Eq. "q_error_max-1" and the text after
// "q_error_all"), and the magnitude is rounded to m bits whose top bit has weight
// 2^(E - tau) (Eq. "max_exp_round").  All scaling is by powers of two through
// ldexp, which is exact, so codes match an integer implementation bit for bit.
#include "bdr_device.hpp"
#include "bdr_internal.hpp"

namespace bdr {

constexpr int kThreads = 256;
// Workgroup size of the Table II quantize kernel.  Measured in the loop of the three formats
// at 1 GiB FP32 (MX9 / MX6 / MX4, microseconds): 64 threads 215 / 202 / 195, 128: 211 / 198 /
// 194, 256: 217 / 198 / 195, 512: 211 / 203 / 199, 1024: 222 / 220 / 213; BF16 rows do not care.
constexpr int kQThreads = 128;
constexpr int kTileElems = kThreads * 8;

// ---------------------------------------------------------------- MX fast path

// Quantize the 8 elements of one lane (half a block; the other half is the
// neighbouring lane).  lo/hi: the 8 codes packed little-endian, (MB+1) bits each.
template <int MB, bool DEQ>
__device__ __forceinline__ void mx_quant8(const uint32_t (&xb)[8], uint32_t &lo, uint32_t &hi,
                                          uint32_t &se, uint32_t &tau4, uint32_t (&yb)[8])
{
    uint32_t w[MxWords<MB, 4>::kN];
    mx_quant_lane<MB, 4, 1, DEQ>(xb, w, se, tau4, yb);
    lo = w[0];
    hi = MxWords<MB, 4>::kN > 1 ? w[MxWords<MB, 4>::kN - 1] : 0u;
}

// One-shot grids (measured: persistent grids are slower on this chip).  Groups of 8
// elements a lane quantizes: BF16 rows bring only 16 bytes per group, so a lane takes
// four to have enough bytes in flight; FP32 rows are best with one (two cost 2 %).
template <typename T>
constexpr int q_iter() { return sizeof(T) == 2 ? 4 : 1; }

// Store the 8 codes of a lane (group g), packed little-endian in lo / hi, CB bits each.
// Whole quads of lanes call it together: for 5- and 3-bit codes a quad's 20 or 12 bytes
// leave as aligned dwords after a funnel shift across the quad.
template <int CB>
__device__ __forceinline__ void store_codes_quad(uint32_t lo, uint32_t hi, int64_t g,
                                                 uint8_t *__restrict__ codes)
{
    static_assert(CB == 8 || CB == 5 || CB == 3, "code widths with a quad funnel");
    const uint32_t i = threadIdx.x & 3u;
    const int64_t quad = g >> 2;
    if (CB == 8) {
        u32x2 v = {lo, hi};
        stg<kNtPlanes>(v, reinterpret_cast<u32x2 *>(codes + 8 * g));
    } else if (CB == 5) {
        // A quad holds 4 x 40 bits = 5 dwords.  Lane 0 writes dwords 0-1, lane i
        // writes dword i + 1; each needs the low word of the next lane.
        const uint32_t nlo = dpp<kQuadNext>(lo);
        const uint32_t whi = hi | (nlo << 8);
        uint8_t *qb = codes + 20 * quad;
        if (i == 0) {
            store_pair_a4(lo, whi, qb);
        } else {
            stg<kNtPlanes>(funnel_r(whi, lo, 32u - 8u * i),
                                  reinterpret_cast<uint32_t *>(qb + 4 * (i + 1)));
        }
    } else {
        // CB == 3: a quad holds 4 x 24 bits = 3 dwords, written by lanes 0-2.
        const uint32_t nlo = dpp<kQuadNext>(lo);
        if (i < 3)
            stg<kNtPlanes>((lo >> (8u * i)) | (nlo << (24u - 8u * i)),
                                  reinterpret_cast<uint32_t *>(codes + 12 * quad + 4 * i));
    }
}

// Pack and store what one lane produced for its 8 elements (group g).
template <int MB>
__device__ __forceinline__ void mx_store_group(uint32_t lo, uint32_t hi, uint32_t se, uint32_t tau4,
                                               int64_t g, uint8_t *__restrict__ codes,
                                               uint8_t *__restrict__ sexp,
                                               uint8_t *__restrict__ mexp)
{
    const uint32_t i = threadIdx.x & 3u;
    const int64_t quad = g >> 2;
    store_codes_quad<MB + 1>(lo, hi, g, codes);

    // The quad's two exponent bytes and two microexponent bytes, gathered with
    // two DPP ORs; lane 0 writes the exponents, lane 2 the microexponents.
    uint32_t r = (tau4 << (4u * i)) | (se << (16u + 8u * (i >> 1)));
    r |= dpp<kQuadXor1>(r);
    r |= dpp<kQuadXor2>(r);
    if ((i & 1u) == 0) {
        uint8_t *dst = i == 0 ? sexp : mexp;
        const uint16_t val = i == 0 ? (uint16_t)(r >> 16) : (uint16_t)(r & 0xffffu);
        *reinterpret_cast<uint16_t *>(dst + 2 * quad) = val;
    }
}

// The planes of the ITERS x 64 consecutive groups one wave quantized (group gw + 64 it + lane in
// it-th place), written from LDS of the wave's own.  A quad's 20 or 12 bytes of 5- or 3-bit codes
// and its 2 + 2 exponent bytes would otherwise leave as 2-, 4- and 8-byte pieces, four store
// instructions of such pieces per 64 groups.  Here they are put together in LDS (the same quad
// funnel, the same DPP gather of the exponent bytes as mx_store_group) and leave as 16-byte
// chunks of consecutive memory: one or two store instructions for the codes (8-bit codes are 8
// consecutive bytes per lane and go out directly), one for both exponent planes.  All 64 lanes
// call it; gw is a multiple of 64, the plane pointers are 16-byte aligned.
template <int MB, int ITERS>
struct WavePlanes {
    static constexpr int CB = MB + 1, kGroups = 64 * ITERS;
    static constexpr int kCodeBytes = CB == 8 ? 0 : kGroups * CB, kExpBytes = kGroups / 2;
    static constexpr int kBytes = kCodeBytes + 2 * kExpBytes;
    static_assert(kCodeBytes % 16 == 0 && kExpBytes % 16 == 0 && 2 * kExpBytes / 16 <= 64, "whole chunks");
};

template <int MB, int ITERS>
__device__ __forceinline__ void wave_store_planes(const uint32_t (&lo)[ITERS], const uint32_t (&hi)[ITERS],
                                                  const uint32_t (&se)[ITERS], const uint32_t (&tau4)[ITERS],
                                                  int64_t gw, uint8_t *sp, uint8_t *__restrict__ codes,
                                                  uint8_t *__restrict__ sexp, uint8_t *__restrict__ mexp)
{
    typedef WavePlanes<MB, ITERS> W;
    constexpr int CB = W::CB;
    const int lane = threadIdx.x & 63;
    const uint32_t i = lane & 3u;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int quad = it * 16 + (lane >> 2);
        uint32_t *qw = reinterpret_cast<uint32_t *>(sp) + quad * CB;  // the quad's CB dwords
        const uint32_t nlo = dpp<kQuadNext>(lo[it]);
        if (CB == 8) {
            stg<kNtPlanes>(u32x2{lo[it], hi[it]}, reinterpret_cast<u32x2 *>(codes + 8 * (gw + it * 64 + lane)));
        } else if (CB == 5) {
            const uint32_t whi = hi[it] | (nlo << 8);
            if (i == 0) {
                qw[0] = lo[it];
                qw[1] = whi;
            } else {
                qw[i + 1] = funnel_r(whi, lo[it], 32u - 8u * i);
            }
        } else {
            if (i < 3) qw[i] = (lo[it] >> (8u * i)) | (nlo << (24u - 8u * i));
        }
        uint32_t r = (tau4[it] << (4u * i)) | (se[it] << (16u + 8u * (i >> 1)));
        r |= dpp<kQuadXor1>(r);
        r |= dpp<kQuadXor2>(r);
        if ((i & 1u) == 0)
            *reinterpret_cast<uint16_t *>(sp + W::kCodeBytes + (i == 0 ? 0 : W::kExpBytes) + 2 * quad) =
                i == 0 ? (uint16_t)(r >> 16) : (uint16_t)(r & 0xffffu);
    }
    // LDS operations of one wave complete in order; keep the compiler from moving them
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const u32x4 *sc = reinterpret_cast<const u32x4 *>(sp);
    if constexpr (CB != 8) {
        u32x4 *gc = reinterpret_cast<u32x4 *>(codes + gw * CB);
#pragma unroll
        for (int k = 0; k < (W::kCodeBytes / 16 + 63) / 64; ++k)
            if (64 * k + lane < W::kCodeBytes / 16) stg<kNtPlanes>(sc[64 * k + lane], gc + 64 * k + lane);
    }
    constexpr int kEC = W::kExpBytes / 16;  // chunks per exponent plane
    if (lane < 2 * kEC) {
        uint8_t *dst = (lane < kEC ? sexp : mexp) + gw / 2;
        *(reinterpret_cast<u32x4 *>(dst) + (lane % kEC)) = sc[W::kCodeBytes / 16 + lane];
    }
}

template <int MB, typename T>
__global__ __launch_bounds__(kQThreads) void mx_quantize_row_kernel(
    const T *__restrict__ x, uint8_t *__restrict__ codes, uint8_t *__restrict__ sexp,
    uint8_t *__restrict__ mexp, int64_t n_groups)
{
    constexpr bool kStage = sizeof(T) == 4;  // FP32 rows arrive through LDS
    __shared__ float s_stage[kStage ? kQThreads / 64 : 1][kStage ? kWaveStage : 1];
    constexpr int kIter = q_iter<T>();
    uint32_t xb[kIter][8];
    // Every workgroup but the last is whole: no bounds checks, no lane masks, and nothing for the
    // compiler to initialise on the paths a check would skip (1.8 of the 15 vector instructions per
    // BF16 element of the checked form).  A wave then takes kIter x 64 consecutive groups.
    if ((int64_t)(blockIdx.x + 1) * (kQThreads * kIter) <= n_groups) {
        typedef WavePlanes<MB, kIter> W;
        __shared__ __attribute__((aligned(16))) uint8_t s_planes[kQThreads / 64][W::kBytes];
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const int64_t gw = (int64_t)blockIdx.x * (kQThreads * kIter) + wave * W::kGroups;  // the wave's first group
#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            if constexpr (kStage)
                wave_load512(reinterpret_cast<const float *>(x) + 8 * (gw + it * 64), xb[it], 512, s_stage[wave]);
            else
                load8(x + 8 * (gw + it * 64 + lane), xb[it]);
        }
        uint32_t lo[kIter], hi[kIter], se[kIter], tau4[kIter];
#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            uint32_t yb[8];
            mx_quant8<MB, false>(xb[it], lo[it], hi[it], se[it], tau4[it], yb);
        }
        wave_store_planes<MB, kIter>(lo, hi, se, tau4, gw, s_planes[wave], codes, sexp, mexp);
        return;
    }
    // The last workgroup: a thread takes kIter groups, kQThreads apart; whole quads of lanes are in
    // or out of range together (n_groups % 4 == 0).
    const int64_t g0 = (int64_t)blockIdx.x * (kQThreads * kIter) + threadIdx.x;
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
        const int64_t g = g0 + it * kQThreads;
        if constexpr (kStage) {
            const int64_t wave_g = g - (threadIdx.x & 63);
            wave_load512(reinterpret_cast<const float *>(x) + 8 * wave_g, xb[it],
                         8 * (n_groups - wave_g), s_stage[threadIdx.x >> 6]);
        } else {
            if (g < n_groups) load8(x + 8 * g, xb[it]);
        }
    }
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
        const int64_t g = g0 + it * kQThreads;
        if (g < n_groups) {
            uint32_t yb[8], lo, hi, se, tau4;
            mx_quant8<MB, false>(xb[it], lo, hi, se, tau4, yb);
            mx_store_group<MB>(lo, hi, se, tau4, g, codes, sexp, mexp);
        }
    }
}

// Dequantize, 8 elements per lane and deq_iter() such groups per lane.  All loads of
// a lane are issued before the first result is needed: a wave cannot write before
// its codes have arrived, so the bytes it has in flight, not its instruction
// count, set the rate when reads queue behind the kernel's own write stream.
constexpr int kDeqThreads = 256;  // workgroup size of the dequantize kernel
// Groups per lane.  Measured in the loop of the three formats at 1 GiB FP32 (workgroup size x
// groups per lane -> MX9 / MX6 / MX4 in microseconds): 128 x 1: 225 / 233 / 245, 128 x 2: 235 /
// 219 / 221, 256 x 1: 213 / 220 / 229, 256 x 2: 236 / 213 / 214, 512 x 1: 214 / 225 / 223,
// 256 x 4: 239 / 234 / 239, 64 x 1: 233 / 260 / 259, 64 x 2: 240 / 240 / 237, 64 x 4: 246 / 249 /
// 255, 128 x 4: 236 / 237 / 239, 512 x 2: 231 / 217 / 221, 1024 x 1: 225 / 250 / 230.  A pure
// store stream is fastest from workgroups that write 4 KiB each, however many stores a lane
// makes (per GiB: 160 us from 256 threads x one 16-byte store, 164 from 128 x two, 169 from
// 64 x four; 8 KiB: 167 from 512 x one, 183 from 256 x two; 16 KiB: 188; 2 KiB: 180 - 187;
// 1 KiB: 224), but a dequantize is not a pure store stream: its 4 KiB shapes (128 x 1, 64 x
// 2) lose more on the loads than they gain, and the 3- and 5-byte code loads of MX4 and MX6
// want two groups per lane in flight where MX9 (8-byte loads) does not.  (A variant with four elements and one 16-byte store per lane, which needs no
// staging at all, took 253 / 243 / 252: too few bytes of codes in flight per wave.  BF16
// rows, 8192 x 12288: two groups per lane 55 / 43 / 39, one 62 / 44 / 42.)
template <int MB, typename T>
constexpr int deq_iter()
{
    return MB == 7 && sizeof(T) == 4 ? 1 : 2;
}
// A gather takes one group per lane: its loads are scattered rows, not a stream, and more of them
// per lane gain nothing (2^27 FP32 values from an MX6 / MX9 / MX4 table image of 128-wide rows: one
// group 106 / 116 / 92 us, two 108 / 118 / 98, four 109 / 119 / 99).
template <int MB, typename T>
constexpr int gather_iter() { return 1; }
template <int MB, typename T>
static inline dim3 gather_grid(int64_t n_groups)
{
    constexpr int64_t per = (int64_t)kDeqThreads * gather_iter<MB, T>();
    return dim3((unsigned)((n_groups + per - 1) / per));
}
template <int MB, typename T>
static inline dim3 deq_grid(int64_t n_groups)
{
    constexpr int64_t per = (int64_t)kDeqThreads * deq_iter<MB, T>();
    return dim3((unsigned)((n_groups + per - 1) / per));
}

// GATHER: the output is [n_idx x cols] and output row j is row idx[j] of the packed
// table (a storage format for embedding tables, Sec. V "Inferencing" / recommendation
// models): a group of the output maps to a group of the table through one index
// load.  An index outside [0, table_rows) gives a row of +0.
struct GatherArgs {
    const int64_t *idx;
    int64_t table_rows;
    int32_t groups_per_row;  // cols / 8, a multiple of 4
    int32_t fixed_se;        // FIXED_SE: the exponent code every block is given
    // ROWS_TOGETHER: the table keeps each row's three runs next to each other (`codes` is the
    // table): row_bytes per row, the exponent bytes codes_row bytes into it, the
    // microexponent bytes sexp_row bytes after those
    int32_t row_bytes, codes_row, sexp_row;
};
// FIXED_SE: the exponent plane is not read; every block takes the exponent code
// ga.fixed_se instead, which turns the elements into the scaled integers
// M 2^(fixed_se - 127 - (MB - 1) - tau) (used by the dot-product pipeline model).
//
// LK1, LK2, D2: log2 k1 (3 .. 6), log2 k2 (<= LK1) and d2 (0 or 1) of the format; Table II's
// own (4, 1, 1) by default.  Only where the lane finds its exponent byte and its microexponent
// bits depends on them: the codes of 8 elements are MB + 1 bytes whatever the block sizes.
template <int MB, typename T, bool GATHER = false, bool FIXED_SE = false, int LK1 = 4, int LK2 = 1,
          int D2 = 1, bool ROWS_TOGETHER = false>
__global__ __launch_bounds__(kDeqThreads) void mx_dequantize_row_kernel(
    const uint8_t *__restrict__ codes, const uint8_t *__restrict__ sexp,
    const uint8_t *__restrict__ mexp, T *__restrict__ y, int64_t n_groups, GatherArgs ga)
{
    constexpr int CB = MB + 1;
    constexpr uint32_t CMASK = (1u << CB) - 1u;
    constexpr uint32_t MMASK = (1u << MB) - 1u;
    constexpr bool kStage = sizeof(T) == 4;  // FP32 rows leave through LDS, see wave_store512
    __shared__ float s_stage[kStage ? kDeqThreads / 64 : 1][kStage ? kWaveStage : 1];
    constexpr int kStep = kDeqThreads;  // distance between a lane's groups
    constexpr int kDeqIter = GATHER ? gather_iter<MB, T>() : deq_iter<MB, T>();
    const int64_t g0 = (int64_t)blockIdx.x * (kDeqThreads * kDeqIter) + threadIdx.x;
    const uint32_t i = threadIdx.x & 3u;

    uint32_t v0[kDeqIter], v1[kDeqIter], seb[kDeqIter], tbb[kDeqIter];
#pragma unroll
    for (int it = 0; it < kDeqIter; ++it) {
        const int64_t go = g0 + it * kStep;  // group of the output
        v0[it] = v1[it] = seb[it] = tbb[it] = 0;
        bool live = go < n_groups;  // whole quads are live or not (n_groups % 4 == 0)
        int64_t g = go;             // group of the packed image it comes from
        const uint8_t *cp = codes, *sp = sexp, *mp = mexp;
        if (GATHER && live) {
            const int64_t j = go / ga.groups_per_row;
            const int64_t r = ga.idx[j];
            live = r >= 0 && r < ga.table_rows;
            g = go - j * ga.groups_per_row;
            if (ROWS_TOGETHER) {
                cp = codes + r * ga.row_bytes;  // the row's own runs; g counts inside the row
                sp = cp + ga.codes_row;
                mp = sp + ga.sexp_row;
            } else {
                g += r * ga.groups_per_row;
            }
        }
        if (live) {
            const int64_t quad = g >> 2;
            if (CB == 8) {
                u32x2 v = ldg<!GATHER>(reinterpret_cast<const u32x2 *>(cp + 8 * g));
                v0[it] = v.x;
                v1[it] = v.y;
            } else if (CB == 5) {
                // aligned dword loads only: lane i takes dword i of the quad's five, the
                // fifth is fetched by all four lanes and used by lane 3
                const uint32_t *cw = reinterpret_cast<const uint32_t *>(cp) + 5 * quad;
                v0[it] = cw[i];
                v1[it] = cw[4];
            } else {
                // lane i takes dword min(i, 2) of the quad's three
                const uint32_t *cw = reinterpret_cast<const uint32_t *>(cp) + 3 * quad;
                v0[it] = cw[i < 2 ? i : 2];
            }
            seb[it] = FIXED_SE ? (uint32_t)ga.fixed_se : sp[g >> (LK1 - 3)];
            // the byte that holds the lane's microexponent bits: 8 >> LK2 of them from bit
            // g (8 >> LK2) of the stream when k2 <= 8, else the one bit of sub-block
            // g / (k2 / 8); byte g >> LK2 either way
            if (D2) tbb[it] = mp[g >> LK2];
        }
    }
#pragma unroll
    for (int it = 0; it < kDeqIter; ++it) {
        const int64_t g = g0 + it * kStep;
        uint32_t lo, hi = 0;
        if (CB == 8) {
            lo = v0[it];
            hi = v1[it];
        } else if (CB == 5) {
            // lane i's 40 bits start 8 i bits into dword i of the quad's 5 dwords; the
            // following dword comes from the next lane (lane 3: the fifth dword)
            const uint32_t nx = dpp<kQuadNext>(v0[it]);
            const uint32_t up = i == 3 ? v1[it] : nx;
            lo = funnel_r(up, v0[it], 8u * i);
            hi = (up >> (8u * i)) & 0xffu;
        } else {
            // lane i's 24 bits start at bit 24 i of the quad's 3 dwords: the end of the
            // previous lane's dword and the start of its own (lane 3: all in dword 2)
            const uint32_t pv = dpp<kQuadPrev>(v0[it]);
            lo = funnel_r(v0[it], pv, 24u * i) & 0xffffffu;
        }
        const uint32_t se = seb[it];
        // the lane's bits moved down to bit 0 (one bit per sub-block; a single bit when the
        // sub-block is as long as the lane's run or longer)
        const uint32_t tau4 =
            LK2 <= 3 ? tbb[it] >> ((uint32_t)(g & ((1 << LK2) - 1)) * (8u >> LK2))
                     : (tbb[it] >> ((uint32_t)(g >> (LK2 - 3)) & 7u)) & 1u;
        uint32_t yb[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int off = e * CB;
            uint32_t c;
            if (off >= 32)
                c = hi >> (off - 32);
            else if (off + CB > 32)
                c = (lo >> off) | (hi << (32 - off));
            else
                c = lo >> off;
            c &= CMASK;
            const int t = D2 ? (int)((tau4 >> (LK2 <= 3 ? e >> LK2 : 0)) & 1u) : 0;
            const int q = (int)se - 127 - t - (MB - 1);
            const float v = __builtin_ldexpf((float)(c & MMASK), q);
            yb[e] = as_u(v) | ((c >> MB) << 31);
        }
        if constexpr (kStage) {
            const int64_t wave_g = g - (threadIdx.x & 63);  // first group of this wave
            wave_store512(reinterpret_cast<float *>(y) + 8 * wave_g, yb, 8 * (n_groups - wave_g),
                          s_stage[threadIdx.x >> 6]);
        } else {
            if (g < n_groups) store8(y + 8 * g, yb);
        }
    }
}

template <int MB, typename T>
__global__ __launch_bounds__(kThreads) void mx_qdq_row_kernel(const T *x, T *y, int64_t n_groups)
{
    // no __restrict__: y may be x (each lane reads its 8 elements before it writes them)
    const int64_t g = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (g >= n_groups) return;  // whole blocks leave together (n_groups % 2 == 0)
    uint32_t xb[8], yb[8];
    load8(x + 8 * g, xb);
    uint32_t lo, hi, se, tau4;
    mx_quant8<MB, true>(xb, lo, hi, se, tau4, yb);
    store8(y + 8 * g, yb);
}

// ------------------------------------------------- FP32 kernels, 4 elements per lane
//
// For FP32 a lane that owns 4 consecutive elements makes every 16-byte access of
// a wave contiguous (64 x 16 bytes), which is what the memory system likes best.
// A block is then a quad of lanes and its maximum takes two DPP quad permutes.

template <int MB, bool DEQ>
__device__ __forceinline__ void mx_quant4(const uint32_t (&xb)[4], uint32_t &codes, uint32_t &se,
                                          uint32_t &tau2, uint32_t (&yb)[4])
{
    uint32_t w[1];
    mx_quant_lane<MB, 2, 2, DEQ>(xb, w, se, tau2, yb);
    codes = w[0];
}

template <int MB>
__global__ __launch_bounds__(kThreads) void mx_qdq_row_f32x4_kernel(const float *x, float *y,
                                                                    int64_t n4)
{
    const int64_t g = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (g >= n4) return;  // whole quads leave together (n4 % 4 == 0)
    const u32x4 v = ldg<true>(reinterpret_cast<const u32x4 *>(x) + g);
    const uint32_t xb[4] = {v.x, v.y, v.z, v.w};
    uint32_t yb[4], codes, se, tau2;
    mx_quant4<MB, true>(xb, codes, se, tau2, yb);
    const u32x4 o = {yb[0], yb[1], yb[2], yb[3]};
    stg<true>(o, reinterpret_cast<u32x4 *>(y) + g);
}

// ------------------------------------------------------------- generic kernels
//
// These see the tensor as a logical [R x C] array with blocks along C, element
// (r, c) at r * sr + c * sc.  Row blocks: sr = ld, sc = 1 (vector loads).  Column
// blocks: the transposed view, sr = 1, sc = ld (STRIDED: one element at a time;
// this is the slow general path, the tiled kernels in bdr_colwise.hip are the
// fast one).

__device__ __forceinline__ uint32_t load1(const float *p) { return as_u(*p); }
__device__ __forceinline__ uint32_t load1(const uint16_t *p) { return (uint32_t)*p << 16; }
__device__ __forceinline__ void store1(float *p, uint32_t b) { *p = as_f(b); }
__device__ __forceinline__ void store1(uint16_t *p, uint32_t b) { *p = (uint16_t)(b >> 16); }


// Sub-block and block maxima (exponent-clamped magnitudes) for the 8 elements
// of a lane; the block or sub-block may be smaller than the lane's run, or span
// up to 32 lanes.
__device__ __forceinline__ void gen_maxima(const GenFmt &f, const uint32_t (&xb)[8],
                                           uint32_t (&pe)[8], uint32_t (&be)[8])
{
#pragma unroll
    for (int i = 0; i < 8; ++i) pe[i] = clamp_mag(xb[i] & kAbsMask);
#pragma unroll
    for (int w = 1; w < 8; w <<= 1) {
        if (f.k2 > w) {
            uint32_t t[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) t[i] = umax(pe[i], pe[i ^ w]);
#pragma unroll
            for (int i = 0; i < 8; ++i) pe[i] = t[i];
        }
    }
    if (f.k2 > 8) {
        uint32_t v = pe[0];
        for (int w = 1; w < f.k2 / 8; w <<= 1) v = umax(v, (uint32_t)__shfl_xor((int)v, w));
#pragma unroll
        for (int i = 0; i < 8; ++i) pe[i] = v;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) be[i] = pe[i];
#pragma unroll
    for (int w = 1; w < 8; w <<= 1) {
        if (f.k1 > w) {
            uint32_t t[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) t[i] = umax(be[i], be[i ^ w]);
#pragma unroll
            for (int i = 0; i < 8; ++i) be[i] = t[i];
        }
    }
    if (f.k1 > 8) {
        uint32_t v = be[0];
        for (int w = 1; w < f.k1 / 8; w <<= 1) v = umax(v, (uint32_t)__shfl_xor((int)v, w));
#pragma unroll
        for (int i = 0; i < 8; ++i) be[i] = v;
    }
}

// The lane's 8 codes of CB bits each as CB bytes at cp (LDS), little-endian bit stream.
template <int CB>
__device__ __forceinline__ void pack_codes(const uint32_t (&code)[8], uint8_t *cp)
{
    uint32_t w[3] = {0, 0, 0};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int off = i * CB;
        w[off >> 5] |= code[i] << (off & 31);
        if ((off & 31) + CB > 32) w[(off >> 5) + 1] |= code[i] >> (32 - (off & 31));
    }
#pragma unroll
    for (int b = 0; b < CB; ++b) cp[b] = (uint8_t)(w[b >> 2] >> (8 * (b & 3)));
}

// MODE 0: write the packed planes.  MODE 1: write the dequantized tensor.
// CONTIG (FP32, pitch = row length): the tensor side moves as contiguous 1 KiB
// wave rows through LDS like in the MX kernels.  The planes of a workgroup's 2048
// elements are contiguous runs of the three planes; they are assembled in LDS and
// leave as coalesced stores by consecutive lanes.
template <typename T, int MODE, bool STRIDED, bool CONTIG, int SPEC = -1>
__global__ __launch_bounds__(kThreads) void generic_quantize_kernel(
    GenFmt f_arg, const T *x, T *y, uint8_t *__restrict__ codes,
    uint8_t *__restrict__ sexp, uint8_t *__restrict__ mexp, int64_t cols, int64_t sr, int64_t sc,
    int64_t n_groups, int64_t valid)
{
    static_assert(!CONTIG || (sizeof(T) == 4 && !STRIDED), "contiguous staging is for FP32 rows");
    const GenFmt f = SPEC >= 0 ? hot_format(SPEC >= 0 ? SPEC : 0) : f_arg;
    __shared__ uint32_t s_mexp[MODE == 0 ? kTileElems * 3 / 32 + 1 : 1];
    __shared__ uint32_t s_codes[MODE == 0 ? kThreads * 9 / 4 : 1];  // up to 9 bytes per lane
    __shared__ uint32_t s_sexp[MODE == 0 ? kTileElems / 4 : 1];     // up to one byte per element
    __shared__ float s_stage[CONTIG ? kThreads / 64 : 1][CONTIG ? kWaveStage : 1];
    const int64_t g = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const bool active = g < n_groups;
    uint32_t xb[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int64_t addr = 0, c0 = 0;
    const int64_t wave_g = g - (threadIdx.x & 63);  // first group of this wave
    const bool mexp_atomics = MODE == 0 && f.d2 > 0 && !(SPEC >= 0 && f.d2 == 1);
    if (mexp_atomics)  // cleared while the loads below are in flight
        for (int t = threadIdx.x; t < kTileElems * 3 / 32 + 1; t += kThreads) s_mexp[t] = 0;
    if (CONTIG) {
        wave_load512(reinterpret_cast<const float *>(x) + 8 * wave_g, xb, 8 * (n_groups - wave_g),
                     s_stage[threadIdx.x >> 6]);
    } else if (active) {
        const int64_t t0 = 8 * g;
        const int64_t r = t0 / cols;
        c0 = t0 - r * cols;
        addr = r * sr + c0 * sc;
        if (STRIDED) {
            // elements past the end of a row whose last block is short read as +0
#pragma unroll
            for (int i = 0; i < 8; ++i) xb[i] = c0 + i < valid ? load1(x + addr + i * sc) : 0u;
        } else {
            load8(x + addr, xb);
        }
    }
    if (mexp_atomics) __syncthreads();
    uint32_t pe[8], be[8];
    gen_maxima(f, xb, pe, be);

    const int beta = (1 << f.d2) - 1;
    const int cb = f.m + 1;
    const float top = (float)((1u << f.m) - 1u);
    uint32_t code[8], tau[8], yb[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int se = (int)(be[i] >> 23);
        int t = se - (int)(pe[i] >> 23);
        t = t < beta ? t : beta;
        tau[i] = (uint32_t)t;
        const int sh = (f.m - 1) + 127 - se + t;
        const float mf = gen_round(__builtin_fabsf(as_f(xb[i])), sh, top, f.rounding);
        code[i] = (uint32_t)mf | ((xb[i] >> 31) << f.m);
        if (MODE == 1) yb[i] = as_u(__builtin_ldexpf(mf, -sh)) | (xb[i] & 0x80000000u);
    }
    if (MODE == 1) {
        if (CONTIG) {
            wave_store512(reinterpret_cast<float *>(y) + 8 * wave_g, yb, 8 * (n_groups - wave_g),
                          s_stage[threadIdx.x >> 6]);
        } else if (active) {
            if (STRIDED) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (c0 + i < valid) store1(y + addr + i * sc, yb[i]);
            } else {
                store8(y + addr, yb);
            }
        }
        return;
    }

    // ---- planes of this workgroup, assembled in LDS
    const int64_t block_g0 = (int64_t)blockIdx.x * kThreads;
    const int n_active = (int)(n_groups - block_g0 < kThreads ? n_groups - block_g0 : kThreads);
    uint8_t *lc = reinterpret_cast<uint8_t *>(s_codes);
    uint8_t *ls = reinterpret_cast<uint8_t *>(s_sexp);
    const int lk1 = __builtin_ctz(f.k1);
    // Compiled-for-the-tuple kernels with 5- or 3-bit codes store them straight from
    // registers, a quad of lanes at a time (the launcher sends only tensors made of whole
    // quads here); everything else assembles the workgroup's codes in LDS first.
    constexpr bool kDirectCodes = SPEC >= 0 && (hot_format(SPEC >= 0 ? SPEC : 0).m == 4 ||
                                                hot_format(SPEC >= 0 ? SPEC : 0).m == 2);
    if (active) {
        if constexpr (kDirectCodes) {
            constexpr int CBK = hot_format(SPEC >= 0 ? SPEC : 0).m + 1;
            uint32_t w[2] = {0, 0};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int off = i * CBK;
                w[off >> 5] |= code[i] << (off & 31);
                if ((off & 31) + CBK > 32) w[(off >> 5) + 1] |= code[i] >> (32 - (off & 31));
            }
            store_codes_quad<CBK>(w[0], w[1], g, codes);
        } else {
        // 8 codes of cb <= 9 bits: cb bytes; the code width is dispatched once so that
        // all shifts are immediate
        uint8_t *cp = lc + cb * threadIdx.x;
        switch (cb) {
        case 2: pack_codes<2>(code, cp); break;
        case 3: pack_codes<3>(code, cp); break;
        case 4: pack_codes<4>(code, cp); break;
        case 5: pack_codes<5>(code, cp); break;
        case 6: pack_codes<6>(code, cp); break;
        case 7: pack_codes<7>(code, cp); break;
        case 8: pack_codes<8>(code, cp); break;
        default: pack_codes<9>(code, cp); break;
        }
        }

        if (f.k1 >= 8) {
            const int lanes = f.k1 / 8;
            if ((threadIdx.x & (lanes - 1)) == 0) ls[threadIdx.x / lanes] = (uint8_t)(be[0] >> 23);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if ((i & (f.k1 - 1)) == 0)
                    ls[((8 * threadIdx.x) >> lk1) + (i >> lk1)] = (uint8_t)(be[i] >> 23);
        }
    }
    // Microexponents.  A tile's stream starts on a byte boundary because kTileElems / k2 is a
    // multiple of 8.
    const int64_t tile_sub0 = (int64_t)blockIdx.x * (kTileElems / f.k2);
    if (SPEC >= 0 && f.d2 == 1) {
        // One bit per sub-block: a byte of the stream is the 8 sub-blocks = 8 k2 elements = k2
        // lanes (k2 a power of two <= 64), so the byte is OR-ed together across those lanes in
        // registers and its first lane stores it: every byte has one writer, no atomics, and
        // nothing to clear.  Lanes past the end of the tensor hold zeros (their byte is not
        // written out below).
        uint32_t field = 0;
        if (f.k2 <= 8) {
            const int nb = 8 / f.k2;  // bits this lane owns
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if ((i & (f.k2 - 1)) == 0) field |= (tau[i] & 1u) << (i / f.k2);
            field <<= (threadIdx.x & (f.k2 - 1)) * nb;
        } else {
            const int lanes = f.k2 / 8;  // lanes per sub-block; its first lane carries the bit
            if ((threadIdx.x & (lanes - 1)) == 0) field = (tau[0] & 1u) << ((threadIdx.x & (f.k2 - 1)) / lanes);
        }
        if (f.k2 >= 2) field |= dpp<kQuadXor1>(field);
        if (f.k2 >= 4) field |= dpp<kQuadXor2>(field);
        if (f.k2 >= 8) field |= dpp<kRowHalfMirror>(field);
        if (f.k2 >= 16) field |= dpp<kRowMirror>(field);
        if (f.k2 >= 32) field |= (uint32_t)__shfl_xor((int)field, 16);
        if (f.k2 >= 64) field |= (uint32_t)__shfl_xor((int)field, 32);
        if ((threadIdx.x & (f.k2 - 1)) == 0)
            reinterpret_cast<uint8_t *>(s_mexp)[threadIdx.x / f.k2] = (uint8_t)field;
    } else if (active && f.d2 > 0) {
        // run-time tuple: each lane ORs its bits into the tile's bit stream
        uint32_t field = 0;
        int width = 0;
        int64_t u0;
        if (f.k2 <= 8) {
            const int lk2 = __builtin_ctz(f.k2);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if ((i & (f.k2 - 1)) == 0) field |= tau[i] << ((i >> lk2) * f.d2);
            width = (8 >> lk2) * f.d2;
            u0 = (8 * g) >> lk2;
        } else {
            const int lanes = f.k2 / 8;
            if ((g & (lanes - 1)) == 0) {
                field = tau[0];
                width = f.d2;
            }
            u0 = g / lanes;
        }
        if (width > 0) {
            const uint32_t bit = (uint32_t)((u0 - tile_sub0) * f.d2);
            const uint32_t sft = bit & 31u;
            atomicOr(&s_mexp[bit >> 5], field << sft);
            if (sft + (uint32_t)width > 32u) atomicOr(&s_mexp[(bit >> 5) + 1], field >> (32u - sft));
        }
    }
    __syncthreads();
    // ---- flush: consecutive lanes write consecutive dwords (bytes at the ragged end)
    if constexpr (!kDirectCodes) {
        const int nbytes = cb * n_active;  // the workgroup's codes start at byte cb * 256 * blockIdx
        uint8_t *gp = codes + (int64_t)cb * block_g0;
        uint32_t *gw = reinterpret_cast<uint32_t *>(gp);
        for (int t = threadIdx.x; t < nbytes / 4; t += kThreads) gw[t] = s_codes[t];
        for (int t = (nbytes & ~3) + threadIdx.x; t < nbytes; t += kThreads) gp[t] = lc[t];
    }
    {
        const int64_t e0 = 8 * block_g0;                  // first element of the workgroup
        const int nbytes = (int)((8 * (int64_t)n_active) >> lk1);  // whole blocks only (host-checked)
        uint8_t *gp = sexp + (e0 >> lk1);
        if (((e0 >> lk1) & 3) == 0) {
            uint32_t *gw = reinterpret_cast<uint32_t *>(gp);
            for (int t = threadIdx.x; t < nbytes / 4; t += kThreads) gw[t] = s_sexp[t];
            for (int t = (nbytes & ~3) + threadIdx.x; t < nbytes; t += kThreads) gp[t] = ls[t];
        } else {
            for (int t = threadIdx.x; t < nbytes; t += kThreads) gp[t] = ls[t];
        }
    }
    if (f.d2 == 0) return;
    const int64_t n_sub = n_groups * 8 / f.k2;
    int64_t tile_subs = n_sub - tile_sub0;
    if (tile_subs > kTileElems / f.k2) tile_subs = kTileElems / f.k2;
    const int nbytes = (int)((tile_subs * f.d2 + 7) / 8);
    uint8_t *mp = mexp + tile_sub0 * f.d2 / 8;
    for (int b = threadIdx.x; b < nbytes; b += kThreads)
        mp[b] = (uint8_t)(s_mexp[b >> 2] >> (8 * (b & 3)));
}

template <typename T, bool STRIDED, bool CONTIG>
__global__ __launch_bounds__(kThreads) void generic_dequantize_kernel(
    GenFmt f, const uint8_t *__restrict__ codes, const uint8_t *__restrict__ sexp,
    const uint8_t *__restrict__ mexp, int64_t mexp_bytes, T *__restrict__ y, int64_t cols,
    int64_t sr, int64_t sc, int64_t n_groups, int64_t valid)
{
    static_assert(!CONTIG || (sizeof(T) == 4 && !STRIDED), "contiguous staging is for FP32 rows");
    __shared__ float s_stage[CONTIG ? kThreads / 64 : 1][CONTIG ? kWaveStage : 1];
    const int64_t g = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const bool active = g < n_groups;
    if (!CONTIG && !active) return;
    const int cb = f.m + 1;
    const uint32_t cmask = (1u << cb) - 1u, mmask = (1u << f.m) - 1u;
    const uint32_t beta = (1u << f.d2) - 1u;
    const int lk1 = __builtin_ctz(f.k1), lk2 = __builtin_ctz(f.k2);

    uint32_t yb[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (active) {
        // the lane's cb bytes sit inside three aligned dwords; at the very end of the
        // plane, where a dword would reach past it, they are fetched one by one
        const int64_t base = (int64_t)cb * g, a0 = base & ~(int64_t)3, total = (int64_t)cb * n_groups;
        uint64_t w = 0;
        uint32_t extra = 0;
        if (a0 + 12 <= total) {
            const uint32_t *dp = reinterpret_cast<const uint32_t *>(codes + a0);
            const uint32_t d0 = dp[0], d1 = dp[1], d2w = dp[2];
            const uint32_t sft = 8u * (uint32_t)(base - a0);
            w = (uint64_t)funnel_r(d1, d0, sft) | ((uint64_t)funnel_r(d2w, d1, sft) << 32);
            extra = (d2w >> sft) & 0xffu;
        } else {
            const uint8_t *cp = codes + base;
            for (int b = 0; b < cb; ++b) {
                if (b < 8)
                    w |= (uint64_t)cp[b] << (8 * b);
                else
                    extra = cp[b];
            }
        }
        // shared exponents: one per lane when the block spans the lane's 8 elements
        int se[8];
        if (lk1 >= 3) {
            const int v = sexp[(8 * g) >> lk1];
#pragma unroll
            for (int i = 0; i < 8; ++i) se[i] = v;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) se[i] = sexp[((8 * g) >> lk1) + (i >> lk1)];
        }
        // microexponents: the lane's fields are at most 24 consecutive bits of the stream
        uint32_t tau[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (f.d2 > 0) {
            const int64_t bit0 = ((8 * g) >> lk2) * f.d2;
            const int64_t byte0 = bit0 >> 3;
            const int nsub = lk2 >= 3 ? 1 : 8 >> lk2;
            const int last = (int)(((bit0 & 7) + nsub * f.d2 - 1) >> 3);  // index of the last byte needed
            uint32_t v = 0;
            for (int b = 0; b <= last; ++b)
                if (byte0 + b < mexp_bytes) v |= (uint32_t)mexp[byte0 + b] << (8 * b);
            v >>= (bit0 & 7);
#pragma unroll
            for (int i = 0; i < 8; ++i) tau[i] = (v >> ((lk2 >= 3 ? 0 : i >> lk2) * f.d2)) & beta;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t c = (uint32_t)(w >> (i * cb));
            if (i == 7 && cb == 9) c |= extra << 1;
            c &= cmask;
            const int q = se[i] - 127 - (int)tau[i] - (f.m - 1);
            yb[i] = as_u(__builtin_ldexpf((float)(c & mmask), q)) | ((c >> f.m) << 31);
        }
    }
    if (CONTIG) {
        const int64_t wave_g = g - (threadIdx.x & 63);
        wave_store512(reinterpret_cast<float *>(y) + 8 * wave_g, yb, 8 * (n_groups - wave_g),
                      s_stage[threadIdx.x >> 6]);
        return;
    }
    const int64_t t0 = 8 * g;
    const int64_t r = t0 / cols;
    const int64_t c0 = t0 - r * cols;
    const int64_t addr = r * sr + c0 * sc;
    if (STRIDED) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (c0 + i < valid) store1(y + addr + i * sc, yb[i]);  // pads of a short last block are not part of y
    } else {
        store8(y + addr, yb);
    }
}

// -------------------------------------------------------------------- launchers

static inline unsigned blocks_for(int64_t n_groups)
{
    return (unsigned)((n_groups + kThreads - 1) / kThreads);
}

static inline GenFmt gen_of(const bdr_format &f)
{
    GenFmt g = {f.k1, f.k2, f.d2, f.m, f.rounding};
    return g;
}

// The fast kernels see the tensor as one flat run of whole quads of lanes.
// decode: reading an image does not depend on how it was rounded
static inline bool mx_fast_ok(const bdr_format &f, int64_t rows, int64_t cols, int64_t ld,
                              bool decode = false)
{
    return (decode ? is_mx_layout(f) : is_mx(f)) && ld == cols && (rows * cols) % 32 == 0;
}

// Launch the quantize kernel compiled for table entry `spec` (FP32 rows with pitch = row
// length, whole quads of lanes).  The fused round trip has no such kernels: it is bound by
// its 2 x 4 bytes per element with the tuple at run time already.
template <typename T, int SP = 0>
static void launch_hot(int spec, dim3 grid, hipStream_t s, const T *x, uint8_t *codes,
                       uint8_t *sexp, uint8_t *mexp, int64_t cols, int64_t ng)
{
    if constexpr (SP < kHotCount) {
        if (spec != SP) return launch_hot<T, SP + 1>(spec, grid, s, x, codes, sexp, mexp, cols, ng);
        // FP32 rows move as contiguous wave rows through LDS; a BF16 lane's 8 elements are one 16-byte load
        hipLaunchKernelGGL((generic_quantize_kernel<T, 0, false, sizeof(T) == 4, SP>), grid, dim3(kThreads), 0, s,
                           hot_format(SP), x, (T *)nullptr, codes, sexp, mexp, cols, cols, (int64_t)1, ng, cols);
    }
}

// Dequantize kernel for table entry `spec`: the Table II kernel with the tuple's block sizes
// (pitch = row length, whole quads of lanes).  Reading an image does not depend on the
// rounding rule, so the table's nearest-even entries serve every rounding.
template <typename T, int SP = 0>
static void launch_hot_dequantize(int spec, hipStream_t s, const uint8_t *codes,
                                  const uint8_t *sexp, const uint8_t *mexp, T *y, int64_t ng)
{
    if constexpr (SP < kHotCount) {
        if (spec != SP) return launch_hot_dequantize<T, SP + 1>(spec, s, codes, sexp, mexp, y, ng);
        constexpr GenFmt f = hot_format(SP);
        constexpr int lk1 = f.k1 == 8 ? 3 : f.k1 == 16 ? 4 : f.k1 == 32 ? 5 : 6;
        constexpr int lk2 = f.k2 == 1 ? 0 : f.k2 == 2 ? 1 : f.k2 == 4 ? 2 : lk1;
        hipLaunchKernelGGL((mx_dequantize_row_kernel<f.m, T, false, false, lk1, lk2, f.d2>),
                           (deq_grid<f.m, T>(ng)), dim3(kDeqThreads), 0, s, codes, sexp, mexp, y, ng, GatherArgs{});
    }
}

template <typename T, int SP = 0>
static void launch_hot_fused(int spec, dim3 grid, hipStream_t s, const T *x, T *y, int64_t cols, int64_t ng)
{
    if constexpr (SP < kHotCount) {
        if (spec != SP) return launch_hot_fused<T, SP + 1>(spec, grid, s, x, y, cols, ng);
        hipLaunchKernelGGL((generic_quantize_kernel<T, 1, false, false, SP>), grid, dim3(kThreads), 0, s,
                           hot_format(SP), x, y, (uint8_t *)nullptr, (uint8_t *)nullptr, (uint8_t *)nullptr, cols,
                           cols, (int64_t)1, ng, cols);
    }
}

// Rows the flat kernels cannot take: a short last block (or, for k1 < 8, a length that is not
// a multiple of 8).  They go through the element-at-a-time view.
static inline bool ragged(const bdr_format &f, int64_t n) { return n % (f.k1 > 8 ? f.k1 : 8) != 0; }

template <typename T>
static int generic_view_t(int what, const bdr_format &f, const T *x, T *y, int64_t R, int64_t n,
                          int64_t sr, int64_t sc, uint8_t *codes, uint8_t *sexp, uint8_t *mexp,
                          hipStream_t s);

template <typename T>
static int quantize_row_t(const bdr_format &f, const T *x, int64_t rows, int64_t cols, int64_t ld,
                          uint8_t *codes, uint8_t *sexp, uint8_t *mexp, hipStream_t s)
{
    if (ragged(f, cols)) return generic_view_t(0, f, x, (T *)nullptr, rows, cols, ld, (int64_t)1, codes, sexp, mexp, s);
    const int64_t ng = rows * cols / 8;
    const dim3 grid(blocks_for(ng)), block(kThreads);
    if (mx_fast_ok(f, rows, cols, ld)) {
        constexpr int kIter = q_iter<T>();
        const dim3 qgrid((unsigned)((ng + kQThreads * kIter - 1) / (kQThreads * kIter))), qblock(kQThreads);
        if (f.m == 7)
            hipLaunchKernelGGL((mx_quantize_row_kernel<7, T>), qgrid, qblock, 0, s, x, codes, sexp, mexp, ng);
        else if (f.m == 4)
            hipLaunchKernelGGL((mx_quantize_row_kernel<4, T>), qgrid, qblock, 0, s, x, codes, sexp, mexp, ng);
        else
            hipLaunchKernelGGL((mx_quantize_row_kernel<2, T>), qgrid, qblock, 0, s, x, codes, sexp, mexp, ng);
    } else {
        bool done = false;
        const int spec = ld == cols && ng % 4 == 0 ? hot_index(f) : -1;
        if (spec >= 0) {
            launch_hot<T>(spec, grid, s, x, codes, sexp, mexp, cols, ng);
            done = true;
        }
        if constexpr (sizeof(T) == 4) {
            if (!done && ld == cols) {
                hipLaunchKernelGGL((generic_quantize_kernel<T, 0, false, true>), grid, block, 0, s, gen_of(f),
                                   x, (T *)nullptr, codes, sexp, mexp, cols, ld, (int64_t)1, ng, cols);
                done = true;
            }
        }
        if (!done)
            hipLaunchKernelGGL((generic_quantize_kernel<T, 0, false, false>), grid, block, 0, s, gen_of(f),
                               x, (T *)nullptr, codes, sexp, mexp, cols, ld, (int64_t)1, ng, cols);
    }
    return launch_status();
}

int quantize_row(const bdr_format &f, const void *x, int dtype, int64_t rows, int64_t cols,
                 int64_t ld, void *codes, void *sexp, void *mexp, hipStream_t s)
{
    if (dtype == BDR_F32)
        return quantize_row_t(f, (const float *)x, rows, cols, ld, (uint8_t *)codes,
                              (uint8_t *)sexp, (uint8_t *)mexp, s);
    return quantize_row_t(f, (const uint16_t *)x, rows, cols, ld, (uint8_t *)codes,
                          (uint8_t *)sexp, (uint8_t *)mexp, s);
}

template <typename T>
static int dequantize_row_t(const bdr_format &f, const uint8_t *codes, const uint8_t *sexp,
                            const uint8_t *mexp, int64_t rows, int64_t cols, T *y, int64_t ld,
                            hipStream_t s)
{
    if (ragged(f, cols))
        return generic_view_t(1, f, (const T *)nullptr, y, rows, cols, ld, (int64_t)1, const_cast<uint8_t *>(codes),
                              const_cast<uint8_t *>(sexp), const_cast<uint8_t *>(mexp), s);
    const int64_t ng = rows * cols / 8;
    const dim3 grid(blocks_for(ng)), block(kThreads);
    if (mx_fast_ok(f, rows, cols, ld, true)) {
        if (f.m == 7)
            hipLaunchKernelGGL((mx_dequantize_row_kernel<7, T>), (deq_grid<7, T>(ng)), dim3(kDeqThreads), 0, s, codes, sexp, mexp, y, ng, GatherArgs{});
        else if (f.m == 4)
            hipLaunchKernelGGL((mx_dequantize_row_kernel<4, T>), (deq_grid<4, T>(ng)), dim3(kDeqThreads), 0, s, codes, sexp, mexp, y, ng, GatherArgs{});
        else
            hipLaunchKernelGGL((mx_dequantize_row_kernel<2, T>), (deq_grid<2, T>(ng)), dim3(kDeqThreads), 0, s, codes, sexp, mexp, y, ng, GatherArgs{});
    } else {
        const int64_t mexp_bytes = (rows * cols / f.k2 * f.d2 + 7) / 8;
        bool done = false;
        bdr_format fr = f;
        fr.rounding = BDR_RNE;
        const int spec = ld == cols && ng % 4 == 0 ? hot_index(fr) : -1;
        if (spec >= 0) {
            launch_hot_dequantize<T>(spec, s, codes, sexp, mexp, y, ng);
            done = true;
        }
        if constexpr (sizeof(T) == 4) {
            if (!done && ld == cols) {
                hipLaunchKernelGGL((generic_dequantize_kernel<T, false, true>), grid, block, 0, s, gen_of(f),
                                   codes, sexp, mexp, mexp_bytes, y, cols, ld, (int64_t)1, ng, cols);
                done = true;
            }
        }
        if (!done)
            hipLaunchKernelGGL((generic_dequantize_kernel<T, false, false>), grid, block, 0, s, gen_of(f),
                               codes, sexp, mexp, mexp_bytes, y, cols, ld, (int64_t)1, ng, cols);
    }
    return launch_status();
}

int dequantize_row(const bdr_format &f, const void *codes, const void *sexp, const void *mexp,
                   int64_t rows, int64_t cols, void *y, int dtype, int64_t ld, hipStream_t s)
{
    if (dtype == BDR_F32)
        return dequantize_row_t(f, (const uint8_t *)codes, (const uint8_t *)sexp,
                                (const uint8_t *)mexp, rows, cols, (float *)y, ld, s);
    return dequantize_row_t(f, (const uint8_t *)codes, (const uint8_t *)sexp,
                            (const uint8_t *)mexp, rows, cols, (uint16_t *)y, ld, s);
}

// BF16 image of a Table II operand with every block's exponent code replaced by se_code.
int dequantize_row_fixed_exponent(const bdr_format &f, const void *codes, const void *mexp, int64_t rows,
                                  int64_t cols, void *y, int se_code, hipStream_t s)
{
    const int64_t ng = rows * cols / 8;
    const uint8_t *c = (const uint8_t *)codes, *m = (const uint8_t *)mexp;
    uint16_t *out = (uint16_t *)y;
    GatherArgs ga{};
    ga.fixed_se = se_code;
    if (f.m == 7)
        hipLaunchKernelGGL((mx_dequantize_row_kernel<7, uint16_t, false, true>), (deq_grid<7, uint16_t>(ng)), dim3(kDeqThreads), 0, s, c, c, m, out, ng, ga);
    else if (f.m == 4)
        hipLaunchKernelGGL((mx_dequantize_row_kernel<4, uint16_t, false, true>), (deq_grid<4, uint16_t>(ng)), dim3(kDeqThreads), 0, s, c, c, m, out, ng, ga);
    else
        hipLaunchKernelGGL((mx_dequantize_row_kernel<2, uint16_t, false, true>), (deq_grid<2, uint16_t>(ng)), dim3(kDeqThreads), 0, s, c, c, m, out, ng, ga);
    return launch_status();
}

// ---- tables that keep a row's three runs together
//
// A lookup of a random row touches three places of the three-plane image (its codes, its
// exponent bytes, its microexponent bytes); each costs at least one memory line, which for
// rows of a few hundred elements is several times the bytes the row holds.  A table whose
// rows are [codes | exponent bytes | microexponent bytes], one after the other, is read as
// one run per lookup.  Same bytes, another order.
__global__ __launch_bounds__(kThreads) void table_pack_kernel(
    const uint32_t *__restrict__ codes, const uint32_t *__restrict__ sexp,
    const uint32_t *__restrict__ mexp, int64_t n_dwords, int32_t codes_dw, int32_t sexp_dw,
    int32_t mexp_dw, uint32_t *__restrict__ table)
{
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= n_dwords) return;
    const int32_t row_dw = codes_dw + sexp_dw + mexp_dw;
    const int64_t r = t / row_dw;
    const int32_t o = (int32_t)(t - r * row_dw);
    uint32_t v;
    if (o < codes_dw)
        v = codes[r * codes_dw + o];
    else if (o < codes_dw + sexp_dw)
        v = sexp[r * sexp_dw + (o - codes_dw)];
    else
        v = mexp[r * mexp_dw + (o - codes_dw - sexp_dw)];
    table[t] = v;
}

int table_pack(const bdr_format &f, const void *codes, const void *sexp, const void *mexp, int64_t rows,
               int64_t cols, void *table, hipStream_t s)
{
    const int32_t codes_dw = (int32_t)(cols / 8 * (f.m + 1) / 4), e_dw = (int32_t)(cols / 64);
    const int64_t n = rows * (codes_dw + 2 * (int64_t)e_dw);
    hipLaunchKernelGGL(table_pack_kernel, dim3(blocks_for(n)), dim3(kThreads), 0, s, (const uint32_t *)codes,
                       (const uint32_t *)sexp, (const uint32_t *)mexp, n, codes_dw, e_dw, e_dw,
                       (uint32_t *)table);
    return launch_status();
}

template <typename T>
static int table_gather_t(const bdr_format &f, const uint8_t *table, int64_t table_rows, int64_t cols,
                          const int64_t *idx, int64_t n_idx, T *y, hipStream_t s)
{
    const int64_t ng = n_idx * cols / 8;
    const int32_t codes_row = (int32_t)(cols / 8 * (f.m + 1)), e_row = (int32_t)(cols / 16);
    const GatherArgs ga = {idx, table_rows, (int32_t)(cols / 8), 0, codes_row + 2 * e_row, codes_row, e_row};
    if (f.m == 7)
        hipLaunchKernelGGL((mx_dequantize_row_kernel<7, T, true, false, 4, 1, 1, true>), (gather_grid<7, T>(ng)), dim3(kDeqThreads), 0, s, table, table, table, y, ng, ga);
    else if (f.m == 4)
        hipLaunchKernelGGL((mx_dequantize_row_kernel<4, T, true, false, 4, 1, 1, true>), (gather_grid<4, T>(ng)), dim3(kDeqThreads), 0, s, table, table, table, y, ng, ga);
    else
        hipLaunchKernelGGL((mx_dequantize_row_kernel<2, T, true, false, 4, 1, 1, true>), (gather_grid<2, T>(ng)), dim3(kDeqThreads), 0, s, table, table, table, y, ng, ga);
    return launch_status();
}

int table_gather_dequantize(const bdr_format &f, const void *table, int64_t table_rows, int64_t cols,
                            const int64_t *idx, int64_t n_idx, void *y, int dtype, hipStream_t s)
{
    if (dtype == BDR_F32)
        return table_gather_t(f, (const uint8_t *)table, table_rows, cols, idx, n_idx, (float *)y, s);
    return table_gather_t(f, (const uint8_t *)table, table_rows, cols, idx, n_idx, (uint16_t *)y, s);
}

template <typename T>
static int gather_row_t(const bdr_format &f, const uint8_t *codes, const uint8_t *sexp,
                        const uint8_t *mexp, int64_t table_rows, int64_t cols, const int64_t *idx,
                        int64_t n_idx, T *y, hipStream_t s)
{
    const int64_t ng = n_idx * cols / 8;
    const GatherArgs ga = {idx, table_rows, (int32_t)(cols / 8), 0, 0, 0, 0};
    if (f.m == 7)
        hipLaunchKernelGGL((mx_dequantize_row_kernel<7, T, true>), (gather_grid<7, T>(ng)), dim3(kDeqThreads), 0, s, codes, sexp, mexp, y, ng, ga);
    else if (f.m == 4)
        hipLaunchKernelGGL((mx_dequantize_row_kernel<4, T, true>), (gather_grid<4, T>(ng)), dim3(kDeqThreads), 0, s, codes, sexp, mexp, y, ng, ga);
    else
        hipLaunchKernelGGL((mx_dequantize_row_kernel<2, T, true>), (gather_grid<2, T>(ng)), dim3(kDeqThreads), 0, s, codes, sexp, mexp, y, ng, ga);
    return launch_status();
}

int gather_dequantize_row(const bdr_format &f, const void *codes, const void *sexp, const void *mexp,
                          int64_t table_rows, int64_t cols, const int64_t *idx, int64_t n_idx, void *y,
                          int dtype, hipStream_t s)
{
    if (dtype == BDR_F32)
        return gather_row_t(f, (const uint8_t *)codes, (const uint8_t *)sexp, (const uint8_t *)mexp,
                            table_rows, cols, idx, n_idx, (float *)y, s);
    return gather_row_t(f, (const uint8_t *)codes, (const uint8_t *)sexp, (const uint8_t *)mexp,
                        table_rows, cols, idx, n_idx, (uint16_t *)y, s);
}

template <typename T>
static int qdq_row_t(const bdr_format &f, const T *x, T *y, int64_t rows, int64_t cols, int64_t ld,
                     hipStream_t s)
{
    if (ragged(f, cols))
        return generic_view_t(2, f, x, y, rows, cols, ld, (int64_t)1, (uint8_t *)nullptr, (uint8_t *)nullptr,
                              (uint8_t *)nullptr, s);
    const int64_t ng = rows * cols / 8;
    const dim3 grid(blocks_for(ng)), block(kThreads);
    if (is_mx(f) && ld == cols && sizeof(T) == 4) {
        const int64_t n4 = rows * cols / 4;
        const dim3 g4(blocks_for(n4));
        if (f.m == 7)
            hipLaunchKernelGGL((mx_qdq_row_f32x4_kernel<7>), g4, block, 0, s, (const float *)x, (float *)y, n4);
        else if (f.m == 4)
            hipLaunchKernelGGL((mx_qdq_row_f32x4_kernel<4>), g4, block, 0, s, (const float *)x, (float *)y, n4);
        else
            hipLaunchKernelGGL((mx_qdq_row_f32x4_kernel<2>), g4, block, 0, s, (const float *)x, (float *)y, n4);
        return launch_status();
    }
    if (is_mx(f) && ld == cols) {
        if (f.m == 7)
            hipLaunchKernelGGL((mx_qdq_row_kernel<7, T>), grid, block, 0, s, x, y, ng);
        else if (f.m == 4)
            hipLaunchKernelGGL((mx_qdq_row_kernel<4, T>), grid, block, 0, s, x, y, ng);
        else
            hipLaunchKernelGGL((mx_qdq_row_kernel<2, T>), grid, block, 0, s, x, y, ng);
    } else {
        bool done = false;
        if constexpr (sizeof(T) == 4) {
            // (the fused round trip writes no planes and gains nothing from a compiled-in
            // tuple: it is bound by its 2 x 4 bytes per element either way)
            if (ld == cols) {
                hipLaunchKernelGGL((generic_quantize_kernel<T, 1, false, true>), grid, block, 0, s, gen_of(f),
                                   x, y, (uint8_t *)nullptr, (uint8_t *)nullptr, (uint8_t *)nullptr, cols,
                                   ld, (int64_t)1, ng, cols);
                done = true;
            }
        }
        if constexpr (sizeof(T) == 2) {
            // BF16 rows carry twice the elements per byte, and there the compiled-in tuple does pay
            const int spec = ld == cols ? hot_index(f) : -1;
            if (spec >= 0) {
                launch_hot_fused<T>(spec, grid, s, x, y, cols, ng);
                done = true;
            }
        }
        if (!done)
            hipLaunchKernelGGL((generic_quantize_kernel<T, 1, false, false>), grid, block, 0, s, gen_of(f),
                               x, y, (uint8_t *)nullptr, (uint8_t *)nullptr, (uint8_t *)nullptr, cols,
                               ld, (int64_t)1, ng, cols);
    }
    return launch_status();
}

int qdq_row(const bdr_format &f, const void *x, void *y, int dtype, int64_t rows, int64_t cols,
            int64_t ld, hipStream_t s)
{
    if (dtype == BDR_F32) return qdq_row_t(f, (const float *)x, (float *)y, rows, cols, ld, s);
    return qdq_row_t(f, (const uint16_t *)x, (uint16_t *)y, rows, cols, ld, s);
}

// Any view through the element-at-a-time forms of the general kernels: R rows of n elements,
// element (r, c) at offset r * sr + c * sc.  A row whose length is not a whole number of
// blocks is stored as if it were padded with +0 to the next multiple of k1 (a last block of
// N < k1 elements is a block of size N: its maximum and its errors are those of the N
// elements; Sec. IX, the remark after Theorem 1); the pads' codes are 0 and dequantize does
// not write them.  The padded length is a multiple of 8 (checked by the caller).
template <typename T>
static int generic_view_t(int what, const bdr_format &f, const T *x, T *y, int64_t R, int64_t n,
                          int64_t sr, int64_t sc, uint8_t *codes, uint8_t *sexp, uint8_t *mexp,
                          hipStream_t s)
{
    const int64_t np = (n + f.k1 - 1) / f.k1 * f.k1;
    const int64_t ng = R * np / 8;
    const dim3 grid(blocks_for(ng)), block(kThreads);
    if (what == 0)
        hipLaunchKernelGGL((generic_quantize_kernel<T, 0, true, false>), grid, block, 0, s, gen_of(f), x,
                           (T *)nullptr, codes, sexp, mexp, np, sr, sc, ng, n);
    else if (what == 1)
        hipLaunchKernelGGL((generic_dequantize_kernel<T, true, false>), grid, block, 0, s, gen_of(f),
                           codes, sexp, mexp, (R * np / f.k2 * f.d2 + 7) / 8, y, np, sr, sc, ng, n);
    else
        hipLaunchKernelGGL((generic_quantize_kernel<T, 1, true, false>), grid, block, 0, s, gen_of(f), x,
                           y, (uint8_t *)nullptr, (uint8_t *)nullptr, (uint8_t *)nullptr, np, sr, sc, ng, n);
    return launch_status();
}

// ---- quantize straight into an operand image of the product kernel
//
// For a tensor that is quantized only to be multiplied (Sec. V: both inputs of every tensor
// operation of a training iteration), the three planes are a detour: the product's two-pass
// form would read them back at once and rewrite them as the image its kernel takes.  Here
// the quantizer writes that image itself:
//   KIND 0 / 1: a block's 16-byte FP6 chunk for an A / B operand (mx_quant_fp6_block), stored at
//               [K step of 4 blocks][row][4 chunks];
//   KIND 2:     a block's 16 dequantized BF16 values, stored at
//               [K step of 2 blocks][row][4 chunks of 8 values];
//   KIND 3:     (MX4 only) a block's 8 bytes of FP4 codes, stored at [K step of 8 blocks][row][4
//               chunks of 2 blocks], and its scale byte in a scale image after the chunks.
constexpr int kOperandFp6A = 0, kOperandFp6B = 1, kOperandBf16 = 2, kOperandFp4 = 3;

// Both images are [K step][row][four 16-byte chunks], and in both row-wise kernels a lane makes
// one chunk, so four consecutive lanes write one 64-byte piece.  A wave takes kImgRows rows x
// kImgSteps K steps (measured on 8192 x 12288 BF16, MX9: 1 step 115 us, 2: 79, 4: 72, 8: 71,
// 16: 93): it reads kImgSteps contiguous steps of each row and writes kImgRows x 64 contiguous
// bytes of each step; the four waves of a workgroup stack on rows.
constexpr int kImgSteps = 4, kImgRows = 16 / kImgSteps, kImgTileRows = kThreads / 64 * kImgRows;

// LANES lanes per K step of a row (4: one chunk each; 8: the FP4 image, half a chunk each).
struct ImgLane { int64_t row; int32_t q, c; bool in; };
template <int LANES = 4>
__device__ __forceinline__ ImgLane img_lane(int64_t rows, int32_t row_steps, int32_t step_tiles)
{
    const int tid = threadIdx.x, j = tid / LANES;
    const int64_t tile = blockIdx.x, rt = tile / step_tiles;
    ImgLane l;
    l.c = tid % LANES;
    l.q = (int32_t)(tile - rt * step_tiles) * kImgSteps + (j % kImgSteps);
    l.row = rt * (kThreads / LANES / kImgSteps) + j / kImgSteps;
    l.in = l.row < rows && l.q < row_steps;  // the lanes of a K step agree
    return l;
}

// KIND 0 or 1: a lane holds one whole block (16 elements of a 64-element K step).
template <int MB, typename T, int KIND>
__global__ __launch_bounds__(kThreads) void mx_quantize_operand_row_kernel(
    const T *__restrict__ x, int64_t rows, int32_t row_steps, int32_t step_tiles, int64_t ld,
    u32x4 *__restrict__ out)
{
    __shared__ uint8_t s_map[128];
    fp6_map_fill<MB>(s_map);
    __syncthreads();
    const ImgLane l = img_lane(rows, row_steps, step_tiles);
    if (!l.in) return;
    const T *src = x + l.row * ld + 64 * (int64_t)l.q + 16 * l.c;
    uint32_t xb[16], lo[8], hi[8];
    if constexpr (sizeof(T) == 4) {
        load8(src, lo);
        load8(src + 8, hi);
    } else {
        widen8(ldg<true>(reinterpret_cast<const u32x4 *>(src)), lo);
        widen8(ldg<true>(reinterpret_cast<const u32x4 *>(src) + 1), hi);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        xb[i] = lo[i];
        xb[8 + i] = hi[i];
    }
    const u32x4 chunk = mx_quant_fp6_block<MB, KIND == kOperandFp6B>(xb, s_map);
    stg<true>(chunk, out + (((int64_t)l.q * rows + l.row) * 4 + l.c));
}

// The BF16 image: a K step is 32 elements = four lanes of the 8-elements-per-lane quantizers, so
// the fused round trip's own shape fits: a block is two adjacent lanes (one DPP exchange) and a
// lane's 8 dequantized values are one chunk.
template <int MB, typename T>
__global__ __launch_bounds__(kThreads) void mx_quantize_bf16_image_row_kernel(
    const T *__restrict__ x, int64_t rows, int32_t row_steps, int32_t step_tiles, int64_t ld,
    u32x4 *__restrict__ out)
{
    const ImgLane l = img_lane(rows, row_steps, step_tiles);
    if (!l.in) return;
    uint32_t xb[8], yb[8], lo, hi, se, tau4;
    load8(x + l.row * ld + 32 * (int64_t)l.q + 8 * l.c, xb);
    mx_quant8<MB, true>(xb, lo, hi, se, tau4, yb);
    const u32x4 v = {__builtin_amdgcn_perm(yb[1], yb[0], 0x07060302u), __builtin_amdgcn_perm(yb[3], yb[2], 0x07060302u),
                     __builtin_amdgcn_perm(yb[5], yb[4], 0x07060302u), __builtin_amdgcn_perm(yb[7], yb[6], 0x07060302u)};
    stg<true>(v, out + (((int64_t)l.q * rows + l.row) * 4 + l.c));
}

// The FP4 image (MX4 only): a K step is 128 elements = 8 blocks = 8 lanes with one block each.
// A lane writes its 8 bytes of E2M1 codes into chunk c / 2 of [K step][row][4 chunks] (rows with
// bit 4 set keep the two blocks of a chunk in swapped order, as the product kernel reads them);
// the step's 8 scale bytes go to the scale image [K step][row padded to 128][even blocks' four,
// odd blocks' four], gathered by three DPP steps and written by lanes 0 and 1.  The rows that only
// pad the scale image are visited too and get zero scales.
template <typename T>
__global__ __launch_bounds__(kThreads) void mx_quantize_fp4_image_row_kernel(
    const T *__restrict__ x, int64_t rows, int64_t rows_pad, int32_t row_steps, int32_t step_tiles,
    int64_t ld, uint8_t *__restrict__ out, uint8_t *__restrict__ scales)
{
    const ImgLane l = img_lane<8>(rows_pad, row_steps, step_tiles);
    if (!l.in) return;
    uint32_t w0 = 0, w1 = 0, scale = 0;
    const bool real = l.row < rows;  // uniform over the 8 lanes
    if (real) {
        const T *src = x + l.row * ld + 128 * (int64_t)l.q + 16 * l.c;
        uint32_t xb[16], lo[8], hi[8];
        if constexpr (sizeof(T) == 4) {
            load8(src, lo);
            load8(src + 8, hi);
        } else {
            widen8(ldg<true>(reinterpret_cast<const u32x4 *>(src)), lo);
            widen8(ldg<true>(reinterpret_cast<const u32x4 *>(src) + 1), hi);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            xb[i] = lo[i];
            xb[8 + i] = hi[i];
        }
        mx_quant_fp4_block(xb, w0, w1, scale);
        const int half = (l.c & 1) ^ (int)((l.row >> 4) & 1);
        stg<true>(u32x2{w0, w1}, reinterpret_cast<u32x2 *>(
                                     out + (((int64_t)l.q * rows + l.row) * 4 + (l.c >> 1)) * 16 + 8 * half));
    }
    // byte c / 2 of the word of this lane's parity, then OR over the four lanes of that parity
    uint32_t sw = scale << (8 * (l.c >> 1));
    sw |= dpp<kQuadXor2>(sw);
    sw |= dpp<kQuadXor1>(dpp<kQuadXor2>(dpp<kRowHalfMirror>(sw)));  // lane c ^ 4 (7 - c, then ^ 3)
    if (l.c < 2)
        *reinterpret_cast<uint32_t *>(scales + ((int64_t)l.q * rows_pad + l.row) * 8 + 4 * l.c) = sw;
}

template <int MB, typename T>
static void launch_operand_row(int kind, dim3 grid, hipStream_t s, const T *x, int64_t rows, int32_t steps,
                               int32_t st, int64_t ld, u32x4 *o)
{
    const dim3 block(kThreads);
    if (kind == kOperandBf16)
        hipLaunchKernelGGL((mx_quantize_bf16_image_row_kernel<MB, T>), grid, block, 0, s, x, rows, steps, st, ld, o);
    else if constexpr (MB <= 4) {
        if (kind == kOperandFp6B)
            hipLaunchKernelGGL((mx_quantize_operand_row_kernel<MB, T, kOperandFp6B>), grid, block, 0, s, x, rows, steps, st, ld, o);
        else
            hipLaunchKernelGGL((mx_quantize_operand_row_kernel<MB, T, kOperandFp6A>), grid, block, 0, s, x, rows, steps, st, ld, o);
    }
}

template <typename T>
static int quantize_operand_row_t(const bdr_format &f, const T *x, int64_t rows, int64_t cols, int64_t ld,
                                  void *out, int kind, hipStream_t s)
{
    if (kind == kOperandFp4) {  // f is MX4; chunks, then the scale image
        const int32_t steps = (int32_t)(cols / 128), st = (steps + kImgSteps - 1) / kImgSteps;
        const int64_t rows_pad = (rows + 127) / 128 * 128;
        constexpr int kTile = kThreads / 8 / kImgSteps;
        uint8_t *o = (uint8_t *)out;
        hipLaunchKernelGGL((mx_quantize_fp4_image_row_kernel<T>), dim3((unsigned)(rows_pad / kTile * st)),
                           dim3(kThreads), 0, s, x, rows, rows_pad, steps, st, ld, o, o + rows * (cols / 2));
        return launch_status();
    }
    const int32_t steps = (int32_t)(cols / (kind == kOperandBf16 ? 32 : 64));
    const int32_t st = (steps + kImgSteps - 1) / kImgSteps;
    const dim3 grid((unsigned)((rows + kImgTileRows - 1) / kImgTileRows * st));
    u32x4 *o = (u32x4 *)out;
    if (f.m == 7)
        launch_operand_row<7, T>(kind, grid, s, x, rows, steps, st, ld, o);
    else if (f.m == 4)
        launch_operand_row<4, T>(kind, grid, s, x, rows, steps, st, ld, o);
    else
        launch_operand_row<2, T>(kind, grid, s, x, rows, steps, st, ld, o);
    return launch_status();
}

// x [rows x cols], blocks along the rows' own direction (K = cols, a multiple of 64; of 128 for the
// FP4 kind); f is one of Table II's formats (the FP6 kinds: MX6 or MX4; the FP4 kind: MX4), kind
// one of kOperand*.
int quantize_operand_row(const bdr_format &f, const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld,
                         void *out, int kind, hipStream_t s)
{
    if (dtype == BDR_F32) return quantize_operand_row_t(f, (const float *)x, rows, cols, ld, out, kind, s);
    return quantize_operand_row_t(f, (const uint16_t *)x, rows, cols, ld, out, kind, s);
}

// Column blocks: the transposed view [cols x rows].
int generic_col(int what, const bdr_format &f, const void *x, void *y, int dtype, int64_t rows,
                int64_t cols, int64_t ld, void *codes, void *sexp, void *mexp, hipStream_t s)
{
    if (dtype == BDR_F32)
        return generic_view_t(what, f, (const float *)x, (float *)y, cols, rows, (int64_t)1, ld,
                              (uint8_t *)codes, (uint8_t *)sexp, (uint8_t *)mexp, s);
    return generic_view_t(what, f, (const uint16_t *)x, (uint16_t *)y, cols, rows, (int64_t)1, ld,
                          (uint8_t *)codes, (uint8_t *)sexp, (uint8_t *)mexp, s);
}

}  // namespace bdr
