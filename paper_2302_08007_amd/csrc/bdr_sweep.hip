// QSNR of many BDR formats on one tensor, reading the tensor once.
//
// QSNR is the ratio of signal power to quantization-noise power in decibels
// (Sec. IV-A, Eq. 3); the design-space study of the paper evaluates it for
// hundreds of format tuples (Sec. IV).  This file does the noise half of that
// study on the GPU: per format f, S_err[f] = sum (Q_f(x) - x)^2, plus one
// S_sig = sum x^2, then 10 log10(S_sig / S_err[f]).
//
// How the work is shared between formats:
//   - The exponent of the maximum over every aligned power-of-two group of
//     1 .. 256 elements is computed once per load (in-lane for groups up to 8,
//     DPP / one shuffle across lanes above that).
//   - Formats are grouped on the host into "classes" (k1, k2, d2): within a
//     class every element has the same effective exponent
//         eps = max(E_block - beta, E_subblock)      (Sec. IX: tau <= beta)
//     so it is computed once per class.  d2 = 0 and k2 = k1 both mean tau = 0
//     and share a class; identical tuples share one accumulator.
//   - A quantizer (class, m, rounding) then costs six VALU operations per
//     element: scale, clamp, round, subtract, unscale, square-accumulate.
//
// Range: squares of FP32 numbers underflow for small tensors, so the kernel works
// on x * 2^s with s chosen from the tensor's largest exponent (a tiny pre-pass)
// and undoes the scale in FP64 at the end.  Scaling by a power of two commutes
// with the quantizer (end of Sec. IX), so nothing changes except for values more
// than 126 binades below the tensor maximum, whose contribution is below 2^-250
// of either sum.
//
// Sums: FP32 inside a lane over at most 32 elements, FP64 from there on;
// per-block partials are combined in a fixed order, so results are reproducible.
#include "bdr_device.hpp"
#include "bdr_internal.hpp"

namespace bdr {

namespace {

constexpr int kSweepThreads = 256;
constexpr int kWaves = kSweepThreads / 64;
constexpr int kG = 4;  // groups of 8 elements per lane per iteration
constexpr int kMaxBlocks = 2048;
constexpr int kChunk = 256;  // formats per launch: keeps the kernel arguments under 4 KiB
constexpr int kMaxClasses = kChunk;
constexpr int kMaxQuant = kChunk;
constexpr size_t kHeaderBytes = 256;                            // Header
constexpr size_t kTotalsBytes = 4096 - 256;                     // kChunk + 1 doubles fit

struct ClassDesc {
    uint8_t lk1, lk2, beta, nq;  // log2 k1, log2 k2, 2^d2 - 1, quantizers in the class
    uint16_t first;              // index of its first quantizer
};
struct QuantDesc {
    uint8_t m, rounding;
};
struct SweepPlan {
    int32_t n_class, n_quant;
    ClassDesc cls[kMaxClasses];
    QuantDesc q[kMaxQuant];
};
struct FormatMap {
    uint16_t idx[kChunk];  // format -> quantizer
};

struct Header {
    uint32_t absmax_bits;
};

__global__ void sweep_clear_kernel(Header *h) { h->absmax_bits = 0; }

// Largest magnitude of the tensor.  Only its exponent is used, so a block whose
// maximum does not raise the exponent already recorded skips the atomic.
template <typename T>
__global__ __launch_bounds__(256) void sweep_absmax_kernel(const T *__restrict__ x, int64_t cols,
                                                           int64_t ld, int64_t n_groups, Header *h)
{
    __shared__ uint32_t s_m[4];
    uint32_t m = 0;
    for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < n_groups;
         g += (int64_t)gridDim.x * 256) {
        const int64_t t0 = 8 * g;
        const int64_t r = ld == cols ? 0 : t0 / cols;
        uint32_t xb[8];
        load8(x + r * ld + (t0 - r * cols), xb);
#pragma unroll
        for (int i = 0; i < 8; ++i) m = umax(m, xb[i] & kAbsMask);
    }
    for (int w = 32; w > 0; w >>= 1) m = umax(m, (uint32_t)__shfl_xor((int)m, w));
    if ((threadIdx.x & 63) == 0) s_m[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = umax(umax(s_m[0], s_m[1]), umax(s_m[2], s_m[3]));
        const uint32_t seen = __atomic_load_n(&h->absmax_bits, __ATOMIC_RELAXED);
        if ((m >> 23) > (seen >> 23)) atomicMax(&h->absmax_bits, m);
    }
}

// Scaling exponents 127 - e of the maxima over aligned groups, for one run of 8
// elements, as signed bytes (127 - e lies in [-127, 126]):
//   w[0], w[1]  per element            w[2]  per pair
//   w[3]        per 4 (bytes 0-1), per 8 and per 16 (bytes 2-3)
//   w[4]        per 32, 64, 128, 256
struct Levels {
    uint32_t w[5];
};

__device__ __forceinline__ uint32_t neg_exp_byte(uint32_t mag) { return (127u - (mag >> 23)) & 0xffu; }

__device__ __forceinline__ uint32_t pack4(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    return a | (b << 8) | (c << 16) | (d << 24);
}

__device__ __forceinline__ void build_levels(const uint32_t (&ab)[8], uint32_t mag_lo, Levels &L)
{
    uint32_t p0[8], p1[4], p2[2], pl[6];
#pragma unroll
    for (int i = 0; i < 8; ++i) p0[i] = umin(umax(ab[i], mag_lo), kMagHi);
#pragma unroll
    for (int i = 0; i < 4; ++i) p1[i] = umax(p0[2 * i], p0[2 * i + 1]);
#pragma unroll
    for (int i = 0; i < 2; ++i) p2[i] = umax(p1[2 * i], p1[2 * i + 1]);
    uint32_t v = umax(p2[0], p2[1]);
    pl[0] = v;
    v = umax(v, dpp<kQuadXor1>(v));
    pl[1] = v;
    v = umax(v, dpp<kQuadXor2>(v));
    pl[2] = v;
    v = umax(v, dpp<kRowHalfMirror>(v));
    pl[3] = v;
    v = umax(v, dpp<kRowMirror>(v));
    pl[4] = v;
    v = umax(v, (uint32_t)__shfl_xor((int)v, 16));
    pl[5] = v;
    L.w[0] = pack4(neg_exp_byte(p0[0]), neg_exp_byte(p0[1]), neg_exp_byte(p0[2]), neg_exp_byte(p0[3]));
    L.w[1] = pack4(neg_exp_byte(p0[4]), neg_exp_byte(p0[5]), neg_exp_byte(p0[6]), neg_exp_byte(p0[7]));
    L.w[2] = pack4(neg_exp_byte(p1[0]), neg_exp_byte(p1[1]), neg_exp_byte(p1[2]), neg_exp_byte(p1[3]));
    L.w[3] = pack4(neg_exp_byte(p2[0]), neg_exp_byte(p2[1]), neg_exp_byte(pl[0]), neg_exp_byte(pl[1]));
    L.w[4] = pack4(neg_exp_byte(pl[2]), neg_exp_byte(pl[3]), neg_exp_byte(pl[4]), neg_exp_byte(pl[5]));
}

__device__ __forceinline__ int sbyte(uint32_t w, int idx)
{
    return __builtin_amdgcn_sbfe((int)w, 8 * idx, 8);
}

// 127 - e for a group of 8 or more elements (lk >= 3): one value per lane.
__device__ __forceinline__ int lane_level(const Levels &L, int lk)
{
    const uint64_t both = ((uint64_t)L.w[4] << 32) | L.w[3];
    return (int)(int8_t)(both >> (8 * (lk - 1)));  // lk = 3 is byte 2 of w[3]
}

// 127 - e of the level-lk group each of the 8 elements belongs to.
__device__ __forceinline__ void level_exps(const Levels &L, int lk, int (&out)[8])
{
    if (lk == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = sbyte(L.w[i >> 2], i & 3);
    } else if (lk == 1) {
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = sbyte(L.w[2], i >> 1);
    } else if (lk == 2) {
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = sbyte(L.w[3], i >> 2);
    } else {
        const int v = lane_level(L, lk);
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = v;
    }
}

// Squared error of one quantizer summed over the lane's kG*8 elements, in the
// tensor's (pre-scaled) units.  yp = |x| * 2^sh lies in [0, 2) with the top
// magnitude bit at weight 2^0; nsh = -sh.
//   nearest-even: adding 2^(24-m) to a value in [0, 2) rounds it to a multiple
//   of 2^-(m-1), which is the step of an m-bit magnitude at that weight.
template <int ROUNDING>
__device__ __forceinline__ float quant_err2(const float (&yp)[kG][8], const int (&nsh)[kG][8], int m)
{
    const float step = __builtin_ldexpf(1.0f, 1 - m);
    const float top = 2.0f - step;
    const float magic = __builtin_ldexpf(1.0f, 24 - m);
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < kG; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // held at the top code; both are non-negative, so the integer minimum of the
            // bit patterns is the float minimum (and needs no NaN canonicalization)
            const float y = as_f(umin(as_u(yp[j][i]), as_u(top)));
            float r;
            if (ROUNDING == BDR_RNE) {
                r = (y + magic) - magic;
            } else {
                const float sc = __builtin_ldexpf(y, m - 1);
                const float t = __builtin_truncf(sc);
                const float up = (ROUNDING == BDR_RNA && (sc - t) >= 0.5f) ? 1.0f : 0.0f;
                r = __builtin_ldexpf(t + up, 1 - m);
            }
            const float d = __builtin_ldexpf(yp[j][i] - r, nsh[j][i]);  // difference is exact
            acc = __builtin_fmaf(d, d, acc);
        }
    return acc;
}

__device__ __forceinline__ float wave_sum(float v)
{
    v += as_f(dpp<kQuadXor1>(as_u(v)));
    v += as_f(dpp<kQuadXor2>(as_u(v)));
    v += as_f(dpp<kRowHalfMirror>(as_u(v)));
    v += as_f(dpp<kRowMirror>(as_u(v)));
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

template <typename T>
__global__ __launch_bounds__(kSweepThreads) void sweep_kernel(
    SweepPlan plan, const T *__restrict__ x, int64_t cols, int64_t ld, int64_t n_groups,
    const Header *__restrict__ hdr, double *__restrict__ partials)
{
    extern __shared__ double s_acc[];  // [kWaves][n_quant + 1]
    const int nq = plan.n_quant;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int t = threadIdx.x; t < kWaves * (nq + 1); t += kSweepThreads) s_acc[t] = 0.0;
    __syncthreads();
    double *wacc = s_acc + wave * (nq + 1);

    // Work on x * 2^sref so that the tensor maximum lands in [1, 2).
    const int eref = (int)(umin(umax(hdr->absmax_bits, kMagLo), kMagHi) >> 23);
    const int sref = 127 - eref;
    // the lowest exponent an element can carry (code 1 before scaling)
    const uint32_t mag_lo = (uint32_t)(1 + (sref > 0 ? sref : 0)) << 23;

    const int64_t per_iter = (int64_t)gridDim.x * kSweepThreads * kG;
    for (int64_t base = (int64_t)blockIdx.x * kSweepThreads * kG; base < n_groups;
         base += per_iter) {
        float ax[kG][8];
        Levels L[kG];
        float sig = 0.f;
#pragma unroll
        for (int j = 0; j < kG; ++j) {
            const int64_t g = base + (int64_t)wave * (64 * kG) + j * 64 + lane;
            uint32_t xb[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            if (g < n_groups) {
                const int64_t t0 = 8 * g;
                const int64_t r = ld == cols ? 0 : t0 / cols;
                load8(x + r * ld + (t0 - r * cols), xb);
            }
            uint32_t ab[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                ax[j][i] = __builtin_ldexpf(__builtin_fabsf(as_f(xb[i])), sref);
                ab[i] = as_u(ax[j][i]);
                sig = __builtin_fmaf(ax[j][i], ax[j][i], sig);
            }
            build_levels(ab, mag_lo, L[j]);
        }
        sig = wave_sum(sig);
        if (lane == 0) wacc[nq] += (double)sig;

        for (int c = 0; c < plan.n_class; ++c) {
            const ClassDesc cd = plan.cls[c];
            // sh = 127 - max(E_block - beta, E_sub) = min(127 - E_block + beta, 127 - E_sub)
            float yp[kG][8];
            int nsh[kG][8];
#pragma unroll
            for (int j = 0; j < kG; ++j) {
                int cb[8], cs[8];
                level_exps(L[j], cd.lk1, cb);
                level_exps(L[j], cd.lk2, cs);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int sh = min(cb[i] + (int)cd.beta, cs[i]);
                    yp[j][i] = __builtin_ldexpf(ax[j][i], sh);
                    nsh[j][i] = -sh;
                }
            }
            for (int k = 0; k < cd.nq; ++k) {
                const QuantDesc qd = plan.q[cd.first + k];
                float e2;
                if (qd.rounding == BDR_RNE)
                    e2 = quant_err2<BDR_RNE>(yp, nsh, qd.m);
                else if (qd.rounding == BDR_RNA)
                    e2 = quant_err2<BDR_RNA>(yp, nsh, qd.m);
                else
                    e2 = quant_err2<BDR_RTZ>(yp, nsh, qd.m);
                e2 = wave_sum(e2);
                if (lane == 0) wacc[cd.first + k] += (double)e2;
            }
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t <= nq; t += kSweepThreads) {
        double v = 0.0;
        for (int w = 0; w < kWaves; ++w) v += s_acc[w * (nq + 1) + t];
        partials[(int64_t)blockIdx.x * (nq + 1) + t] = v;
    }
}

// Column t of the per-block partial sums, added up in a fixed order: lane i takes
// blocks i, i + 256, ... and the 256 lane sums go through a fixed tree.
__global__ __launch_bounds__(256) void sweep_reduce_kernel(int32_t n_quant, int32_t n_blocks,
                                                           const double *__restrict__ partials,
                                                           double *__restrict__ totals)
{
    __shared__ double s_v[256];
    const int t = blockIdx.x;
    double v = 0.0;
    for (int b = threadIdx.x; b < n_blocks; b += 256) v += partials[(int64_t)b * (n_quant + 1) + t];
    s_v[threadIdx.x] = v;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) s_v[threadIdx.x] += s_v[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) totals[t] = s_v[0];
}

__global__ __launch_bounds__(256) void sweep_finalize_kernel(
    FormatMap map, int32_t n_fmts, int32_t n_quant, const Header *__restrict__ hdr,
    const double *__restrict__ totals, double *__restrict__ qsnr_db, double *__restrict__ sums,
    double *sig_out)
{
    // undo the pre-scale: sums were taken on x * 2^(127 - eref)
    const int eref = (int)(umin(umax(hdr->absmax_bits, kMagLo), kMagHi) >> 23);
    const double unscale = __builtin_ldexp(1.0, -2 * (127 - eref));
    const double sig = totals[n_quant] * unscale;
    for (int f = threadIdx.x; f <= n_fmts; f += blockDim.x) {
        if (f == n_fmts) {
            *sig_out = sig;
        } else {
            const double err = totals[map.idx[f]] * unscale;
            sums[f] = err;
            qsnr_db[f] = err > 0.0 ? 10.0 * log10(sig / err) : __builtin_inf();
        }
    }
}

inline int ilog2(int v) { return __builtin_ctz((unsigned)v); }

}  // namespace

size_t sweep_workspace_bytes(int32_t n_fmts)
{
    const int per_launch = n_fmts < kChunk ? n_fmts : kChunk;
    return kHeaderBytes + kTotalsBytes + (size_t)kMaxBlocks * (size_t)(per_launch + 1) * sizeof(double);
}

namespace {

// Host plan for up to kChunk formats: classes of (k1, k2, beta) with the tau = 0
// formats merged, and within a class one quantizer per distinct (m, rounding).
void make_plan(const bdr_format *fmts, int n_fmts, SweepPlan &plan, FormatMap &map)
{
    struct Key {
        int lk1, lk2, beta, m, rnd;
    };
    Key keys[kMaxQuant];
    int order[kChunk];
    int nq = 0;
    for (int f = 0; f < n_fmts; ++f) {
        Key k = {ilog2(fmts[f].k1), ilog2(fmts[f].k2), (1 << fmts[f].d2) - 1, fmts[f].m,
                 fmts[f].rounding};
        if (k.beta == 0 || k.lk2 == k.lk1) {  // no sub-block shift: plain block floating point
            k.beta = 0;
            k.lk2 = k.lk1;
        }
        int found = -1;
        for (int j = 0; j < nq && found < 0; ++j)
            if (keys[j].lk1 == k.lk1 && keys[j].lk2 == k.lk2 && keys[j].beta == k.beta &&
                keys[j].m == k.m && keys[j].rnd == k.rnd)
                found = j;
        if (found < 0) {
            keys[nq] = k;
            found = nq++;
        }
        order[f] = found;
    }
    int newidx[kMaxQuant];
    bool placed[kMaxQuant] = {false};
    int nc = 0, pos = 0;
    for (int j = 0; j < nq; ++j) {
        if (placed[j]) continue;
        ClassDesc &cd = plan.cls[nc++];
        cd.lk1 = (uint8_t)keys[j].lk1;
        cd.lk2 = (uint8_t)keys[j].lk2;
        cd.beta = (uint8_t)keys[j].beta;
        cd.first = (uint16_t)pos;
        int cnt = 0;
        for (int i = j; i < nq; ++i) {
            if (placed[i] || keys[i].lk1 != keys[j].lk1 || keys[i].lk2 != keys[j].lk2 ||
                keys[i].beta != keys[j].beta)
                continue;
            placed[i] = true;
            newidx[i] = pos;
            plan.q[pos].m = (uint8_t)keys[i].m;
            plan.q[pos].rounding = (uint8_t)keys[i].rnd;
            ++pos;
            ++cnt;
        }
        cd.nq = (uint8_t)cnt;  // at most 8 values of m x 3 roundings
    }
    plan.n_class = nc;
    plan.n_quant = nq;
    for (int f = 0; f < n_fmts; ++f) map.idx[f] = (uint16_t)newidx[order[f]];
}

}  // namespace

int qsnr_sweep(const bdr_format *fmts, int32_t n_fmts, const void *x, int dtype, int64_t rows,
               int64_t cols, int64_t ld, double *qsnr_db, double *sums, void *workspace,
               hipStream_t s)
{
    static_assert(sizeof(SweepPlan) + 64 < 4096, "kernel arguments must stay under 4 KiB");
    Header *hdr = reinterpret_cast<Header *>(workspace);
    static_assert((kChunk + 1) * sizeof(double) <= kTotalsBytes, "totals area too small");
    double *totals = reinterpret_cast<double *>(static_cast<char *>(workspace) + kHeaderBytes);
    double *partials = reinterpret_cast<double *>(static_cast<char *>(workspace) + kHeaderBytes +
                                                  kTotalsBytes);
    const int64_t n_groups = rows * cols / 8;
    const int64_t per_block = (int64_t)kSweepThreads * kG;
    int64_t nb = (n_groups + per_block - 1) / per_block;
    if (nb > kMaxBlocks) nb = kMaxBlocks;
    if (nb < 1) nb = 1;

    hipLaunchKernelGGL(sweep_clear_kernel, dim3(1), dim3(1), 0, s, hdr);
    if (n_groups > 0) {
        const int64_t want = (n_groups + 255) / 256;
        const unsigned ab = (unsigned)(want < 1024 ? want : 1024);
        if (dtype == BDR_F32)
            hipLaunchKernelGGL(sweep_absmax_kernel<float>, dim3(ab), dim3(256), 0, s,
                               (const float *)x, cols, ld, n_groups, hdr);
        else
            hipLaunchKernelGGL(sweep_absmax_kernel<uint16_t>, dim3(ab), dim3(256), 0, s,
                               (const uint16_t *)x, cols, ld, n_groups, hdr);
    }
    // Chunks of formats run one after the other on the stream and reuse the
    // partial-sum area; each launch gets its own copy of the plan by value.
    for (int32_t f0 = 0; f0 < n_fmts; f0 += kChunk) {
        const int nf = n_fmts - f0 < kChunk ? n_fmts - f0 : kChunk;
        SweepPlan plan;
        FormatMap map;
        make_plan(fmts + f0, nf, plan, map);
        const int nq = plan.n_quant;
        const size_t lds = (size_t)kWaves * (size_t)(nq + 1) * sizeof(double);
        if (dtype == BDR_F32)
            hipLaunchKernelGGL(sweep_kernel<float>, dim3((unsigned)nb), dim3(kSweepThreads), lds,
                               s, plan, (const float *)x, cols, ld, n_groups, hdr, partials);
        else
            hipLaunchKernelGGL(sweep_kernel<uint16_t>, dim3((unsigned)nb), dim3(kSweepThreads),
                               lds, s, plan, (const uint16_t *)x, cols, ld, n_groups, hdr,
                               partials);
        hipLaunchKernelGGL(sweep_reduce_kernel, dim3((unsigned)(nq + 1)), dim3(256), 0, s, nq,
                           (int32_t)nb, partials, totals);
        hipLaunchKernelGGL(sweep_finalize_kernel, dim3(1), dim3(256), 0, s, map, nf, nq, hdr,
                           totals, qsnr_db + f0, sums + f0, sums + n_fmts);
    }
    return launch_status();
}

}  // namespace bdr
