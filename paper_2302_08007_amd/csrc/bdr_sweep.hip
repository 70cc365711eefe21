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
//   - Formats are put on the host into groups of equal k1.  With E the block
//     exponent, a format of the group quantizes an element at the effective
//     exponent E - tau, tau = min(beta, E - E_sub) (Sec. IX), so for a given
//     (m, rounding) the error of an element can only take beta + 1 values.  When
//     every format of the group has beta <= 1 the two candidate squared errors
//     (tau = 0 and tau = 1) are computed once per (m, rounding) and each
//     (k2, d2) class just selects between them: one compare per element per
//     class, one select and one add per element per quantizer.  d2 = 0 and
//     k2 = k1 both mean tau = 0 and share a class; identical tuples share one
//     accumulator.  Groups with a larger beta evaluate every class directly
//     (scale, clamp, round, subtract, unscale, square-accumulate).
//
// Range: squares of FP32 numbers underflow for small tensors, so the kernel works
// on x * 2^s with s chosen from the tensor's largest exponent (a tiny pre-pass)
// and undoes the scale in FP64 at the end.  Scaling by a power of two commutes
// with the quantizer (end of Sec. IX), so nothing changes except for values more
// than 126 binades below the tensor maximum, whose contribution is below 2^-250
// of either sum.
//
// Sums: every lane keeps one FP32 partial per quantizer in LDS (a lane sees only
// n / 524288 elements, so FP32 is ample), lanes and workgroups are combined in
// FP64 in a fixed order, so results are reproducible.
#include "bdr_device.hpp"
#include "bdr_internal.hpp"

namespace bdr {

namespace {

constexpr int kSweepThreads = 256;
constexpr int kG = 2;  // groups of 8 elements per lane per iteration
constexpr int kMaxBlocks = 2048;
constexpr int kChunk = 128;  // formats per launch: bounds kernel arguments (< 4 KiB) and LDS
constexpr int kMaxGroups = kChunk;
constexpr int kMaxClasses = kChunk;
constexpr int kMR = 2;       // (m, rounding) pairs evaluated together in one group
constexpr size_t kHeaderBytes = 256;          // Header
constexpr size_t kTotalsBytes = 4096 - 256;   // kChunk + 1 doubles fit
constexpr uint16_t kNone = 0xffff;

struct GroupDesc {
    uint8_t lk1;       // log2 k1
    uint8_t shared;    // 1: all classes have beta <= 1 and select between two candidates
    uint8_t n_mr;      // (m, rounding) pairs in use (<= kMR)
    uint8_t n_cls;     // classes of this group
    uint16_t first;    // index of its first class
    uint8_t m[kMR], rnd[kMR];
};
struct ClassDesc {
    uint8_t lk2, beta;   // log2 k2, 2^d2 - 1
    uint16_t q[kMR];     // accumulator of (this class, mr), kNone when no format asks for it
};
struct SweepPlan {
    int32_t n_group, n_quant;
    GroupDesc grp[kMaxGroups];
    ClassDesc cls[kMaxClasses];
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

// y in [0, 2) is |x| scaled so that the top magnitude bit has weight 2^0.  Returns
// y minus its m-bit quantized value (exact): nearest-even by adding 2^(24-m)
// (a value in [0, 2) then rounds to a multiple of 2^-(m-1), the step of an m-bit
// magnitude at that weight), or through an integer for ties-away / truncation.
struct MrConst {
    float top, magic;
    int m, rounding;
};
__device__ __forceinline__ MrConst mr_const(int m, int rounding)
{
    MrConst c;
    c.top = 2.0f - __builtin_ldexpf(1.0f, 1 - m);
    c.magic = __builtin_ldexpf(1.0f, 24 - m);
    c.m = m;
    c.rounding = rounding;
    return c;
}
template <int ROUNDING>
__device__ __forceinline__ float quant_diff(float yp, const MrConst &c)
{
    // held at the top code; both are non-negative, so the integer minimum of the
    // bit patterns is the float minimum (and needs no NaN canonicalization)
    const float y = as_f(umin(as_u(yp), as_u(c.top)));
    float r;
    if (ROUNDING == BDR_RNE) {
        r = (y + c.magic) - c.magic;
    } else {
        const float sc = __builtin_ldexpf(y, c.m - 1);
        const float t = __builtin_truncf(sc);
        const float up = (ROUNDING == BDR_RNA && (sc - t) >= 0.5f) ? 1.0f : 0.0f;
        r = __builtin_ldexpf(t + up, 1 - c.m);
    }
    return yp - r;
}

// squared error, in the tensor's (pre-scaled) units, of |x| = y * 2^-sh
template <int ROUNDING>
__device__ __forceinline__ float quant_err2(float y, int sh, const MrConst &c)
{
    const float d = __builtin_ldexpf(quant_diff<ROUNDING>(y, c), -sh);
    return d * d;
}

// both candidate squared errors of one (m, rounding): block exponent as is, and one lower
template <int ROUNDING>
__device__ __forceinline__ void candidates(const float (&ax)[kG][8], const int (&cb)[kG][8],
                                           const MrConst &c, float (&e0)[kG][8],
                                           float (&e1)[kG][8])
{
#pragma unroll
    for (int j = 0; j < kG; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float y0 = __builtin_ldexpf(ax[j][i], cb[j][i]);
            e0[j][i] = quant_err2<ROUNDING>(y0, cb[j][i], c);
            e1[j][i] = quant_err2<ROUNDING>(y0 + y0, cb[j][i] + 1, c);
        }
}

template <int ROUNDING>
__device__ __forceinline__ float direct(const float (&yp)[kG][8], const int (&sh)[kG][8],
                                        const MrConst &c)
{
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < kG; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) sum += quant_err2<ROUNDING>(yp[j][i], sh[j][i], c);
    return sum;
}

template <typename T>
__global__ __launch_bounds__(kSweepThreads) void sweep_kernel(
    SweepPlan plan, const T *__restrict__ x, int64_t cols, int64_t ld, int64_t n_groups,
    const Header *__restrict__ hdr, double *__restrict__ partials)
{
    extern __shared__ float s_lane[];  // [n_quant + 1][kSweepThreads]: one partial per lane
    const int nq = plan.n_quant;
    const int tid = threadIdx.x, lane = tid & 63;
    for (int q = 0; q <= nq; ++q) s_lane[q * kSweepThreads + tid] = 0.f;
    auto add_to = [&](int q, float v) { s_lane[q * kSweepThreads + tid] += v; };

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
            const int64_t g = base + (int64_t)(tid >> 6) * (64 * kG) + j * 64 + lane;
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
        add_to(nq, sig);

        for (int gi = 0; gi < plan.n_group; ++gi) {
            const GroupDesc gd = plan.grp[gi];
            int cb[kG][8];  // 127 - E_block: scaling |x| by 2^cb puts the block maximum in [1, 2)
#pragma unroll
            for (int j = 0; j < kG; ++j) level_exps(L[j], gd.lk1, cb[j]);

            if (gd.shared) {
                // candidates: squared error at tau = 0 and at tau = 1, per (m, rounding)
                float e0[kMR][kG][8], e1[kMR][kG][8];
#pragma unroll
                for (int r = 0; r < kMR; ++r) {
                    if (r < gd.n_mr) {
                        const MrConst c = mr_const(gd.m[r], gd.rnd[r]);
                        if (c.rounding == BDR_RNE)
                            candidates<BDR_RNE>(ax, cb, c, e0[r], e1[r]);
                        else if (c.rounding == BDR_RNA)
                            candidates<BDR_RNA>(ax, cb, c, e0[r], e1[r]);
                        else
                            candidates<BDR_RTZ>(ax, cb, c, e0[r], e1[r]);
                    }
                }
                for (int ci = 0; ci < gd.n_cls; ++ci) {
                    const ClassDesc cd = plan.cls[gd.first + ci];
                    if (cd.beta == 0) {
#pragma unroll
                        for (int r = 0; r < kMR; ++r) {
                            if (r < gd.n_mr && cd.q[r] != kNone) {
                                float sum = 0.f;
#pragma unroll
                                for (int j = 0; j < kG; ++j)
#pragma unroll
                                    for (int i = 0; i < 8; ++i) sum += e0[r][j][i];
                                add_to(cd.q[r], sum);
                            }
                        }
                    } else {
                        // tau = 1 exactly where the sub-block exponent is below the block's
                        bool down[kG][8];
#pragma unroll
                        for (int j = 0; j < kG; ++j) {
                            int cs[8];
                            level_exps(L[j], cd.lk2, cs);
#pragma unroll
                            for (int i = 0; i < 8; ++i) down[j][i] = cs[i] > cb[j][i];
                        }
#pragma unroll
                        for (int r = 0; r < kMR; ++r) {
                            if (r < gd.n_mr && cd.q[r] != kNone) {
                                float sum = 0.f;
#pragma unroll
                                for (int j = 0; j < kG; ++j)
#pragma unroll
                                    for (int i = 0; i < 8; ++i)
                                        sum += down[j][i] ? e1[r][j][i] : e0[r][j][i];
                                add_to(cd.q[r], sum);
                            }
                        }
                    }
                }
            } else {
                for (int ci = 0; ci < gd.n_cls; ++ci) {
                    const ClassDesc cd = plan.cls[gd.first + ci];
                    // sh = 127 - max(E_block - beta, E_sub) = min(127 - E_block + beta, 127 - E_sub)
                    int sh[kG][8];
                    float yp[kG][8];
#pragma unroll
                    for (int j = 0; j < kG; ++j) {
                        int cs[8];
                        level_exps(L[j], cd.lk2, cs);
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            sh[j][i] = min(cb[j][i] + (int)cd.beta, cs[i]);
                            yp[j][i] = __builtin_ldexpf(ax[j][i], sh[j][i]);
                        }
                    }
#pragma unroll
                    for (int r = 0; r < kMR; ++r) {
                        if (r < gd.n_mr && cd.q[r] != kNone) {
                            const MrConst c = mr_const(gd.m[r], gd.rnd[r]);
                            float sum;
                            if (c.rounding == BDR_RNE)
                                sum = direct<BDR_RNE>(yp, sh, c);
                            else if (c.rounding == BDR_RNA)
                                sum = direct<BDR_RNA>(yp, sh, c);
                            else
                                sum = direct<BDR_RTZ>(yp, sh, c);
                            add_to(cd.q[r], sum);
                        }
                    }
                }
            }
        }
    }
    __syncthreads();
    // Lane partials -> one FP64 value per quantizer for this workgroup.  32 quantizers
    // at a time: 8 threads share a quantizer, each sums 32 lanes (start rotated so a
    // wave touches 64 distinct banks), then the 8 are combined in a fixed order.
    const int part = tid & 7, slot = tid >> 3;
    const int rot = (slot & 7) + 8 * (part >> 1);
    for (int q0 = 0; q0 <= nq; q0 += 32) {
        const int q = q0 + slot;
        double v = 0.0;
        if (q <= nq) {
            const float *src = s_lane + q * kSweepThreads + part * 32;
#pragma unroll 8
            for (int i = 0; i < 32; ++i) v += (double)src[(i + rot) & 31];
        }
        v += __shfl_xor(v, 1);
        v += __shfl_xor(v, 2);
        v += __shfl_xor(v, 4);
        if (q <= nq && part == 0) partials[(int64_t)blockIdx.x * (nq + 1) + q] = v;
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

// Host plan for up to kChunk formats: groups of equal k1 (split so that a group
// holds at most kMR (m, rounding) pairs and is either all beta <= 1 or all
// beta >= 2), classes (k2, beta) inside a group with the tau = 0 formats merged,
// and one accumulator per distinct (class, m, rounding).
void make_plan(const bdr_format *fmts, int n_fmts, SweepPlan &plan, FormatMap &map)
{
    int ng = 0;
    int f_group[kChunk], f_mr[kChunk], f_lk2[kChunk], f_beta[kChunk];
    for (int f = 0; f < n_fmts; ++f) {
        const int lk1 = ilog2(fmts[f].k1);
        int lk2 = ilog2(fmts[f].k2), beta = (1 << fmts[f].d2) - 1;
        const int m = fmts[f].m, rnd = fmts[f].rounding;
        if (beta == 0 || lk2 == lk1) {  // no sub-block shift: plain block floating point
            beta = 0;
            lk2 = lk1;
        }
        const int shared = beta <= 1;
        // a group of this k1 and kind that has this (m, rounding), else one with room for it
        int gi = -1, r = -1;
        for (int g = 0; g < ng && gi < 0; ++g) {
            const GroupDesc &gd = plan.grp[g];
            if (gd.lk1 != lk1 || gd.shared != shared) continue;
            for (int k = 0; k < gd.n_mr; ++k)
                if (gd.m[k] == m && gd.rnd[k] == rnd) {
                    gi = g;
                    r = k;
                }
        }
        for (int g = 0; g < ng && gi < 0; ++g) {
            GroupDesc &gd = plan.grp[g];
            if (gd.lk1 != lk1 || gd.shared != shared || gd.n_mr == kMR) continue;
            gi = g;
            r = gd.n_mr++;
            gd.m[r] = (uint8_t)m;
            gd.rnd[r] = (uint8_t)rnd;
        }
        if (gi < 0) {
            gi = ng++;
            GroupDesc &gd = plan.grp[gi];
            gd = GroupDesc{};
            gd.lk1 = (uint8_t)lk1;
            gd.shared = (uint8_t)shared;
            gd.n_mr = 1;
            gd.m[0] = (uint8_t)m;
            gd.rnd[0] = (uint8_t)rnd;
            r = 0;
        }
        f_group[f] = gi;
        f_mr[f] = r;
        f_lk2[f] = lk2;
        f_beta[f] = beta;
    }
    // classes of a group are contiguous; accumulators are numbered in that order
    int nc = 0, nq = 0;
    for (int g = 0; g < ng; ++g) {
        GroupDesc &gd = plan.grp[g];
        gd.first = (uint16_t)nc;
        int n_cls = 0;
        for (int f = 0; f < n_fmts; ++f) {
            if (f_group[f] != g) continue;
            int ci = -1;
            for (int c = 0; c < n_cls && ci < 0; ++c)
                if (plan.cls[nc + c].lk2 == f_lk2[f] && plan.cls[nc + c].beta == f_beta[f]) ci = c;
            if (ci < 0) {
                ci = n_cls++;
                ClassDesc &cd = plan.cls[nc + ci];
                cd.lk2 = (uint8_t)f_lk2[f];
                cd.beta = (uint8_t)f_beta[f];
                for (int k = 0; k < kMR; ++k) cd.q[k] = kNone;
            }
            ClassDesc &cd = plan.cls[nc + ci];
            if (cd.q[f_mr[f]] == kNone) cd.q[f_mr[f]] = (uint16_t)nq++;
            map.idx[f] = cd.q[f_mr[f]];
        }
        gd.n_cls = (uint8_t)n_cls;
        nc += n_cls;
    }
    plan.n_group = ng;
    plan.n_quant = nq;
}

// The lane-partial array needs (n_quant + 1) KiB of LDS; allow the full 160 KiB once.
template <typename T>
int sweep_lds_ok(size_t bytes)
{
    static int state = 0;  // 0 unknown, 1 ok, -1 failed
    if (bytes <= 64 * 1024) return 1;
    if (state == 0)
        state = hipFuncSetAttribute((const void *)sweep_kernel<T>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)((kChunk + 1) * kSweepThreads * sizeof(float))) ==
                        hipSuccess
                    ? 1
                    : -1;
    return state;
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
        const size_t lds = (size_t)(nq + 1) * kSweepThreads * sizeof(float);
        if ((dtype == BDR_F32 ? sweep_lds_ok<float>(lds) : sweep_lds_ok<uint16_t>(lds)) < 0)
            return BDR_ERR_LAUNCH;
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
