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
// Range: squares of FP32 numbers underflow for small tensors and overflow for large
// ones, so a workgroup works on x * 2^s with s chosen from the largest exponent it
// has met so far (found in the registers of each iteration's loads: no pass over the
// tensor beforehand) and undoes the scale, exactly, whenever it folds its FP32
// partials into FP64; when a larger exponent turns up, the partials are folded at the
// old scale first.  Scaling by a power of two commutes with the quantizer (end of
// Sec. IX), so nothing changes except for values more than 126 binades below the
// largest one the workgroup has seen, whose contribution is below 2^-250 of either
// sum.
//
// Sums: every lane keeps one FP32 partial per quantizer in LDS; after at most
// 256 elements per lane the partials are folded, in a fixed order, into FP64
// sums held by the workgroup, and workgroups are combined in FP64 in a fixed
// order as well, so results are reproducible.
#include <atomic>

#include "bdr_device.hpp"
#include "bdr_internal.hpp"

namespace bdr {

namespace {

constexpr int kSweepThreads = 256;
constexpr int kG = 2;  // groups of 8 elements per lane per iteration
// Three resident workgroups per compute unit (64 formats x 2^24 values: 512 workgroups 0.099 ms, 768
// 0.086, 1024 0.096, 1536 0.088).
constexpr int kSweepBlocks = 768;

constexpr int kChunk = 128;  // formats per launch: bounds kernel arguments (< 4 KiB) and LDS
constexpr int kMaxGroups = kChunk;
constexpr int kMaxClasses = kChunk;
constexpr int kMR = 2;       // (m, rounding) pairs evaluated together in a group that selects
constexpr int kMRd = 8;      // ... and in a group that evaluates every class directly
constexpr size_t kHeaderBytes = 0;            // the workspace holds the FP64 partials and nothing else
constexpr int kFoldPasses = (kChunk + 1 + 31) / 32;  // quantizers + signal, 32 per pass
constexpr int kFoldEvery = 256 / (8 * kG);           // iterations between folds: 256 elements per lane

// Both descriptors are sized and aligned so that a wave fetches one with a single
// scalar load.
struct alignas(16) GroupDesc {
    uint8_t lk1;       // log2 k1
    uint8_t shared;    // 1: all classes have beta <= 1 and select between two candidates
    uint8_t n_mr;      // (m, rounding) pairs in use (<= kMR when shared, else <= kMRd)
    uint8_t n_cls;     // classes of this group
    uint16_t first;    // index of its first class
    uint8_t mr[kMRd];  // m in the low nibble, rounding in the high one
    __host__ __device__ int m(int r) const { return mr[r] & 15; }
    __host__ __device__ int rnd(int r) const { return mr[r] >> 4; }
};
struct alignas(8) ClassDesc {
    uint8_t lk2, beta;   // log2 k2, 2^d2 - 1
    uint8_t mask;        // bit r: some format asks for (this class, mr r)
    uint8_t pad;
    uint16_t base;       // accumulators of the requested pairs follow each other from here
    uint16_t q1;         // accumulator of pair 1 (base, or base + 1 when pair 0 is requested too)
    __host__ __device__ bool wants(int r) const { return (mask >> r) & 1; }
    __host__ __device__ int q(int r) const { return base + __builtin_popcount(mask & ((1u << r) - 1u)); }
    __host__ __device__ int q01(int r) const { return r == 0 ? base : q1; }  // r < 2
};
static_assert(sizeof(GroupDesc) == 16 && sizeof(ClassDesc) == 8, "descriptor sizes");
struct SweepPlan {
    int32_t n_group, n_quant;
    GroupDesc grp[kMaxGroups];
    ClassDesc cls[kMaxClasses + 1];  // one past the end may be read ahead
};
struct FormatMap {
    uint16_t idx[kChunk];  // format -> quantizer
};

// Maxima over aligned groups for one run of 8 elements of a lane:
//   p1, p2   magnitudes (held to the normal range) of the pairs and runs of 4
//   w[0..1]  scaling exponents 127 - e, as signed bytes (range [-127, 126]), of
//            the groups of 8, 16, 32, 64 (w[0]) and 128, 256 (w[1]) the lane is in
struct Levels {
    uint32_t p1[4], p2[2];
    uint32_t w[2];
};

__device__ __forceinline__ uint32_t neg_exp_byte(uint32_t mag) { return (127u - (mag >> 23)) & 0xffu; }

__device__ __forceinline__ uint32_t pack4(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    return a | (b << 8) | (c << 16) | (d << 24);
}

__device__ __forceinline__ void build_levels(const uint32_t (&ab)[8], uint32_t mag_lo, Levels &L)
{
    uint32_t p0[8], pl[6];
    uint32_t(&p1)[4] = L.p1;
    uint32_t(&p2)[2] = L.p2;
#pragma unroll
    for (int i = 0; i < 8; ++i) p0[i] = ab[i];
#pragma unroll
    for (int i = 0; i < 4; ++i) p1[i] = umax(p0[2 * i], p0[2 * i + 1]);
    // holding a maximum to the range is the same as holding each element to it
#pragma unroll
    for (int i = 0; i < 4; ++i) p1[i] = umin(umax(p1[i], mag_lo), kMagHi);
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
    L.w[0] = pack4(neg_exp_byte(pl[0]), neg_exp_byte(pl[1]), neg_exp_byte(pl[2]), neg_exp_byte(pl[3]));
    L.w[1] = pack4(neg_exp_byte(pl[4]), neg_exp_byte(pl[5]), 0, 0);
}

// 127 - e for a group of 8 or more elements (lk >= 3): one value per lane.
__device__ __forceinline__ int lane_level(const Levels &L, int lk)
{
    const uint64_t both = ((uint64_t)L.w[1] << 32) | L.w[0];
    return (int)(int8_t)(both >> (8 * (lk - 3)));
}

// 127 - e of the level-lk group each of the 8 elements belongs to.
__device__ __forceinline__ void level_exps(const Levels &L, const uint32_t (&ab)[8],
                                           uint32_t mag_lo, int lk, int (&out)[8])
{
    if (lk == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            out[i] = 127 - (int)(umin(umax(ab[i], mag_lo), kMagHi) >> 23);
    } else if (lk == 1) {
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = 127 - (int)(L.p1[i >> 1] >> 23);
    } else if (lk == 2) {
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = 127 - (int)(L.p2[i >> 2] >> 23);
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

// Both candidate differences |x| - Q(|x|) of one (m, rounding) for a lane whose 8
// elements share the block exponent: d0 with the block exponent as it is, d1 with
// it lowered by one.  cb = 127 - E_block.  Nearest-even works on |x| directly with
// the clamp value and the rounding constant moved to the block's scale (their
// exponent fields lowered by cb resp. cb + 1; a field that would fall below 1
// belongs to a candidate that no element selects, see the caller).
template <int ROUNDING>
__device__ __forceinline__ void candidates(const float (&ax)[8], int cb, const MrConst &c,
                                           float (&d0)[8], float (&d1)[8])
{
    if (ROUNDING == BDR_RNE) {
        const uint32_t dn = (uint32_t)cb << 23;
        const uint32_t top0 = as_u(c.top) - dn, top1 = top0 - (1u << 23);
        const float mg0 = as_f(as_u(c.magic) - dn), mg1 = as_f(as_u(c.magic) - dn - (1u << 23));
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float y0 = as_f(umin(as_u(ax[i]), top0));
            const float y1 = as_f(umin(as_u(ax[i]), top1));
            d0[i] = ax[i] - ((y0 + mg0) - mg0);
            d1[i] = ax[i] - ((y1 + mg1) - mg1);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float y0 = __builtin_ldexpf(ax[i], cb);
            d0[i] = __builtin_ldexpf(quant_diff<ROUNDING>(y0, c), -cb);
            d1[i] = __builtin_ldexpf(quant_diff<ROUNDING>(y0 + y0, c), -cb - 1);
        }
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

// ALL_RNE: every format of the launch rounds to nearest even (the usual case);
// the other two modes are then compiled out.
template <typename T, bool ALL_RNE, bool WIDE>
__global__ __launch_bounds__(kSweepThreads, 3) void sweep_kernel(
    SweepPlan plan, const T *__restrict__ x, int64_t cols, int64_t ld, int64_t n_groups,
    double *__restrict__ partials)
{
    extern __shared__ float s_lane[];  // [n_quant + 1][kSweepThreads]: one partial per lane
    __shared__ int s_wsref[kSweepThreads / 64];
    const int nq = plan.n_quant;
    const int tid = threadIdx.x, lane = tid & 63;
    for (int q = 0; q <= nq; ++q) s_lane[q * kSweepThreads + tid] = 0.f;
    if (tid < kSweepThreads / 64) s_wsref[tid] = 0;
    __syncthreads();
    auto add_to = [&](int q, float v) { s_lane[q * kSweepThreads + tid] += v; };

    // The FP32 work of a wave is done on x * 2^sref, sref = 127 - eref, where eref is the
    // exponent of the largest magnitude the wave has met so far (so that it lands in [1, 2) and
    // squares neither overflow nor lose more than they would at the tensor's own scale; scaling
    // by a power of two commutes with the quantizer, end of Sec. IX).  When an iteration brings
    // a larger one, the wave moves its lanes' partials to the new scale (a power of two:
    // exact).  The fold takes every wave's partials back to the tensor's own scale, so the FP64
    // sums are unscaled.  No pass over the tensor is needed beforehand, and no barrier here.
    int eref = 0, sref = 0;
    uint32_t mag_lo = 0;  // the lowest exponent an element can carry (code 1 before scaling)

    // Lane partials -> FP64 sums of this workgroup, 32 quantizers at a time: 8 threads
    // share a quantizer, each adds up 32 lanes (start rotated so that a wave touches
    // 64 distinct banks) and clears them, then the 8 are combined in a fixed order.
    const int part = tid & 7, slot = tid >> 3;
    const int rot = (slot & 7) + 8 * (part >> 1);
    double acc[kFoldPasses];
#pragma unroll
    for (int p = 0; p < kFoldPasses; ++p) acc[p] = 0.0;
    auto fold = [&]() {
        __syncthreads();
#pragma unroll
        for (int p = 0; p < kFoldPasses; ++p) {
            const int q = 32 * p + slot;
            if (32 * p <= nq) {  // uniform
                double v = 0.0;
                if (q <= nq) {
                    float *src = s_lane + q * kSweepThreads + part * 32;
#pragma unroll 8
                    for (int i = 0; i < 32; ++i) {
                        v += (double)src[(i + rot) & 31];
                        src[(i + rot) & 31] = 0.f;
                    }
                }
                v = __builtin_ldexp(v, -2 * s_wsref[part >> 1]);  // the 32 lanes are half of one wave; exact
                v += __shfl_xor(v, 1);
                v += __shfl_xor(v, 2);
                v += __shfl_xor(v, 4);
                acc[p] += v;
            }
        }
        __syncthreads();
    };

    int since_fold = 0;
    const int64_t per_iter = (int64_t)gridDim.x * kSweepThreads * kG;
    for (int64_t base = (int64_t)blockIdx.x * kSweepThreads * kG; base < n_groups;
         base += per_iter) {
        uint32_t xr[kG][8];
        uint32_t mx = 0;
#pragma unroll
        for (int j = 0; j < kG; ++j) {
            const int64_t g = base + (int64_t)(tid >> 6) * (64 * kG) + j * 64 + lane;
#pragma unroll
            for (int i = 0; i < 8; ++i) xr[j][i] = 0;
            if (g < n_groups) {
                const int64_t t0 = 8 * g;
                const int64_t r = ld == cols ? 0 : t0 / cols;
                load8(x + r * ld + (t0 - r * cols), xr[j]);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) mx = umax(mx, xr[j][i] & kAbsMask);
        }
        // largest magnitude of the wave's iteration (uniform across the wave: scalar registers)
        // (within rows of 16 lanes by DPP, the four rows by lane reads: no trip through LDS)
        mx = umax(mx, dpp<kQuadXor1>(mx));
        mx = umax(mx, dpp<kQuadXor2>(mx));
        mx = umax(mx, dpp<kRowHalfMirror>(mx));
        mx = umax(mx, dpp<kRowMirror>(mx));
        const uint32_t wmx = umax(umax((uint32_t)__builtin_amdgcn_readlane((int)mx, 0),
                                       (uint32_t)__builtin_amdgcn_readlane((int)mx, 16)),
                                  umax((uint32_t)__builtin_amdgcn_readlane((int)mx, 32),
                                       (uint32_t)__builtin_amdgcn_readlane((int)mx, 48)));
        const int e_it = (int)(umin(umax(wmx, kMagLo), kMagHi) >> 23);
        if (e_it > eref) {
            if (eref != 0)  // partials taken at the old scale move to the new one
                for (int q = 0; q <= nq; ++q)
                    s_lane[q * kSweepThreads + tid] =
                        __builtin_ldexpf(s_lane[q * kSweepThreads + tid], 2 * (eref - e_it));
            eref = e_it;
            sref = 127 - eref;
            mag_lo = (uint32_t)(1 + (sref > 0 ? sref : 0)) << 23;
            if (lane == 0) s_wsref[tid >> 6] = sref;  // read by the fold, after its barrier
        }
        if (since_fold == kFoldEvery) {  // same trip count for every lane of the workgroup
            fold();
            since_fold = 0;
        }
        ++since_fold;
        float ax[kG][8];
        Levels L[kG];
        float sig = 0.f;
#pragma unroll
        for (int j = 0; j < kG; ++j) {
            const uint32_t(&xb)[8] = xr[j];
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
            ClassDesc cd = plan.cls[gd.first];  // the next one is fetched while this one runs
            if (gd.shared) {
                // k1 >= 8: one block exponent per lane.  cb = 127 - E_block.
                int cb[kG];
                uint32_t thr[kG];  // elements / sub-blocks whose maximum is below 2^E_block get tau = 1
                float d0[kMR][kG][8], d1[kMR][kG][8];
#pragma unroll
                for (int j = 0; j < kG; ++j) {
                    cb[j] = lane_level(L[j], gd.lk1);
                    // E_block at the bottom of the range: no sub-block can lie below it
                    // (its own exponent is held at that bottom as well)
                    const uint32_t t = (uint32_t)(127 - cb[j]) << 23;
                    thr[j] = t > mag_lo ? t : 0u;
                }
#pragma unroll
                for (int r = 0; r < kMR; ++r) {
                    // an unused slot repeats slot 0 (the host fills it so): computing it
                    // anyway keeps the candidate arrays free of conditional definitions
                    const MrConst c = mr_const(gd.m(r), gd.rnd(r));
#pragma unroll
                    for (int j = 0; j < kG; ++j) {
                        if (ALL_RNE || c.rounding == BDR_RNE)
                            candidates<BDR_RNE>(ax[j], cb[j], c, d0[r][j], d1[r][j]);
                        else if (c.rounding == BDR_RNA)
                            candidates<BDR_RNA>(ax[j], cb[j], c, d0[r][j], d1[r][j]);
                        else
                            candidates<BDR_RTZ>(ax[j], cb[j], c, d0[r][j], d1[r][j]);
                    }
                }
                for (int ci = 0; ci < gd.n_cls; ++ci) {
                    const ClassDesc nxt = plan.cls[gd.first + ci + 1];
                    // which elements take the lowered exponent: per element, pair or run
                    // of 4 by comparing that maximum with 2^E_block, per lane above that
                    const int kind = cd.beta == 0 ? -1 : (cd.lk2 < 3 ? (int)cd.lk2 : 3);
                    auto run = [&](auto pick) {
#pragma unroll
                        for (int r = 0; r < kMR; ++r) {
                            if (cd.wants(r)) {
                                float sum = 0.f;
#pragma unroll
                                for (int j = 0; j < kG; ++j)
#pragma unroll
                                    for (int i = 0; i < 8; ++i) {
                                        const float d = pick(r, j, i);
                                        sum = __builtin_fmaf(d, d, sum);
                                    }
                                add_to(cd.q01(r), sum);
                            }
                        }
                    };
                    if (kind < 0) {
                        run([&](int r, int j, int i) { return d0[r][j][i]; });
                    } else if (kind == 0) {
                        run([&](int r, int j, int i) {
                            return as_u(ax[j][i]) < thr[j] ? d1[r][j][i] : d0[r][j][i];
                        });
                    } else if (kind == 1) {
                        run([&](int r, int j, int i) {
                            return L[j].p1[i >> 1] < thr[j] ? d1[r][j][i] : d0[r][j][i];
                        });
                    } else if (kind == 2) {
                        run([&](int r, int j, int i) {
                            return L[j].p2[i >> 2] < thr[j] ? d1[r][j][i] : d0[r][j][i];
                        });
                    } else {
                        bool dl[kG];
#pragma unroll
                        for (int j = 0; j < kG; ++j) dl[j] = lane_level(L[j], cd.lk2) > cb[j];
                        run([&](int r, int j, int i) { return dl[j] ? d1[r][j][i] : d0[r][j][i]; });
                    }
                    cd = nxt;
                }
            } else {
                for (int ci = 0; ci < gd.n_cls; ++ci) {
                    const ClassDesc nxt = plan.cls[gd.first + ci + 1];
                    // sh = 127 - max(E_block - beta, E_sub) = min(127 - E_block + beta, 127 - E_sub)
                    int sh[kG][8];
                    float yp[kG][8];
#pragma unroll
                    for (int j = 0; j < kG; ++j) {
                        int cbe[8], cs[8];
                        uint32_t ab[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) ab[i] = as_u(ax[j][i]);
                        level_exps(L[j], ab, mag_lo, gd.lk1, cbe);
                        level_exps(L[j], ab, mag_lo, cd.lk2, cs);
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            sh[j][i] = min(cbe[i] + (int)cd.beta, cs[i]);
                            yp[j][i] = __builtin_ldexpf(ax[j][i], sh[j][i]);
                        }
                    }
#pragma unroll
                    for (int r = 0; r < (WIDE ? kMRd : kMR); ++r) {
                        if (r < gd.n_mr && cd.wants(r)) {
                            const MrConst c = mr_const(gd.m(r), gd.rnd(r));
                            float sum;
                            if (ALL_RNE || c.rounding == BDR_RNE)
                                sum = direct<BDR_RNE>(yp, sh, c);
                            else if (c.rounding == BDR_RNA)
                                sum = direct<BDR_RNA>(yp, sh, c);
                            else
                                sum = direct<BDR_RTZ>(yp, sh, c);
                            add_to(cd.q(r), sum);
                        }
                    }
                    cd = nxt;
                }
            }
        }
    }
    fold();
    for (int p = 0; p < kFoldPasses; ++p) {
        const int q = 32 * p + slot;
        if (q <= nq && part == 0) partials[(int64_t)blockIdx.x * (nq + 1) + q] = acc[p];
    }
}

// One workgroup per format (plus one for the signal power alone): adds up the
// format's column and the signal column of the per-workgroup partial sums in a
// fixed order (lane i takes rows i, i + 256, ..., the 256 lane sums go through a
// fixed tree) and writes noise power and QSNR (Sec. III).
__global__ __launch_bounds__(256) void sweep_finalize_kernel(
    FormatMap map, int32_t n_fmts, int32_t n_quant, int32_t n_blocks,
    const double *__restrict__ partials, double *__restrict__ qsnr_db, double *__restrict__ sums,
    double *sig_out)
{
    __shared__ double s_e[256], s_s[256];
    const int f = blockIdx.x;
    const int col = f < n_fmts ? map.idx[f] : n_quant;
    double e = 0.0, sg = 0.0;
    for (int b = threadIdx.x; b < n_blocks; b += 256) {
        e += partials[(int64_t)b * (n_quant + 1) + col];
        sg += partials[(int64_t)b * (n_quant + 1) + n_quant];
    }
    s_e[threadIdx.x] = e;
    s_s[threadIdx.x] = sg;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            s_e[threadIdx.x] += s_e[threadIdx.x + w];
            s_s[threadIdx.x] += s_s[threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const double sig = s_s[0];
        if (f == n_fmts) {
            *sig_out = sig;
        } else {
            const double err = s_e[0];
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
    return kHeaderBytes + (size_t)kSweepBlocks * (size_t)(per_launch + 1) * sizeof(double);
}

namespace {

// Host plan for up to kChunk formats: groups of equal k1 (split so that a group
// is either all beta <= 1 or all beta >= 2 and holds at most kMR, respectively
// kMRd, (m, rounding) pairs), classes (k2, beta) inside a group with the tau = 0
// formats merged, and one accumulator per distinct (class, m, rounding).
void make_plan(const bdr_format *fmts, int n_fmts, SweepPlan &plan, FormatMap &map)
{
    int ng = 0;
    int f_group[kChunk], f_mr[kChunk], f_lk2[kChunk], f_beta[kChunk], f_cls[kChunk];
    for (int f = 0; f < n_fmts; ++f) {
        const int lk1 = ilog2(fmts[f].k1);
        int lk2 = ilog2(fmts[f].k2), beta = (1 << fmts[f].d2) - 1;
        const int m = fmts[f].m, rnd = fmts[f].rounding;
        if (beta == 0 || lk2 == lk1) {  // no sub-block shift: plain block floating point
            beta = 0;
            lk2 = lk1;
        }
        const int shared = beta <= 1 && lk1 >= 3;  // one block exponent per lane
        // a group of this k1 and kind that has this (m, rounding), else one with room for it
        int gi = -1, r = -1;
        for (int g = 0; g < ng && gi < 0; ++g) {
            const GroupDesc &gd = plan.grp[g];
            if (gd.lk1 != lk1 || gd.shared != shared) continue;
            for (int k = 0; k < gd.n_mr; ++k)
                if (gd.m(k) == m && gd.rnd(k) == rnd) {
                    gi = g;
                    r = k;
                }
        }
        for (int g = 0; g < ng && gi < 0; ++g) {
            GroupDesc &gd = plan.grp[g];
            if (gd.lk1 != lk1 || gd.shared != shared || gd.n_mr == (shared ? kMR : kMRd)) continue;
            gi = g;
            r = gd.n_mr++;
            gd.mr[r] = (uint8_t)(m | (rnd << 4));
        }
        if (gi < 0) {
            gi = ng++;
            GroupDesc &gd = plan.grp[gi];
            gd = GroupDesc{};
            gd.lk1 = (uint8_t)lk1;
            gd.shared = (uint8_t)shared;
            gd.n_mr = 1;
            for (int k = 0; k < kMRd; ++k) gd.mr[k] = (uint8_t)(m | (rnd << 4));  // unused slots repeat slot 0
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
                cd = ClassDesc{};
                cd.lk2 = (uint8_t)f_lk2[f];
                cd.beta = (uint8_t)f_beta[f];
            }
            plan.cls[nc + ci].mask |= (uint8_t)(1u << f_mr[f]);
            f_cls[f] = nc + ci;
        }
        for (int c = 0; c < n_cls; ++c) {  // accumulators: class by class, requested pairs in slot order
            plan.cls[nc + c].base = (uint16_t)nq;
            plan.cls[nc + c].q1 = (uint16_t)(nq + (plan.cls[nc + c].mask & 1));
            nq += __builtin_popcount(plan.cls[nc + c].mask);
        }
        gd.n_cls = (uint8_t)n_cls;
        nc += n_cls;
    }
    for (int f = 0; f < n_fmts; ++f) map.idx[f] = (uint16_t)plan.cls[f_cls[f]].q(f_mr[f]);
    plan.n_group = ng;
    plan.n_quant = nq;
}

// One launch of the sweep kernel.  The lane-partial array needs (n_quant + 1) KiB
// of LDS: above the default limit the kernel is allowed the full 160 KiB, once.
// dry: only make sure the launch is possible (the grant), launch nothing.
template <typename T, bool ALL_RNE, bool WIDE>
int launch_sweep_w(const SweepPlan &plan, bool dry, unsigned nb, const void *x, int64_t cols,
                   int64_t ld, int64_t n_groups, double *partials, hipStream_t s)
{
    static signed char granted[kMaxDevices];
    const size_t lds = (size_t)(plan.n_quant + 1) * kSweepThreads * sizeof(float);
    if (lds > 64 * 1024 &&
        !grant_dynamic_lds((const void *)sweep_kernel<T, ALL_RNE, WIDE>,
                           (kChunk + 1) * kSweepThreads * sizeof(float), granted))
        return BDR_ERR_LAUNCH;
    if (dry) return BDR_OK;
    hipLaunchKernelGGL((sweep_kernel<T, ALL_RNE, WIDE>), dim3(nb), dim3(kSweepThreads), lds, s, plan,
                       (const T *)x, cols, ld, n_groups, partials);
    return BDR_OK;
}

// WIDE: some directly evaluated group holds more than kMR (m, rounding) pairs.  The
// narrow kernel is kept for the plans that do not need it (its loop over the pairs is
// a quarter as long and the compiler's register assignment for the selecting path is
// better without the long one next to it).
template <typename T, bool ALL_RNE>
int launch_sweep(const SweepPlan &plan, bool dry, unsigned nb, const void *x, int64_t cols,
                 int64_t ld, int64_t n_groups, double *partials, hipStream_t s)
{
    bool wide = false;
    for (int g = 0; g < plan.n_group; ++g) wide = wide || plan.grp[g].n_mr > kMR;
    return wide ? launch_sweep_w<T, ALL_RNE, true>(plan, dry, nb, x, cols, ld, n_groups, partials, s)
                : launch_sweep_w<T, ALL_RNE, false>(plan, dry, nb, x, cols, ld, n_groups, partials, s);
}

}  // namespace

int qsnr_sweep(const bdr_format *fmts, int32_t n_fmts, const void *x, int dtype, int64_t rows,
               int64_t cols, int64_t ld, double *qsnr_db, double *sums, void *workspace,
               hipStream_t s)
{
    static_assert(sizeof(SweepPlan) + 64 < 4096, "kernel arguments must stay under 4 KiB");
    double *partials = reinterpret_cast<double *>(static_cast<char *>(workspace) + kHeaderBytes);
    const int64_t n_groups = rows * cols / 8;
    // enough workgroups to fill the chip at two per compute unit, each taking several
    // rounds of kSweepThreads * kG groups so that set-up and the final combine amortize
    const int64_t per_block = (int64_t)kSweepThreads * kG;
    int64_t nb = (n_groups + per_block - 1) / per_block;
    if (nb > kSweepBlocks) nb = kSweepBlocks;
    if (nb < 1) nb = 1;

    // Chunks of formats run one after the other on the stream and reuse the
    // partial-sum area; each launch gets its own copy of the plan by value.  The first
    // walk over the chunks builds the plans and launches nothing: it only settles whether
    // every launch of the second walk can be made (kernels that need more than 64 KiB of
    // LDS have to be given that limit once per device), so a refusal is reported before
    // anything is enqueued.
    constexpr int kMaxChunks = (1024 + kChunk - 1) / kChunk;  // the entry point takes <= 1024 formats
    SweepPlan plans[kMaxChunks];
    FormatMap maps[kMaxChunks];
    if (n_fmts > kMaxChunks * kChunk) return BDR_ERR_SHAPE;
    auto chunk_launch = [&](int c, bool dry) {
        const int32_t f0 = c * kChunk;
        const int nf = n_fmts - f0 < kChunk ? n_fmts - f0 : kChunk;
        bool all_rne = true;
        for (int f = 0; f < nf; ++f) all_rne = all_rne && fmts[f0 + f].rounding == BDR_RNE;
        const SweepPlan &plan = plans[c];
        if (dtype == BDR_F32)
            return all_rne ? launch_sweep<float, true>(plan, dry, (unsigned)nb, x, cols, ld, n_groups, partials, s)
                           : launch_sweep<float, false>(plan, dry, (unsigned)nb, x, cols, ld, n_groups, partials, s);
        return all_rne ? launch_sweep<uint16_t, true>(plan, dry, (unsigned)nb, x, cols, ld, n_groups, partials, s)
                       : launch_sweep<uint16_t, false>(plan, dry, (unsigned)nb, x, cols, ld, n_groups, partials, s);
    };
    const int n_chunks = (n_fmts + kChunk - 1) / kChunk;
    for (int c = 0; c < n_chunks; ++c) {
        const int32_t f0 = c * kChunk;
        const int nf = n_fmts - f0 < kChunk ? n_fmts - f0 : kChunk;
        plans[c] = SweepPlan{};
        maps[c] = FormatMap{};
        make_plan(fmts + f0, nf, plans[c], maps[c]);
        const int st = chunk_launch(c, true);
        if (st != BDR_OK) return st;
    }
    for (int c = 0; c < n_chunks; ++c) {
        const int32_t f0 = c * kChunk;
        const int nf = n_fmts - f0 < kChunk ? n_fmts - f0 : kChunk;
        const int st = chunk_launch(c, false);
        if (st != BDR_OK) return st;  // not reached: the first walk settled it
        hipLaunchKernelGGL(sweep_finalize_kernel, dim3((unsigned)(nf + 1)), dim3(256), 0, s, maps[c],
                           nf, plans[c].n_quant, (int32_t)nb, partials, qsnr_db + f0,
                           sums + f0, sums + n_fmts);
    }
    return launch_status();
}

// ---------------------------------------------------------------- no workspace
//
// Scratch of the entry point that takes no workspace: a fixed array in device memory
// (every GPU the library runs on holds its own copy until the process ends), large
// enough for one launch of kChunk formats; longer format lists reuse it chunk by
// chunk, exactly as they reuse a caller's workspace.  In host code the array's name
// is only a handle: its device address is looked up once per device and that
// address is what the kernels are given.
constexpr size_t kStaticScratchBytes =
    kHeaderBytes + (size_t)kSweepBlocks * (size_t)(kChunk + 1) * sizeof(double);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

size_t sweep_static_scratch_bytes() { return kStaticScratchBytes; }

int qsnr_sweep_static(const bdr_format *fmts, int32_t n_fmts, const void *x, int dtype, int64_t rows,
                      int64_t cols, int64_t ld, double *qsnr_db, double *sums, hipStream_t s)
{
    static_assert(kStaticScratchBytes % 256 == 0, "scratch size");
    static std::atomic<void *> resolved[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) {
        (void)hipGetLastError();
        return BDR_ERR_LAUNCH;
    }
    void *ptr = dev < kMaxDevices ? resolved[dev].load(std::memory_order_acquire) : nullptr;
    if (!ptr) {
        // two host threads that race here look up the same address
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return BDR_ERR_LAUNCH;
        }
        if (dev < kMaxDevices) resolved[dev].store(ptr, std::memory_order_release);
    }
    if (sweep_workspace_bytes(n_fmts) > kStaticScratchBytes) return BDR_ERR_WORKSPACE;
    return qsnr_sweep(fmts, n_fmts, x, dtype, rows, cols, ld, qsnr_db, sums, ptr, s);
}

}  // namespace bdr
