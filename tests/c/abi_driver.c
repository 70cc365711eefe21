/* A plain C caller of libbdr_mx.so: no Python, no PyTorch, only the HIP runtime for device
 * memory.  It runs the hot path of the library through its C ABI (packed sizes, quantize,
 * dequantize, the fused round trip, the QSNR sweep, operand images and their products) on a seeded
 * tensor and checks every byte of the three planes, every dequantized value and every product
 * against the CPU oracle, which it also calls through its C interface.  Test infrastructure: built and run by tests/test_gpu_c_abi.py. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "bdr_mx.h"
#include "bdr_ref.h"

#define CHECK_HIP(e)                                                                  \
    do {                                                                              \
        hipError_t err_ = (e);                                                        \
        if (err_ != hipSuccess) {                                                     \
            fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(err_)); \
            return 2;                                                                 \
        }                                                                             \
    } while (0)
#define CHECK_BDR(e)                                                               \
    do {                                                                           \
        int st_ = (e);                                                             \
        if (st_ != BDR_OK) {                                                       \
            fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, bdr_status_string(st_)); \
            return 3;                                                              \
        }                                                                          \
    } while (0)

/* seeded values spread over a few binades, with zeros: a 64-bit LCG, nothing of the method */
static uint64_t lcg_state = 0x2545F4914F6CDD1DULL;
static double uniform01(void)
{
    lcg_state = lcg_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (double)(lcg_state >> 11) / 9007199254740992.0;
}

static int run_format(const bdr_format *f, const bdr_ref_format *rf, int64_t rows, int64_t cols, int axis,
                      const float *x, void *dx, void *dy)
{
    size_t nc, ns, nm, rc, rs, rm;
    CHECK_BDR(bdr_packed_sizes(f, rows, cols, axis, &nc, &ns, &nm));
    if (bdr_ref_packed_sizes(rf, rows, cols, axis, &rc, &rs, &rm) != 0 || nc != rc || ns != rs || nm != rm) {
        fprintf(stderr, "packed sizes differ from the oracle's\n");
        return 4;
    }
    void *dc, *dsx, *dm;
    CHECK_HIP(hipMalloc(&dc, nc ? nc : 16));
    CHECK_HIP(hipMalloc(&dsx, ns ? ns : 16));
    CHECK_HIP(hipMalloc(&dm, nm ? nm : 16));
    CHECK_BDR(bdr_quantize(f, dx, BDR_F32, rows, cols, cols, axis, dc, dsx, dm, NULL));
    CHECK_BDR(bdr_dequantize(f, dc, dsx, dm, rows, cols, axis, dy, BDR_F32, cols, NULL));
    CHECK_HIP(hipDeviceSynchronize());

    uint8_t *codes = malloc(nc + 1), *sexp = malloc(ns + 1), *mexp = malloc(nm + 1);
    uint8_t *wc = calloc(nc + 1, 1), *ws = calloc(ns + 1, 1), *wm = calloc(nm + 1, 1);
    float *y = malloc(sizeof(float) * rows * cols), *wy = malloc(sizeof(float) * rows * cols);
    CHECK_HIP(hipMemcpy(codes, dc, nc, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(sexp, dsx, ns, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(mexp, dm, nm, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(y, dy, sizeof(float) * rows * cols, hipMemcpyDeviceToHost));
    if (bdr_ref_quantize(rf, x, 0, rows, cols, cols, axis, wc, ws, wm) != 0 ||
        bdr_ref_dequantize(rf, wc, ws, wm, rows, cols, axis, wy, 0, cols) != 0) {
        fprintf(stderr, "oracle call failed\n");
        return 4;
    }
    if (memcmp(codes, wc, nc) || memcmp(sexp, ws, ns) || memcmp(mexp, wm, nm)) {
        fprintf(stderr, "planes differ from the oracle's (m %d axis %d)\n", f->m, axis);
        return 5;
    }
    if (memcmp(y, wy, sizeof(float) * rows * cols)) {
        fprintf(stderr, "dequantized values differ from the oracle's (m %d axis %d)\n", f->m, axis);
        return 5;
    }
    /* the fused round trip gives the same bits */
    CHECK_BDR(bdr_quantize_dequantize(f, dx, dy, BDR_F32, rows, cols, cols, axis, NULL));
    CHECK_HIP(hipMemcpy(y, dy, sizeof(float) * rows * cols, hipMemcpyDeviceToHost));
    if (memcmp(y, wy, sizeof(float) * rows * cols)) {
        fprintf(stderr, "fused round trip differs (m %d axis %d)\n", f->m, axis);
        return 5;
    }
    free(codes); free(sexp); free(mexp); free(wc); free(ws); free(wm); free(y); free(wy);
    CHECK_HIP(hipFree(dc));
    CHECK_HIP(hipFree(dsx));
    CHECK_HIP(hipFree(dm));
    return 0;
}

int main(void)
{
    const int64_t rows = 384, cols = 1024;
    float *x = malloc(sizeof(float) * rows * cols);
    for (int64_t i = 0; i < rows * cols; ++i) {
        const double u = uniform01(), v = uniform01(), w = uniform01();
        const double g = sqrt(-2.0 * log(u + 1e-300)) * cos(6.283185307179586 * v); /* a normal deviate */
        x[i] = w < 0.03 ? 0.0f : (float)ldexp(g, (int)(w * 12.0) - 6);
    }
    void *dx, *dy;
    CHECK_HIP(hipSetDevice(0));
    CHECK_HIP(hipMalloc(&dx, sizeof(float) * rows * cols));
    CHECK_HIP(hipMalloc(&dy, sizeof(float) * rows * cols));
    CHECK_HIP(hipMemcpy(dx, x, sizeof(float) * rows * cols, hipMemcpyHostToDevice));

    const bdr_format fm[] = {BDR_FORMAT_MX9, BDR_FORMAT_MX6, BDR_FORMAT_MX4, {32, 8, 4, 2, 5, BDR_RNA}};
    const int nf = (int)(sizeof(fm) / sizeof(fm[0]));
    bdr_ref_format rf[4];
    for (int k = 0; k < nf; ++k) {
        /* the same six integers, in the oracle's own struct */
        rf[k].k1 = fm[k].k1; rf[k].d1 = fm[k].d1; rf[k].k2 = fm[k].k2;
        rf[k].d2 = fm[k].d2; rf[k].m = fm[k].m; rf[k].rounding = fm[k].rounding;
        for (int axis = 0; axis < 2; ++axis) {
            const int st = run_format(&fm[k], &rf[k], rows, cols, axis, x, dx, dy);
            if (st) return st;
        }
        /* a shape with a short last block */
        const int st = run_format(&fm[k], &rf[k], 37, 1000, BDR_AXIS_ROW, x, dx, dy);
        if (st) return st;
    }

    /* QSNR sweep (Sec. IV-A, Eq. 3) of the four formats against the oracle's */
    const size_t wsb = bdr_qsnr_sweep_workspace_bytes(nf);
    void *ws;
    double *dq, *dsum, q[4], s[5], wq[4], wsum[5];
    CHECK_HIP(hipMalloc(&ws, wsb));
    CHECK_HIP(hipMalloc((void **)&dq, sizeof(double) * nf));
    CHECK_HIP(hipMalloc((void **)&dsum, sizeof(double) * (nf + 1)));
    CHECK_BDR(bdr_qsnr_sweep(fm, nf, dx, BDR_F32, rows, cols, cols, dq, dsum, ws, wsb, NULL));
    CHECK_HIP(hipMemcpy(q, dq, sizeof(double) * nf, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(s, dsum, sizeof(double) * (nf + 1), hipMemcpyDeviceToHost));
    if (bdr_ref_qsnr_sweep(rf, nf, x, 0, rows, cols, cols, wq, wsum) != 0) return 4;
    for (int k = 0; k < nf; ++k)
        if (fabs(q[k] - wq[k]) > 1e-4 * fabs(wq[k]) || fabs(s[k] - wsum[k]) > 2e-5 * wsum[k]) {
            fprintf(stderr, "QSNR of format %d: %.9g dB against %.9g\n", k, q[k], wq[k]);
            return 6;
        }
    /* Products on operand images the quantizer writes itself (Sec. V: both inputs of a tensor
     * operation quantized along the reduction axis): A = the first M rows of x, B = its first N
     * rows, K = cols; few rows of A (the streaming kernel) and many (the tiled ones), each image kind.
     * Expected: the oracle's product of the oracle's planes, within 1e-4 of sum |a b|. */
    {
        const int64_t N = 256, K = cols, Ms[2] = {16, 192};
        const int kinds[3] = {BDR_OPERAND_BF16, BDR_OPERAND_FP6, BDR_OPERAND_FP4}; /* for MX9, MX6, MX4 */
        float *c = malloc(sizeof(float) * 192 * N), *want = malloc(sizeof(float) * 192 * N);
        double *absdot = malloc(sizeof(double) * 192 * N);
        int64_t *ii = malloc(sizeof(int64_t) * 192 * N), *jj = malloc(sizeof(int64_t) * 192 * N);
        void *dc, *ia, *ib;
        CHECK_HIP(hipMalloc(&dc, sizeof(float) * 192 * N));
        CHECK_HIP(hipMalloc(&ia, (size_t)192 * K * 2));
        CHECK_HIP(hipMalloc(&ib, (size_t)N * K * 2));
        for (int k = 0; k < 3; ++k) {
            size_t cb, sb, mb;
            if (bdr_ref_packed_sizes(&rf[k], rows, K, 0, &cb, &sb, &mb) != 0) return 4;
            uint8_t *pc = malloc(cb), *ps = malloc(sb), *pm = malloc(mb);
            if (bdr_ref_quantize(&rf[k], x, 0, rows, K, K, 0, pc, ps, pm) != 0) return 4;
            for (int t = 0; t < 2; ++t) {
                const int64_t M = Ms[t];
                if (mx_operand_bytes(&fm[k], M, K, kinds[k]) == 0 || mx_operand_bytes(&fm[k], M, K, kinds[k]) > (size_t)192 * K * 2)
                    return 7;
                CHECK_BDR(bdr_quantize_operand(&fm[k], dx, BDR_F32, M, K, K, BDR_AXIS_ROW, kinds[k], 0, ia, NULL));
                CHECK_BDR(bdr_quantize_operand(&fm[k], dx, BDR_F32, N, K, K, BDR_AXIS_ROW, kinds[k], 1, ib, NULL));
                CHECK_BDR(mx_gemm_operands(&fm[k], &fm[k], ia, ib, kinds[k], M, N, K, dc, BDR_F32, N, NULL));
                CHECK_HIP(hipDeviceSynchronize());
                CHECK_HIP(hipMemcpy(c, dc, sizeof(float) * M * N, hipMemcpyDeviceToHost));
                for (int64_t e = 0; e < M * N; ++e) {
                    ii[e] = e / N;
                    jj[e] = e % N;
                }
                /* rows of A and of B are rows of the same planes (blocks along K) */
                if (bdr_ref_mx_gemm_sampled(&rf[k], &rf[k], pc, ps, pm, pc, ps, pm, rows, rows, K, M * N, ii, jj, want, absdot) != 0)
                    return 4;
                for (int64_t e = 0; e < M * N; ++e)
                    if (!(fabs((double)c[e] - (double)want[e]) <= 1e-4 * absdot[e] + 1e-30)) {
                        fprintf(stderr, "product, format %d, M %ld, entry %ld: %.9g against %.9g\n", k, (long)M, (long)e,
                                (double)c[e], (double)want[e]);
                        return 8;
                    }
            }
            free(pc); free(ps); free(pm);
        }
    }
    printf("ok: %d formats, both axes, a ragged shape, the sweep (MX9 %.3f dB, MX6 %.3f dB, MX4 %.3f dB), products on "
           "operand images of every kind\n", nf, q[0], q[1], q[2]);
    return 0;
}
