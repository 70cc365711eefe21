/* A plain C caller of libbdr_mx.so: no Python, no PyTorch, only the HIP runtime for device
 * memory.  It runs the hot path of the library through its C ABI (packed sizes, quantize,
 * dequantize, the fused round trip, the QSNR sweep) on a seeded tensor and checks every byte of
 * the three planes and every dequantized value against the CPU oracle, which it also calls
 * through its C interface.  Test infrastructure: built and run by tests/test_gpu_c_abi.py. */
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
    printf("ok: %d formats, both axes, a ragged shape, the sweep (MX9 %.3f dB, MX6 %.3f dB, MX4 %.3f dB)\n", nf, q[0],
           q[1], q[2]);
    return 0;
}
