"""The library allocates nothing, clears nothing with memset and never synchronizes, so a
sequence of its calls can be captured in a HIP graph and replayed.  Every replay, with the
program's own eager work and synchronizations in between, is checked against the eager result."""
import pytest
import torch

import paper_2302_08007_amd as B
import synth_inputs as S

pytestmark = pytest.mark.gpu


def test_calls_replay_from_a_graph():
    f = B.MX6
    rows, cols = 512, 2048
    M = N = 256
    x = torch.zeros(rows, cols, device="cuda")
    planes = B.alloc_planes(f, rows, cols)
    y = torch.empty_like(x)
    yf = torch.empty_like(x)
    fmts = [B.MX9, B.MX6, B.MX4, B.fmt(32, 4, 2, 3)]
    ws = torch.empty(B.lib.bdr_qsnr_sweep_workspace_bytes(len(fmts)), dtype=torch.uint8, device="cuda")
    out = (torch.empty(len(fmts), dtype=torch.float64, device="cuda"),
           torch.empty(len(fmts) + 1, dtype=torch.float64, device="cuda"))
    pa = B.alloc_planes(f, M, cols)
    C = torch.empty(M, N, device="cuda")
    gws = torch.empty(B.mx_gemm_workspace_bytes(M, N, cols), dtype=torch.uint8, device="cuda")
    out_s = (torch.empty(len(fmts), dtype=torch.float64, device="cuda"),
             torch.empty(len(fmts) + 1, dtype=torch.float64, device="cuda"))
    fh = B.fmt(32, 2, 1, 4)                      # a tuple with kernels compiled for it
    ph = B.alloc_planes(fh, rows, cols)
    yh = torch.empty_like(x)
    Cp = torch.empty(M, N, device="cuda")
    # the calls added for tables, operand images, BF16 results and ragged shapes
    idx = torch.randint(0, rows, (300,), device="cuda", dtype=torch.int64,
                        generator=torch.Generator(device="cuda").manual_seed(3))
    table = torch.empty(rows * B.bdr_table_row_bytes(f, cols), dtype=torch.uint8, device="cuda")
    yt = torch.empty(300, cols, device="cuda")
    ia = torch.empty(B.mx_operand_bytes(f, M, cols), dtype=torch.uint8, device="cuda")
    ib = torch.empty(B.mx_operand_bytes(f, cols, rows), dtype=torch.uint8, device="cuda")
    Co = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    i9 = torch.empty(B.mx_operand_bytes(B.MX9, M, cols, B.OPERAND_BF16), dtype=torch.uint8, device="cuda")
    C9 = torch.empty(M, N, device="cuda")
    Ct = torch.empty(cols, cols, device="cuda")
    i4 = torch.empty(B.mx_operand_bytes(B.MX4, M, cols, B.OPERAND_FP4), dtype=torch.uint8, device="cuda")
    i4t = torch.empty(B.mx_operand_bytes(B.MX4, cols, rows, B.OPERAND_FP4), dtype=torch.uint8, device="cuda")
    C4 = torch.empty(M, N, device="cuda")
    C4t = torch.empty(cols, cols, dtype=torch.bfloat16, device="cuda")
    Cb = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    xr = x[:, :1000]                             # rows with a short last block, pitched
    pr = B.alloc_planes(f, rows, 1000)
    yr = torch.zeros(rows, 1000, device="cuda")

    def work():
        B.bdr_quantize(f, x, out=planes)
        B.bdr_dequantize(f, planes, rows, cols, out=y)
        B.bdr_quantize_dequantize(f, x, out=yf)
        B.bdr_qsnr_sweep(fmts, x, workspace=ws, out=out)
        B.bdr_quantize(f, x[:M], out=pa)
        B.mx_gemm(f, f, pa, pa, M, N, cols, out=C, workspace=gws)
        B.bdr_qsnr_sweep_static(fmts, x, out_s)                     # the library's own scratch array
        B.bdr_quantize(fh, x, out=ph)
        B.bdr_dequantize(fh, ph, rows, cols, out=yh)
        B.mx_dot_pipeline(f, f, pa, pa, M, N, cols, r=256, out=Cp, workspace=gws)
        B.bdr_table_pack(f, planes, rows, cols, out=table)
        B.bdr_table_gather_dequantize(f, table, rows, cols, idx, out=yt)
        B.bdr_quantize_operand(f, x[:M], out=ia)
        B.mx_gemm_operands(f, f, ia, ia, M, N, cols, out=Co)
        B.bdr_quantize_operand(B.MX9, x[:M], image=B.OPERAND_BF16, out=i9)
        B.mx_gemm_operands(B.MX9, B.MX9, i9, i9, M, N, cols, image=B.OPERAND_BF16, out=C9)
        B.bdr_quantize_operand(f, x, axis=B.AXIS_COL, b_operand=True, out=ib)     # image of x^T [cols x rows]
        B.mx_gemm_operands(f, f, ib, ib, cols, cols, rows, out=Ct)
        B.mx_gemm(f, f, pa, pa, M, N, cols, out=Cb, workspace=gws)
        B.bdr_quantize_operand(B.MX4, x[:M], image=B.OPERAND_FP4, out=i4)
        B.mx_gemm_operands(B.MX4, B.MX4, i4, i4, M, N, cols, image=B.OPERAND_FP4, out=C4)
        B.bdr_quantize_operand(B.MX4, x, axis=B.AXIS_COL, image=B.OPERAND_FP4, out=i4t)
        B.mx_gemm_operands(B.MX4, B.MX4, i4t, i4t, cols, cols, rows, image=B.OPERAND_FP4, out=C4t)
        B.bdr_quantize(f, xr, out=pr)
        B.bdr_dequantize(f, pr, rows, 1000, out=yr)

    x.copy_(S.wide_range(rows, cols, device="cuda", seed=0, spread=3))
    work()                      # first use outside the capture (one-time kernel attributes)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        work()
    for seed in (1, 2, 3):
        x.copy_(S.wide_range(rows, cols, device="cuda", seed=seed, spread=3))
        graph.replay()
        torch.cuda.synchronize()
        every = (*planes, y, yf, out[0], out[1], C, out_s[0], out_s[1], *ph, yh, Cp, table, yt, ia, Co, ib, Ct, i9, C9,
                 Cb, i4, C4, i4t, C4t, *pr, yr)
        got = [t.clone() for t in every]
        for t in every:
            t.zero_()           # eager work of the program between replays
        work()
        torch.cuda.synchronize()
        want = every
        for a, b in zip(got, want):
            a = a.view(torch.uint8) if a.dtype != torch.uint8 else a
            b = b.view(torch.uint8) if b.dtype != torch.uint8 else b
            assert torch.equal(a, b), seed
