"""Seeded synthetic inputs for the tests, the smoke check and the bench.

Pure tensor generation: nothing of the quantizer's arithmetic lives here, so both the CPU
oracle's tests and the GPU library's tests may use it.  Each recipe stands in for a tensor
family of the paper's workloads (Sec. IV: Gaussian vectors for the QSNR study; Sec. II:
activations and gradients with outliers); none of the paper's datasets is used.

Every function takes ``device`` ("cpu" or "cuda") and draws from a torch.Generator seeded with
the recipe's seed on that device, so a given (recipe, shape, device) is reproducible.
"""
import torch


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def tiny(rows=4096, cols=256, device="cpu", seed=0):
    """i.i.d. N(0,1), fp32."""
    return torch.randn(rows, cols, generator=_gen(seed, device), device=device)


def bandwidth(n=1 << 28, cols=4096, device="cpu", seed=1):
    """0.02 * Student-t(3): z0 / sqrt((z1^2 + z2^2 + z3^2) / 3), fp32, shaped [n/cols, cols]."""
    g = _gen(seed, device)
    x = torch.randn(n, generator=g, device=device)
    d = torch.randn(n, generator=g, device=device).square_()
    for _ in range(2):
        d += torch.randn(n, generator=g, device=device).square_()
    x.div_(d.div_(3.0).sqrt_()).mul_(0.02)
    return x.view(n // cols, cols)


def sweep(n=1 << 24, cols=256, device="cpu", seed=2):
    """N(0,1) with 0.1% of the entries multiplied by 100 (outliers), fp32, [n/cols, cols]."""
    g = _gen(seed, device)
    x = torch.randn(n, generator=g, device=device)
    mask = torch.rand(n, generator=g, device=device) < 0.001
    x[mask] *= 100.0
    return x.view(n // cols, cols)


def design_space(vectors=16384, k=256, device="cpu", seed=5):
    """The workload of the paper's QSNR-versus-cost study (caption of the Pareto figure in
    Sec. IV): X ~ N(0, |N(0,1)|) -- Gaussian vectors whose variance is itself drawn, once per
    vector, as the magnitude of a standard normal ("variable variance" in Sec. IV-C); more than
    10K vectors.  fp32, [vectors, k]."""
    g = _gen(seed, device)
    var = torch.randn(vectors, 1, generator=g, device=device).abs()
    return torch.randn(vectors, k, generator=g, device=device) * var.sqrt()


def activation(rows=8192, cols=12288, device="cpu", seed=3):
    """N(0,1) with round(1%) of the columns scaled by 50 (channel outliers), cast to bf16."""
    g = _gen(seed, device)
    x = torch.randn(rows, cols, generator=g, device=device)
    k = int(round(0.01 * cols))
    idx = torch.randperm(cols, generator=g, device=device)[:k]
    x[:, idx] *= 50.0
    return x.to(torch.bfloat16)


def gemm_operands(M=8192, N=8192, K=8192, device="cpu", seed=4):
    """A [M x K] and B [N x K] (B already laid out along K), i.i.d. N(0,1), fp32."""
    g = _gen(seed, device)
    A = torch.randn(M, K, generator=g, device=device)
    B = torch.randn(N, K, generator=g, device=device)
    return A, B


def wide_range(rows, cols, device="cpu", seed=100, spread=6, dtype=torch.float32):
    """Edge-case mix: exponents spread over 2*spread binades, exact zeros, negative zeros."""
    g = _gen(seed, device)
    x = torch.randn(rows, cols, generator=g, device=device)
    e = torch.randint(-spread, spread + 1, (rows, cols), generator=g, device=device)
    x = torch.ldexp(x, e)
    u = torch.rand(rows, cols, generator=g, device=device)
    x[u < 0.05] = 0.0
    x[(u >= 0.05) & (u < 0.07)] = -0.0
    return x.to(dtype)
