"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds none of the method's arithmetic: it only draws random
numbers with torch's generators and casts them with torch's own bf16
conversion.  It imports neither the HIP binding nor the CPU oracle, so both
can be fed the very same bytes.

The paper evaluates on LLaMA3 / Qwen3 activations over WikiText2; none of
those exist here.  What is reproduced is their shape and structure as the
paper describes it (Section 1: heavy-tailed block variances, a few outlier
channels, most mass near zero): i.i.d. Student-t entries, a small set of
outlier channels multiplied by a large factor and, optionally, a log-normal
scale per token.
"""
import math

import numpy as np
import torch

SEED_BASE = 0x70A90000


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def student_t(shape, nu: float, gen: torch.Generator, device="cpu") -> torch.Tensor:
    """Student-t(nu) = N(0,1) / sqrt(chi2(nu) / nu), chi2(nu) = 2 Gamma(nu/2)."""
    z = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    alpha = torch.full(shape, nu / 2.0, device=device, dtype=torch.float32)
    chi2 = 2.0 * torch._standard_gamma(alpha, generator=gen)
    del alpha
    return z * torch.rsqrt(chi2 / nu)


def outlier_channels(d: int, count: int, gen: torch.Generator, device="cpu") -> torch.Tensor:
    """`count` distinct channel indices, drawn before the values."""
    return torch.randperm(d, generator=gen, device=device)[:count].sort().values


def activations(M: int, d: int, *, nu: float = 3.0, outliers: int = 8, outlier_scale: float = 50.0,
                token_lognormal: bool = False, seed: int = SEED_BASE, device="cpu",
                chunk_rows: int = 4096) -> torch.Tensor:
    """bf16 tensor [M, d]: Student-t(nu) entries, `outliers` channels scaled by
    `outlier_scale`, optional per-token factor exp(N(0,1))."""
    g = _gen(seed, device)
    ch = outlier_channels(d, outliers, g, device)
    out = torch.empty((M, d), dtype=torch.bfloat16, device=device)
    for r0 in range(0, M, chunk_rows):
        r1 = min(M, r0 + chunk_rows)
        x = student_t((r1 - r0, d), nu, g, device)
        if outliers:
            x[:, ch] *= outlier_scale
        if token_lognormal:
            x *= torch.exp(torch.randn((r1 - r0, 1), generator=g, device=device))
        out[r0:r1] = x.to(torch.bfloat16)
    return out


def weights(N: int, d: int, *, std: float = 0.02, seed: int = SEED_BASE + 0x100, device="cpu",
            chunk_rows: int = 4096) -> torch.Tensor:
    """bf16 tensor [N, d] ~ N(0, std^2)."""
    g = _gen(seed, device)
    out = torch.empty((N, d), dtype=torch.bfloat16, device=device)
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        out[r0:r1] = (torch.randn((r1 - r0, d), generator=g, device=device) * std).to(torch.bfloat16)
    return out


def random_orthogonal(n: int, seed: int) -> np.ndarray:
    """Seeded random orthogonal n x n matrix: QR of a Gaussian matrix in double,
    column signs fixed so that diag(R) > 0, returned as float32."""
    rng = np.random.default_rng(int(seed))
    a = rng.standard_normal((n, n))
    q, r = np.linalg.qr(a)
    q = q * np.sign(np.diag(r))[None, :]
    return np.ascontiguousarray(q.astype(np.float32))


def rotations(G: int, seed: int = SEED_BASE + 0x200):
    """(R_inter [G, G], R_intra [32, 32]) float32."""
    return random_orthogonal(G, seed), random_orthogonal(32, seed + 1)


def default_G(d: int) -> int:
    """Size of the inter-block rotation used for feature dimension d: 128 where
    128 divides d/32, else the largest multiple of 16 that divides d/32 and is
    at most 128."""
    B = d // 32
    for G in range(128, 0, -16):
        if B % G == 0:
            return G
    raise ValueError(f"d/32 = {B} has no divisor that is a multiple of 16")


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> numpy uint16 bit patterns (host)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_bf16(a: np.ndarray, device="cpu") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)


# The named workloads (shapes and distributions of the benchmark configurations).
WORKLOADS = {
    # name: (M, d, nu, outlier fraction or count, outlier scale, token_lognormal, weight std)
    "tiny": dict(M=64, d=4096, nu=3.0, outliers=8, outlier_scale=50.0, token_lognormal=False, N=1024, wstd=0.02),
    "llama3_8b_prefill": dict(M=2048, d=4096, nu=3.0, outliers=20, outlier_scale=50.0, token_lognormal=False, N=14336, wstd=0.02),
    "qwen3_32b": dict(M=4096, d=5120, nu=3.0, outliers=26, outlier_scale=50.0, token_lognormal=True, N=25600, wstd=0.02),
    "llama3_70b_up": dict(M=8192, d=8192, nu=2.5, outliers=82, outlier_scale=100.0, token_lognormal=False, N=28672, wstd=0.01),
    "llama3_70b_down": dict(M=8192, d=28672, nu=2.5, outliers=287, outlier_scale=100.0, token_lognormal=False, N=8192, wstd=0.01),
    # the down-projection inputs of the two smaller configurations (appended: a workload's seed is its position)
    "llama3_8b_down": dict(M=2048, d=14336, nu=3.0, outliers=72, outlier_scale=50.0, token_lognormal=False, N=4096, wstd=0.02),
    "qwen3_32b_down": dict(M=4096, d=25600, nu=3.0, outliers=128, outlier_scale=50.0, token_lognormal=True, N=5120, wstd=0.02),
}


def workload_activations(name: str, device="cpu", M=None) -> torch.Tensor:
    w = WORKLOADS[name]
    idx = list(WORKLOADS).index(name)
    return activations(M if M is not None else w["M"], w["d"], nu=w["nu"], outliers=w["outliers"],
                       outlier_scale=w["outlier_scale"], token_lognormal=w["token_lognormal"],
                       seed=SEED_BASE + idx, device=device)


def workload_weights(name: str, device="cpu", N=None) -> torch.Tensor:
    w = WORKLOADS[name]
    idx = list(WORKLOADS).index(name)
    return weights(N if N is not None else w["N"], w["d"], std=w["wstd"], seed=SEED_BASE + 0x100 + idx,
                   device=device)
