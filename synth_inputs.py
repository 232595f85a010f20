"""Seeded synthetic inputs for the DCT hot path (shared by the oracle tests, the
GPU parity tests and bench.py).

This module holds none of the method's arithmetic: it only draws random tensors
with the shapes and value structure of the workloads and computes the integer
keep-count k of each.  It imports neither the HIP binding nor the oracle.

The five workloads (c1..c5) stand in for the paper's data, which is not
available here: flat per-layer FC gradients (Sec. 2.1, layer-wise compression),
post-ReLU activations at a model split (Sec. 3.1 / 3.3: splits are placed after
ReLU layers, so about half the entries are exact zeros), keep fractions of
about 5 % for DCT-MP and <= 1 % for DCT-DP, and a threshold life-span L = 1000
(Sec. 3.3).

Every generator takes a torch device; the same bytes are then handed to both
sides of a comparison (the caller copies device tensors to the host for the
oracle).  CPU and GPU generators give different streams for one seed: a
comparison always uses ONE generated tensor.
"""
from __future__ import annotations

import torch

BASE_SEED = 20100889


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


# ---------------------------------------------------------------- keep counts
def ceil_frac(n: int, num: int, den: int) -> int:
    """ceil(n * num / den) in integer arithmetic."""
    return (n * num + den - 1) // den


C1_N = 1 << 20
C1_K = ceil_frac(C1_N, 1, 100)          # 10486
C2_B, C2_D = 2048, 1024
C2_K = C2_D // 20                       # 51
C3_N = 25_000_000
C3_K = ceil_frac(C3_N, 1, 1000)         # 25000
C3_DRAWS = 1000
C3_CAPACITY = 2 * C3_K
C4_ROWS, C4_DIM = 1 << 22, 64
C4_N = C4_ROWS * C4_DIM                 # 2^28
C4_K = ceil_frac(C4_N, 5, 1000)         # 1342178
C4_NZ_ROWS = (C4_ROWS * 5) // 100       # 209715
C5_B, C5_D = 65536, 4096
C5_K = C5_D // 20                       # 204


# ---------------------------------------------------------------- DP gradients
def gaussian_gradient(n: int, device, seed: int, scale: float = 1e-3) -> torch.Tensor:
    """c1: fp32 vector, i.i.d. N(0, scale^2)."""
    g = torch.randn(n, device=device, dtype=torch.float32, generator=_gen(device, seed))
    return g.mul_(scale)


def student_t3_gradient(n: int, device, seed: int, scale: float = 1e-3) -> torch.Tensor:
    """c3: fp32 vector, Student-t with 3 degrees of freedom times `scale`,
    built as z0 / sqrt((z1^2 + z2^2 + z3^2) / 3) from four normal draws."""
    gen = _gen(device, seed)
    z = torch.randn(n, device=device, dtype=torch.float32, generator=gen)
    s = torch.zeros(n, device=device, dtype=torch.float32)
    for _ in range(3):
        w = torch.randn(n, device=device, dtype=torch.float32, generator=gen)
        s.addcmul_(w, w)
        del w
    s.div_(3.0).sqrt_()
    z.div_(s).mul_(scale)
    return z


def embedding_gradient(rows: int, dim: int, nz_rows: int, device, seed: int) -> torch.Tensor:
    """c4: flattened fp32 table of `rows` x `dim`; exactly `nz_rows` distinct rows
    (the head of a seeded permutation) hold N(0,1) values, every other row is
    exactly zero."""
    gen = _gen(device, seed)
    table = torch.zeros(rows, dim, device=device, dtype=torch.float32)
    picked = torch.randperm(rows, device=device, generator=gen)[:nz_rows]
    vals = torch.randn(nz_rows, dim, device=device, dtype=torch.float32, generator=gen)
    table[picked] = vals
    return table.view(-1)


# ---------------------------------------------------------------- MP matrices
def relu_activations(b: int, d: int, device, seed: int, dtype=torch.float32,
                     row_stride: int | None = None) -> torch.Tensor:
    """c2 / c5: post-ReLU activations, each entry 0 w.p. 1/2 else |N(0,1)|,
    rounded to `dtype` (round-to-nearest-even for bf16).  With row_stride > d the
    result is a [b, d] view into a [b, row_stride] buffer whose padding holds
    large values that must never be selected."""
    x = torch.randn(b, d, device=device, dtype=torch.float32, generator=_gen(device, seed))
    x = torch.relu_(x).to(dtype)
    if row_stride is None or row_stride == d:
        return x
    buf = torch.full((b, row_stride), 1.0e4, device=device, dtype=dtype)
    buf[:, :d] = x
    return buf[:, :d]


def normal_matrix(b: int, d: int, device, seed: int, dtype=torch.float32,
                  row_stride: int | None = None) -> torch.Tensor:
    """c2 / c5: upstream gradient X_grad, i.i.d. N(0,1), rounded to `dtype`."""
    x = torch.randn(b, d, device=device, dtype=torch.float32, generator=_gen(device, seed)).to(dtype)
    if row_stride is None or row_stride == d:
        return x
    buf = torch.full((b, row_stride), -7.0, device=device, dtype=dtype)
    buf[:, :d] = x
    return buf[:, :d]


# ---------------------------------------------------------------- the five configs
def config_c1(device):
    return gaussian_gradient(C1_N, device, BASE_SEED + 1), C1_K


def config_c2(device):
    x = relu_activations(C2_B, C2_D, device, BASE_SEED + 2)
    dy = normal_matrix(C2_B, C2_D, device, BASE_SEED + 2 + 500)
    return x, dy, C2_K


def config_c3_draw(device, j: int, n: int = C3_N):
    """Draw j of c3 (j = 0 selects the threshold, j = 1..1000 are compacted)."""
    return student_t3_gradient(n, device, BASE_SEED + 3000 + j)


def config_c4(device, rows: int = C4_ROWS):
    nz = (rows * 5) // 100
    n = rows * C4_DIM
    return embedding_gradient(rows, C4_DIM, nz, device, BASE_SEED + 4), ceil_frac(n, 5, 1000)


def config_c5(device, b: int = C5_B):
    x = relu_activations(b, C5_D, device, BASE_SEED + 5, dtype=torch.bfloat16)
    dy = normal_matrix(b, C5_D, device, BASE_SEED + 5 + 500, dtype=torch.bfloat16)
    return x, dy, C5_K


# ---------------------------------------------------------------- residuals (error feedback)
def residual_vector(n: int, device, seed: int, scale: float = 1e-3, clip: float = 2.0) -> torch.Tensor:
    """A residual E_grad as it looks in steady state: what earlier iterations
    dropped, i.e. values below the threshold.  N(0, scale^2) clipped to
    +-clip*scale (about the 1 % threshold of a N(0, scale^2) gradient)."""
    e = torch.randn(n, device=device, dtype=torch.float32, generator=_gen(device, seed))
    return e.clamp_(-clip, clip).mul_(scale)


def error_feedback_pairs(n: int, device, seed: int):
    """(name, g, e) fp32 pairs whose SUM is awkward: cancellation to exact zeros,
    exponents far apart, denormal sums, many exactly equal sums."""
    gen = _gen(device, seed)
    g = torch.randn(n, device=device, generator=gen)
    out = [("normal", g * 1e-3, residual_vector(n, device, seed + 1))]
    steps = torch.randint(-2, 3, (n,), device=device, generator=gen).float() * 2.0 ** -20
    out.append(("cancelling", g, steps - g))
    ex_g = torch.randint(-40, 40, (n,), device=device, generator=gen).float()
    ex_e = torch.randint(-40, 40, (n,), device=device, generator=gen).float()
    out.append(("wide_exponents", g * torch.exp2(ex_g), torch.randn(n, device=device, generator=gen) * torch.exp2(ex_e)))
    den_g = torch.randint(1, 1 << 22, (n,), device=device, generator=gen, dtype=torch.int32).view(torch.float32)
    den_e = torch.randint(0, 1 << 22, (n,), device=device, generator=gen, dtype=torch.int32).view(torch.float32)
    sign = torch.where(torch.rand(n, device=device, generator=gen) < 0.5, -1.0, 1.0)
    out.append(("denormals", den_g * sign, den_e))
    q_g = torch.randint(-3, 4, (n,), device=device, generator=gen).float() * 0.25
    q_e = torch.randint(-3, 4, (n,), device=device, generator=gen).float() * 0.25
    out.append(("quantised_ties", q_g, q_e))
    out.append(("zero_residual", g * 1e-3, torch.zeros(n, device=device)))
    return [(name, a.contiguous(), b.contiguous()) for name, a, b in out]


# ---------------------------------------------------------------- adversarial sets
def adversarial_vectors(n: int, device, seed: int):
    """Tie-heavy and special-value fp32 vectors of length n, as (name, tensor)."""
    gen = _gen(device, seed)
    out = []
    out.append(("all_equal", torch.full((n,), 0.75, device=device)))
    out.append(("all_zero", torch.zeros(n, device=device)))
    sign = torch.where(torch.arange(n, device=device) % 2 == 0, 1.0, -1.0)
    out.append(("alternating_sign", sign * 3.0))
    few = torch.randint(0, 4, (n,), device=device, generator=gen).float() * 0.5
    fsign = torch.where(torch.rand(n, device=device, generator=gen) < 0.5, -1.0, 1.0)
    out.append(("few_distinct", few * fsign))
    pz = torch.zeros(n, device=device)
    pz[::3] = -0.0
    pz[1::5] = 1.0
    out.append(("signed_zeros", pz))
    den = torch.randint(1, 1 << 20, (n,), device=device, generator=gen, dtype=torch.int32)
    out.append(("denormals", den.view(torch.float32) * fsign))
    sp = torch.randn(n, device=device, generator=gen)
    if n >= 8:
        sp[1] = float("inf")
        sp[n // 2] = float("-inf")
        sp[n - 2] = float("inf")
    out.append(("infinities", sp))
    out.append(("permutation", (torch.randperm(n, device=device, generator=gen) + 1).float() * fsign))
    return out
