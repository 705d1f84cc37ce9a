"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws numbers.  It holds none of the method's arithmetic (no
mixing, no gradients, no topology) and is the single piece of code that both
the CPU oracle's tests and the GPU library's tests feed from, so that both
sides see the same arrays.

All draws use ``torch.Generator(device).manual_seed(seed)``; a tensor drawn on
the GPU differs from one drawn on the CPU with the same seed, which is fine
because a test always hands the *same* tensor (or its host copy) to both sides.
The paper's own workloads (ImageNet / BERT training, tutorial regressions) are
not available; these inputs take their shapes only.

Matrices are agent-major: row i is agent i's vector.  ``ld`` is the leading
dimension in elements (row stride); the returned tensor is the ``[:, :d]`` view
of an ``(n, ld)`` allocation so rows can be padded to 128-byte multiples.
"""

import torch

RESNET50_PARAMS = 25_557_032


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def padded_ld(d, elem_bytes, align_bytes=128):
    per = align_bytes // elem_bytes
    return (d + per - 1) // per * per


def alloc_rows(n, d, dtype, device, ld=None, fill=None):
    """(n, d) view with row stride ld of a fresh allocation (zeros unless fill is None -> empty)."""
    ld = d if ld is None else ld
    base = torch.zeros((n, ld), dtype=dtype, device=device) if fill == 0 else \
        torch.empty((n, ld), dtype=dtype, device=device)
    return base[:, :d]


def uniform_rows(n, d, seed, device, lo=-1.0, hi=1.0, ld=None, dtype=torch.float32):
    out = alloc_rows(n, d, dtype, device, ld)
    g = _gen(device, seed)
    for i in range(n):                      # row by row: keeps peak memory at one row
        out[i].copy_(torch.rand(d, generator=g, device=device, dtype=torch.float32) * (hi - lo) + lo)
    return out


def normal_rows(n, d, seed, device, mean=0.0, std=1.0, ld=None, dtype=torch.float32):
    out = alloc_rows(n, d, dtype, device, ld)
    g = _gen(device, seed)
    for i in range(n):
        out[i].copy_(torch.randn(d, generator=g, device=device, dtype=torch.float32) * std + mean)
    return out


# --- configuration 1: decentralized gradient descent on least squares -------------------------
def config1_least_squares(device, n=16, m=32, d=1024):
    """A_i ~ N(0,1) (seed 101), x* ~ N(0,1) (102), b_i = A_i x* + 0.01 N(0,1) (103) formed in
    fp64 and rounded to fp32.  Returns dict(A (n,m,d), b (n,m), xstar (d,))."""
    A = torch.randn((n, m, d), generator=_gen(device, 101), device=device, dtype=torch.float32)
    xs = torch.randn((d,), generator=_gen(device, 102), device=device, dtype=torch.float32)
    noise = torch.randn((n, m), generator=_gen(device, 103), device=device, dtype=torch.float32)
    b = (torch.einsum("imd,d->im", A.double(), xs.double()) + 0.01 * noise.double()).float()
    return {"A": A.contiguous(), "b": b.contiguous(), "xstar": xs, "alpha": 1e-3, "iters": 200}


# --- configuration 2: pure averaging, static exponential graph --------------------------------
def config2_state(device, n=64, d=1 << 20, ld=None):
    return uniform_rows(n, d, 201, device, -1.0, 1.0, ld)


# --- configuration 3: dynamic one-peer exponential-2 ------------------------------------------
def config3_state(device, n=256, d=1 << 22, ld=None):
    return normal_rows(n, d, 301, device, 0.0, 1.0, ld)


# --- configuration 4: push-sum on a random directed graph -------------------------------------
CONFIG4_GRAPH_SEED = 401


def config4_state(device, n=128, d=1 << 21, ld=None):
    """X ~ N(5, std 2) (seed 402)."""
    return normal_rows(n, d, 402, device, 5.0, 2.0, ld)


# --- configuration 5: momentum SGD on a ResNet-50-sized vector, bf16 storage ------------------
def config5_centres(device, n=32, d=RESNET50_PARAMS, ld=None):
    """c_i ~ N(0,1), stored bf16 (seed 501)."""
    return normal_rows(n, d, 501, device, 0.0, 1.0, ld, dtype=torch.bfloat16)


def config5_noise(device, k, n=32, d=RESNET50_PARAMS, ld=None, out=None):
    """Step-k gradient noise e ~ N(0,1), stored bf16 (seed 510+k)."""
    if out is None:
        return normal_rows(n, d, 510 + k, device, 0.0, 1.0, ld, dtype=torch.bfloat16)
    g = _gen(device, 510 + k)
    for i in range(n):
        out[i].copy_(torch.randn(d, generator=g, device=device, dtype=torch.float32))
    return out


CONFIG5 = {"lam": 1.0, "sigma": 0.1, "alpha": 0.1, "beta": 0.9, "steps": 20}
