"""Seeded synthetic inputs for the model-averaging step: workload table and generators.

This module holds no arithmetic of the method.  It only draws Gaussian replicas and
gradients with the shapes of the paper's workloads (flat parameter vectors of a
ResNet-50-sized and an LSTM-acoustic-model-sized network, Sec. 5.2) and hands the very
same bit patterns to whichever implementation asks.  Data is drawn in one place (host
numpy for small cases, torch's device generator for HBM-resident cases) and copied to the
other side; it is never re-derived independently, because host and device normal
generators differ in the last bits.
"""
from dataclasses import dataclass

import numpy as np

TOPO_RING = 0
TOPO_RAND_RING = 1
TOPO_FULL = 2


@dataclass(frozen=True)
class Workload:
    name: str
    n: int              # learners (rows of X)
    d: int              # parameters per learner (columns of X)
    g_dtype: str        # "f32" or "bf16"
    topology: int
    lr: float
    steps: int
    sigma_x: float
    sigma_g: float
    delay: bool = False  # delay-by-one gradient (Sec. 4, Eq. 14)
    grad_pull: float = 0.0  # c in G = c * X_{k-1} + noise for the delayed workload
    seed_x: int = 0
    seed_g: int = 0
    seed_perm: int = 0


def _wl(idx, **kw):
    return Workload(seed_x=1000 + idx, seed_g=2000 + idx, seed_perm=3000 + idx, **kw)


# The five synthetic workloads, in the order the baseline lists them.
WORKLOADS = (
    _wl(1, name="cfg1_n8_d1M_ring", n=8, d=1_000_000, g_dtype="f32", topology=TOPO_RING,
        lr=0.1, steps=10, sigma_x=1.0, sigma_g=0.01),
    _wl(2, name="cfg2_n16_d32M_randring", n=16, d=32_000_000, g_dtype="f32",
        topology=TOPO_RAND_RING, lr=0.05, steps=50, sigma_x=0.05, sigma_g=1e-3),
    _wl(3, name="cfg3_n64_d25.6M_ring_vs_rand", n=64, d=25_600_000, g_dtype="f32",
        topology=TOPO_RAND_RING, lr=0.1, steps=100, sigma_x=0.02, sigma_g=1e-3),
    _wl(4, name="cfg4_n128_d8M_d1d_randring", n=128, d=8_000_000, g_dtype="f32",
        topology=TOPO_RAND_RING, lr=0.1, steps=100, sigma_x=0.02, sigma_g=1e-3,
        delay=True, grad_pull=0.01),
    _wl(5, name="cfg5_n64_d100M_bf16g_randring", n=64, d=100_000_000, g_dtype="bf16",
        topology=TOPO_RAND_RING, lr=0.05, steps=20, sigma_x=0.02, sigma_g=1e-3),
)


def workload(idx):
    """1-based lookup (cfg 1 .. cfg 5)."""
    return WORKLOADS[idx - 1]


# ----------------------------------------------------------------------------- host side
def host_normal_f32(shape, sigma, seed):
    """N(0, sigma^2) fp32 array from numpy's Philox stream keyed by `seed`."""
    rng = np.random.Generator(np.random.Philox(seed))
    a = rng.standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(sigma)
    return a


def f32_to_bf16_bits(a):
    """Round fp32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def host_normal_bf16_bits(shape, sigma, seed):
    return f32_to_bf16_bits(host_normal_f32(shape, sigma, seed))


# --------------------------------------------------------------------------- device side
def device_normal_f32(shape, sigma, seed, device="cuda:0"):
    """N(0, sigma^2) fp32 tensor drawn in place by torch's device generator."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(0.0, sigma, generator=g)
    return t


def device_normal_bf16(shape, sigma, seed, device="cuda:0"):
    """N(0, sigma^2) drawn in fp32 and rounded once to bfloat16, one row at a time."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    t = torch.empty(shape, dtype=torch.bfloat16, device=device)
    rows = t.view(shape[0], -1)
    tmp = torch.empty(rows.shape[1], dtype=torch.float32, device=device)
    for i in range(rows.shape[0]):
        tmp.normal_(0.0, sigma, generator=g)
        rows[i].copy_(tmp)
    return t


def fill_normal_rows_(t, sigma, seed):
    """Fill an [n, d] device tensor (any row pitch, fp32 or bf16) with N(0, sigma^2) one row at
    a time, so no temporary larger than a row is needed.  bf16 rows are drawn in fp32 and
    rounded once."""
    import torch
    g = torch.Generator(device=t.device)
    g.manual_seed(seed)
    tmp = torch.empty(t.shape[1], dtype=torch.float32, device=t.device)
    for i in range(t.shape[0]):
        tmp.normal_(0.0, sigma, generator=g)
        t[i].copy_(tmp)
    return t


def bf16_tensor_bits(t):
    """uint16 bit patterns (numpy) of a bfloat16 torch tensor."""
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def sample_columns(d, count, seed):
    """Sorted distinct column indices in [0, d) for sampled full-size parity checks.

    Always includes the first and last few columns so the ragged ends are covered.
    """
    rng = np.random.Generator(np.random.Philox(seed))
    edge = np.concatenate([np.arange(min(8, d)), np.arange(max(d - 8, 0), d)])
    body = rng.integers(0, d, size=max(count - edge.size, 0), dtype=np.int64)
    return np.unique(np.concatenate([edge, body]))
