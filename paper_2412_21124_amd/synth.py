"""Seeded synthetic workloads for the norm-test step.

This module only draws random inputs; it contains none of the method's
arithmetic and is the one piece of code that both the GPU tests / benchmark
and the CPU oracle tests use.  Everything is generated with a seeded
``torch.Generator`` on the requested device, in bounded chunks, so the
1.5e9-coordinate workload can be filled directly in HBM.

Workloads stand in for the gradients of the paper's language-model
pre-training runs (Sec. 5): J worker (or micro-batch, or per-sample) gradient
vectors whose common part is a fixed "signal" mu and whose worker-to-worker
part is i.i.d. noise, optionally scaled per parameter block.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional, Sequence

import torch

_CHUNK = 1 << 25  # coordinates generated per temporary


@dataclass
class Hyper:
    """Scalars of one step: AdamW (Alg. 1 Require line) and the test (eta, b_k, rounding)."""
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.1
    eta: float = 0.1
    step: int = 10
    b_k: int = 32
    b_max: int = 8192
    round_to: int = 4
    ddof: int = 1


@dataclass
class Workload:
    name: str
    J: int
    d: int
    ld: int
    grads: torch.Tensor  # (J, ld) float32 or bfloat16; columns >= d are padding
    w: torch.Tensor      # (d,) float32
    m: torch.Tensor
    v: torch.Tensor
    hyper: Hyper
    meta: dict = field(default_factory=dict)

    @property
    def grad_bytes(self) -> int:
        return self.grads.element_size()

    def algorithmic_bytes(self) -> int:
        """J gradient reads + read and write of w, m, v, per coordinate."""
        return self.d * (self.J * self.grad_bytes + 24)


def gpt2_small_blocks() -> list[int]:
    """Tensor sizes of a 12-layer, width-768, vocabulary-50257, context-1024 decoder: 148 blocks, 124,439,808 parameters."""
    width, vocab, ctx, layers = 768, 50257, 1024, 12
    per_layer = [width, width, width * 3 * width, 3 * width, width * width, width,
                 width, width, width * 4 * width, 4 * width, 4 * width * width, width]
    return [vocab * width, ctx * width] + per_layer * layers + [width, width]


def scaled_blocks(sizes: Sequence[int], d_target: int, multiple: int = 1) -> list[int]:
    """Shrink a block list to about d_target coordinates, keeping the number of blocks and their proportions."""
    total = sum(sizes)
    out = [max(multiple, int(round(s * d_target / total / multiple)) * multiple) for s in sizes]
    return out


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _state(d: int, device, gen) -> tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """w, m ~ 0.02 N(0,1); v = (0.02 N(0,1))^2 so that it is non-negative and on the scale of m^2."""
    w = torch.empty(d, dtype=torch.float32, device=device)
    m = torch.empty(d, dtype=torch.float32, device=device)
    v = torch.empty(d, dtype=torch.float32, device=device)
    for lo in range(0, d, _CHUNK):
        hi = min(d, lo + _CHUNK)
        w[lo:hi] = torch.randn(hi - lo, device=device, generator=gen) * 0.02
        m[lo:hi] = torch.randn(hi - lo, device=device, generator=gen) * 0.02
        v[lo:hi] = (torch.randn(hi - lo, device=device, generator=gen) * 0.02) ** 2
    return w, m, v


def _block_scale_vector(sizes: Sequence[int], scales: torch.Tensor, lo: int, hi: int, device) -> torch.Tensor:
    """Per-coordinate scale for coordinates [lo, hi) of a vector laid out as consecutive blocks."""
    out = torch.empty(hi - lo, dtype=torch.float32, device=device)
    pos = 0
    for size, s in zip(sizes, scales.tolist()):
        a, b = max(pos, lo), min(pos + size, hi)
        if a < b:
            out[a - lo:b - lo] = s
        pos += size
        if pos >= hi:
            break
    return out


def _fill(grads, d, mu_fn, sigma, noise, gen, device, block_sizes=None, block_scales=None):
    J = grads.shape[0]
    for lo in range(0, d, _CHUNK):
        hi = min(d, lo + _CHUNK)
        n = hi - lo
        mu = mu_fn(n)
        scale = None
        if block_sizes is not None:
            scale = _block_scale_vector(block_sizes, block_scales, lo, hi, device)
        for j in range(J):
            if noise == "normal":
                eps = torch.randn(n, device=device, generator=gen)
            elif noise == "student_t3":
                z = torch.randn(n, device=device, generator=gen)
                chi = torch.zeros(n, device=device)
                for _ in range(3):
                    chi += torch.randn(n, device=device, generator=gen) ** 2
                eps = z / torch.sqrt(chi / 3.0)
            else:
                raise ValueError(noise)
            g = mu + sigma * eps
            if scale is not None:
                g = g * scale
            grads[j, lo:hi] = g.to(grads.dtype)


def make(name: str, J: int, d: int, *, gdtype=torch.float32, sigma: float = 1e-2,
         mu: str = "normal", mu_scale: float = 1e-2, noise: str = "normal",
         block_sizes: Optional[Sequence[int]] = None, scale_range=(1e-4, 1e-1),
         hyper: Optional[Hyper] = None, seed: int = 0, device="cpu", ld: Optional[int] = None,
         with_state: bool = True) -> Workload:
    """General recipe: g_j = s_l * (mu + sigma * eps_j).

    mu = "normal": mu_i ~ N(0, mu_scale^2), fixed across j;  mu = "sign": mu_i = +-mu_scale.
    noise = "normal" or "student_t3" (unnormalised t with 3 degrees of freedom).
    block_sizes: consecutive parameter blocks, block l scaled by s_l ~ LogUniform(scale_range).
    """
    device = torch.device(device)
    gen = _gen(device, seed)
    ld = d if ld is None else ld
    if ld < d:
        raise ValueError("ld < d")
    grads = torch.zeros((J, ld), dtype=gdtype, device=device)
    scales = None
    if block_sizes is not None:
        if sum(block_sizes) != d:
            raise ValueError("block sizes must sum to d")
        lo_s, hi_s = math.log(scale_range[0]), math.log(scale_range[1])
        u = torch.rand(len(block_sizes), device=device, generator=gen)
        scales = torch.exp(lo_s + (hi_s - lo_s) * u)

    if mu == "normal":
        mu_fn = lambda n: torch.randn(n, device=device, generator=gen) * mu_scale
    elif mu == "sign":
        mu_fn = lambda n: (torch.randint(0, 2, (n,), device=device, generator=gen).float() * 2 - 1) * mu_scale
    else:
        raise ValueError(mu)
    _fill(grads, d, mu_fn, sigma, noise, gen, device, block_sizes, scales)
    if with_state:
        w, m, v = _state(d, device, gen)
    else:
        w = m = v = torch.empty(0, dtype=torch.float32, device=device)
    meta = dict(sigma=sigma, mu=mu, mu_scale=mu_scale, noise=noise, seed=seed,
                n_blocks=0 if block_sizes is None else len(block_sizes),
                block_sizes=None if block_sizes is None else list(block_sizes))
    return Workload(name, J, d, ld, grads, w, m, v, hyper or Hyper(), meta)


# ---- the five workloads -------------------------------------------------------------------

def tiny(sigma: float = 1e-2, *, d: int = 1 << 20, seed: int = 0, device="cpu", ld=None) -> Workload:
    """J=4 fp32 rows, mu_i ~ N(0, variance 1e-4); sigma 1e-3 passes the test at b_k=32, sigma 1e-2 fails it."""
    return make("tiny", 4, d, gdtype=torch.float32, sigma=sigma, mu="normal", mu_scale=1e-2,
                hyper=Hyper(lr=1e-3, step=10, b_k=32, b_max=8192, round_to=4, ddof=1),
                seed=seed, device=device, ld=ld)


def gpt2_small(ratio: float = 1.0, *, block_sizes: Optional[Sequence[int]] = None, seed: int = 0,
               device="cpu") -> Workload:
    """J=8 bf16 rows over 148 parameter blocks with log-uniform scales; |mu| = 1e-2, sigma = ratio * |mu|."""
    sizes = list(block_sizes) if block_sizes is not None else gpt2_small_blocks()
    return make("gpt2_small", 8, sum(sizes), gdtype=torch.bfloat16, sigma=ratio * 1e-2, mu="sign",
                mu_scale=1e-2, block_sizes=sizes,
                hyper=Hyper(lr=4e-4, step=10, b_k=256, b_max=8192, round_to=128, ddof=1),
                seed=seed, device=device)


def flat_1p5b(*, d: int = 1_500_000_000, J: int = 8, sigma: float = 1e-2, seed: int = 0,
              device="cpu") -> Workload:
    """The headline workload: J=8 bf16 rows of a flat 1.5e9-coordinate vector, tiny's distribution."""
    return make("flat_1p5b", J, d, gdtype=torch.bfloat16, sigma=sigma, mu="normal", mu_scale=1e-2,
                hyper=Hyper(lr=1e-3, step=10, b_k=256, b_max=8192, round_to=128, ddof=1),
                seed=seed, device=device)


def fsdp_shard(shard_id: int = 3, *, d_shard: int = 875_000_000, J: int = 16, sigma: float = 1e-2,
               seed: int = 0, device="cpu") -> Workload:
    """One of 8 parameter shards of a 7e9-parameter model with J=16 bf16 micro-batch gradients."""
    wl = make("fsdp_shard", J, d_shard, gdtype=torch.bfloat16, sigma=sigma, mu="normal", mu_scale=1e-2,
              hyper=Hyper(lr=4e-4, step=10, b_k=256, b_max=8192, round_to=128, ddof=1),
              seed=seed * 1000 + shard_id, device=device)
    wl.meta.update(shard_id=shard_id, num_shards=8, shard_offset=shard_id * d_shard, d_global=8 * d_shard)
    return wl


def per_sample(*, b: int = 512, d: int = 1 << 24, n_blocks: int = 64, seed: int = 0,
               device="cpu") -> Workload:
    """b per-example bf16 gradients with Student-t(3) noise scaled per block; statistics over samples."""
    if d % n_blocks:
        raise ValueError("d must be a multiple of n_blocks")
    return make("per_sample", b, d, gdtype=torch.bfloat16, sigma=1e-2, mu="sign", mu_scale=1e-2,
                noise="student_t3", block_sizes=[d // n_blocks] * n_blocks,
                hyper=Hyper(lr=4e-4, step=10, b_k=b, b_max=8192, round_to=1, ddof=1),
                seed=seed, device=device)


def paper_model(which: str = "1.1b", *, J: int = 4, sigma: float = 1e-2, seed: int = 0, device="cpu",
                d: Optional[int] = None) -> Workload:
    """A flat vector with the parameter count of one of the paper's models (Table 4: 304.6M, 1.1B, 3.4B) and
    J = 4 bf16 worker gradients (the data-parallel size of its runs, Tables 5-7); tiny's distribution."""
    sizes = {"300m": 304_600_000, "1.1b": 1_100_000_000, "3.4b": 3_400_000_000}
    d = sizes[which] if d is None else d
    return make("paper_" + which, J, d, gdtype=torch.bfloat16, sigma=sigma, mu="normal", mu_scale=1e-2,
                hyper=Hyper(lr=4e-4, step=10, b_k=256, b_max=8192, round_to=J * 16, ddof=1),
                seed=seed, device=device)


# ---- views for the oracle -----------------------------------------------------------------

def grads_as_numpy(grads: torch.Tensor, lo: int = 0, hi: Optional[int] = None):
    """(J, hi-lo) numpy view/copy of the gradient bits: float32, or uint16 for bfloat16."""
    hi = grads.shape[1] if hi is None else hi
    g = grads[:, lo:hi]
    if g.dtype == torch.bfloat16:
        g = g.view(torch.uint16)
    return g.cpu().numpy()
