"""Seeded synthetic inputs shaped like the paper's training runs.

This module only draws random tensors; it contains none of the optimizer's
arithmetic, so both the HIP path and the CPU oracle can be fed from it.  The
recipes stand in for the gradients of the paper's runs (Section 5: ViT on
CIFAR-10 / ImageNet, GPT2++ on OpenWebText), whose datasets are not available:
sizes, worker counts and hyper-parameters follow those runs, values are drawn
from fixed distributions with fixed seeds.

Seeding: the tensor of worker ``i`` at step ``t`` is drawn from a generator
seeded with ``seed + 1000*t + i`` on the device it is asked for; initial
weights use ``seed - 1``.  A CPU generator and a GPU generator give different
bits for the same seed, so a parity test draws once (on one device) and hands
the very same values to both sides.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional, Sequence, Tuple

import torch

VOTE = 0
AVG = 1
BASE_SEED = 20240400


@dataclass(frozen=True)
class Workload:
    name: str
    d: int                      # total coordinates (sum over tensors for a tensor list)
    N: int                      # workers
    mode: int                   # VOTE / AVG
    g_dtype: torch.dtype
    g_dist: str                 # "normal" | "student_t3" | "normal_outliers"
    g_scale: float
    beta1: float = 0.9
    beta2: float = 0.99
    lr: float = 1e-4
    lam: float = 0.1
    steps: int = 10
    shapes: Optional[Tuple[Tuple[int, ...], ...]] = None    # tensor list, else one flat buffer
    seed: int = BASE_SEED
    note: str = ""

    def numels(self) -> List[int]:
        if self.shapes is None:
            return [self.d]
        out = []
        for s in self.shapes:
            n = 1
            for k in s:
                n *= k
            out.append(n)
        return out


def vit_b16_shapes() -> Tuple[Tuple[int, ...], ...]:
    """ViT-B/16-shaped tensor list: 12 blocks of attention + MLP weights with their bias and
    norm vectors, a [768, 768] patch embedding with bias, and the final norm."""
    shapes: List[Tuple[int, ...]] = [(768, 768), (768,)]             # patch embedding
    for _ in range(12):
        shapes += [
            (768,), (768,),                 # norm 1 weight, bias
            (2304, 768), (2304,),           # qkv
            (768, 768), (768,),             # attention projection
            (768,), (768,),                 # norm 2 weight, bias
            (3072, 768), (3072,),           # mlp in
            (768, 3072), (768,),            # mlp out
        ]
    shapes += [(768,), (768,)]                                       # final norm
    return tuple(shapes)


def _vit_total() -> int:
    w = Workload("tmp", 0, 1, VOTE, torch.float32, "normal", 1.0, shapes=vit_b16_shapes())
    return sum(w.numels())


CONFIGS = {
    # small case the oracle finishes in seconds; d is not a multiple of 64
    "tiny": Workload("tiny", 1_000_003, 4, VOTE, torch.float32, "normal", 1.0,
                     lr=1e-4, lam=0.1, steps=10),
    # GPT-2-small-sized flat buffer, averaging, heavy-tailed bf16 gradients -- the benchmark line
    "gpt2s_avg8": Workload("gpt2s_avg8", 124_000_000, 8, AVG, torch.bfloat16, "student_t3", 1e-3,
                           lr=3e-4, lam=0.1, steps=20),
    # ViT-B/16 tensor list with the paper's ImageNet Lion setting for that model
    "vitb16_vote16": Workload("vitb16_vote16", _vit_total(), 16, VOTE, torch.float32, "normal", 1e-3,
                              lr=1e-4, lam=10.0, steps=10, shapes=vit_b16_shapes()),
    # GPT2++ 350M with 32 workers (the paper's OpenWebText setting), bf16 with outliers
    "gpt350m_vote32": Workload("gpt350m_vote32", 350_000_000, 32, VOTE, torch.bfloat16, "normal_outliers",
                               1e-3, lr=9e-5, lam=1.0, steps=10),
    "gpt350m_avg32": Workload("gpt350m_avg32", 350_000_000, 32, AVG, torch.bfloat16, "normal_outliers",
                              1e-3, lr=9e-5, lam=1.0, steps=10),
    # large-model stress
    "stress1p3b_vote8": Workload("stress1p3b_vote8", 1_300_000_000, 8, VOTE, torch.bfloat16, "normal", 1e-3,
                                 lr=1e-4, lam=0.1, steps=10),
    # vote-only pass over pre-packed random sign streams
    "packed256_1b": Workload("packed256_1b", 1_000_000_000, 256, VOTE, torch.float32, "packed_bernoulli", 0.5,
                             lr=1e-4, lam=0.1, steps=1),
}


def scaled(w: Workload, d: int, **kw) -> Workload:
    """Same recipe at a smaller flat size (for cases the CPU oracle runs in full)."""
    return replace(w, d=d, shapes=None, name=f"{w.name}@d={d}", **kw)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def draw(dist: str, scale: float, n: int, gen: torch.Generator, device) -> torch.Tensor:
    """fp32 draws of one recipe."""
    if dist == "normal":
        return torch.randn(n, generator=gen, device=device, dtype=torch.float32) * scale
    if dist == "student_t3":
        z = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
        chi = torch.zeros(n, device=device, dtype=torch.float32)
        for _ in range(3):
            y = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
            chi.addcmul_(y, y)
        return z / torch.sqrt(chi / 3.0) * scale
    if dist == "normal_outliers":
        z = torch.randn(n, generator=gen, device=device, dtype=torch.float32) * scale
        u = torch.rand(n, generator=gen, device=device, dtype=torch.float32)
        return torch.where(u < 0.01, z * 100.0, z)
    raise ValueError(dist)


def init_x(w: Workload, device, numel: Optional[int] = None, tensor: int = 0) -> torch.Tensor:
    """Initial weights N(0, 0.02^2) for one tensor (the flat buffer if there is no list)."""
    n = w.numels()[tensor] if numel is None else numel
    return torch.randn(n, generator=_gen(device, w.seed - 1 - tensor), device=device, dtype=torch.float32) * 0.02


def padded_stride(numel: int) -> int:
    """Row stride (elements) that starts every worker's row of a flat buffer on a 1 KB boundary of the
    fp32 momentum (512 B of bf16 gradients): the layout the library's header names as its fastest."""
    return (numel + 255) // 256 * 256


def init_m(w: Workload, device, numel: Optional[int] = None, row_stride: Optional[int] = None) -> torch.Tensor:
    """Momentum starts at zero (Algorithm 1, initialisation); ``[N, numel]`` view of padded rows."""
    n = w.d if numel is None else numel
    rs = n if row_stride is None else row_stride
    buf = torch.zeros((w.N, rs), device=device, dtype=torch.float32)
    return buf[:, :n]


def make_grads(w: Workload, step: int, device, numel: Optional[int] = None, tensor: int = 0,
               out: Optional[torch.Tensor] = None, row_stride: Optional[int] = None) -> torch.Tensor:
    """Per-worker gradients of one step, ``[N, numel]`` of ``w.g_dtype`` (cast round-to-nearest-even);
    ``row_stride`` pads the rows (the values do not depend on it)."""
    n = w.numels()[tensor] if numel is None else numel
    if out is None:
        out = torch.empty((w.N, n if row_stride is None else row_stride), device=device, dtype=w.g_dtype)[:, :n]
    for i in range(w.N):
        gen = _gen(device, w.seed + 1000 * step + i + 100_000 * tensor)
        out[i].copy_(draw(w.g_dist, w.g_scale, n, gen, device))
    return out


def padded_words(W: int) -> int:
    """Row stride (uint64 words) that starts every row of packed words on a 1 KB boundary."""
    return (W + 127) // 128 * 128


def random_packed(N: int, W: int, device, seed: int = BASE_SEED, p: float = 0.5,
                  row_stride: Optional[int] = None) -> torch.Tensor:
    """``[N, W]`` int64 words whose 64 bits are iid Bernoulli(p) (p = 0.5: uniform random bits); a view of
    rows ``row_stride`` words apart if given."""
    out = torch.zeros((N, W if row_stride is None else row_stride), device=device, dtype=torch.int64)[:, :W]
    for i in range(N):
        gen = _gen(device, seed + i)
        if p == 0.5:
            lo = torch.randint(0, 1 << 32, (W,), generator=gen, device=device, dtype=torch.int64)
            hi = torch.randint(0, 1 << 32, (W,), generator=gen, device=device, dtype=torch.int64)
            out[i] = lo | (hi << 32)
        else:
            word = torch.zeros(W, device=device, dtype=torch.int64)
            for b in range(64):
                bit = (torch.rand(W, generator=gen, device=device) < p).to(torch.int64)
                word |= bit << b
            out[i] = word
    return out
