"""Seeded synthetic inputs for the FSS Gen/Eval hot path.

This module holds no arithmetic of the method itself (no PRG, no tree walk, no key
layout): it only draws the random values that key generation and evaluation take as
*arguments* -- the secret offsets alpha, the alpha-share randomness r, both parties'
root seeds and the public inputs x, and for the ReLU layer the additive shares of the
activations and the dealer's multiplication triples -- so that the CPU oracle and the HIP
library can be fed identical bytes.  Both the tests and the benchmark import it; neither the oracle nor
the HIP path does.

The paper samples alpha and the root seeds uniformly inside KeyGen (initialisation lines
of the equality and comparison KeyGen algorithms); here that sampling is lifted out into
these generators so that KeyGen is a deterministic function of its arguments.

The five workloads mirror the shapes the paper's networks produce (a ReLU after the first
convolution of a 224x224 ResNet18 has 64x112x112 activations, its 3x3 stride-2 max-pool
yields 64x56x56) with fixed-point activations that are small against 2^32, which is the
regime the Sign protocol's failure analysis (section 3.2.2) assumes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

BASE_SEED = 200604593

# name -> (kind, batch) for the five benchmark configurations
CONFIGS = {
    1: ("cmp", 16_384),
    2: ("eq", 1 << 20),
    3: ("cmp", 64 * 112 * 112),
    4: ("cmp", 64 * 56 * 56),      # per round; 8 dependent rounds
    5: ("cmp", 1 << 22),
}

FRAC_BITS = 12          # fixed-point fractional bits of the synthetic activations
MAXPOOL_ROUNDS = 8      # 3x3 window -> 9 taps -> 8 running-max comparisons
MAXPOOL_PAD = -(1 << 16)


@dataclass
class GenInputs:
    """Arguments of one batched KeyGen call (all host arrays, C-contiguous)."""
    n: int
    alpha: np.ndarray        # [B] uint32, < 2^n
    r: np.ndarray            # [B] uint32, party-0 share of alpha
    seed0: np.ndarray        # [B,16] uint8, party-0 root seed block
    seed1: np.ndarray        # [B,16] uint8, party-1 root seed block

    @property
    def batch(self) -> int:
        return int(self.alpha.shape[0])


@dataclass
class Workload:
    name: str
    kind: str                # "cmp" or "eq"
    gen: GenInputs
    x: np.ndarray            # [B] uint32 public inputs, < 2^n
    extra: Dict[str, np.ndarray] = field(default_factory=dict)


def ring_mask(n: int) -> int:
    return 0xFFFFFFFF if n == 32 else (1 << n) - 1


def uniform_ring(rng: np.random.Generator, n: int, size) -> np.ndarray:
    return rng.integers(0, 1 << n, size=size, dtype=np.uint64).astype(np.uint32)


def gen_inputs(rng: np.random.Generator, n: int, batch: int,
               alpha: Optional[np.ndarray] = None) -> GenInputs:
    """Uniform alpha (unless given), uniform r, uniform 16-byte root seeds."""
    if alpha is None:
        alpha = uniform_ring(rng, n, batch)
    alpha = np.ascontiguousarray(alpha, dtype=np.uint32)
    r = uniform_ring(rng, n, batch)
    seed0 = rng.integers(0, 256, size=(batch, 16), dtype=np.uint8)
    seed1 = rng.integers(0, 256, size=(batch, 16), dtype=np.uint8)
    return GenInputs(n=n, alpha=alpha, r=r, seed0=seed0, seed1=seed1)


def uniform_workload(kind: str, n: int, batch: int, seed: int, name: str = "uniform") -> Workload:
    """alpha and x uniform in Z_{2^n} (configurations 1 and 5)."""
    rng = np.random.default_rng(seed)
    g = gen_inputs(rng, n, batch)
    x = uniform_ring(rng, n, batch)
    return Workload(name=name, kind=kind, gen=g, x=x)


def equality_workload(n: int, batch: int, seed: int, hit_rate: float = 0.1) -> Workload:
    """x = alpha on a seeded Bernoulli(hit_rate) subset, uniform elsewhere (configuration 2)."""
    rng = np.random.default_rng(seed)
    g = gen_inputs(rng, n, batch)
    hit = rng.random(batch) < hit_rate
    x = np.where(hit, g.alpha, uniform_ring(rng, n, batch)).astype(np.uint32)
    return Workload(name="equality", kind="eq", gen=g, x=x, extra={"hit": hit})


def fixed_point_normal(rng: np.random.Generator, size, frac_bits: int = FRAC_BITS) -> np.ndarray:
    """N(0,1) activations in two's-complement fixed point, as int64 values."""
    return np.rint(rng.standard_normal(size) * float(1 << frac_bits)).astype(np.int64)


def relu_workload(batch: int, seed: int, n: int = 32, scale_bits: int = FRAC_BITS) -> Workload:
    """Masked activations x = y + alpha mod 2^n with y ~ N(0,1) in fixed point (configuration 3)."""
    rng = np.random.default_rng(seed)
    g = gen_inputs(rng, n, batch)
    y = fixed_point_normal(rng, batch, scale_bits)
    x = ((y + g.alpha.astype(np.int64)) & ring_mask(n)).astype(np.uint32)
    return Workload(name="relu", kind="cmp", gen=g, x=x, extra={"y": y})


@dataclass
class ReluInputs:
    """Per-party inputs of a shared ReLU layer: additive shares of the activations and of one
    multiplication triple per element (dealer material, like the keys): c = a * b mod 2^n."""
    y_share: tuple           # ([B] uint32, [B] uint32)
    tri_a: tuple
    tri_b: tuple
    tri_c: tuple


def additive_shares(rng: np.random.Generator, n: int, value: np.ndarray):
    m = np.uint64(ring_mask(n))
    v = value.astype(np.uint64) & m
    s0 = uniform_ring(rng, n, v.shape[0]).astype(np.uint64)
    s1 = (v - s0) & m
    return s0.astype(np.uint32), s1.astype(np.uint32)


def relu_inputs(rng: np.random.Generator, n: int, y: np.ndarray) -> ReluInputs:
    m = np.uint64(ring_mask(n))
    batch = y.shape[0]
    a = uniform_ring(rng, n, batch).astype(np.uint64)
    b = uniform_ring(rng, n, batch).astype(np.uint64)
    c = (a * b) & m
    return ReluInputs(y_share=additive_shares(rng, n, y.astype(np.int64).astype(np.uint64)),
                      tri_a=additive_shares(rng, n, a), tri_b=additive_shares(rng, n, b), tri_c=additive_shares(rng, n, c))


@dataclass
class TripleShares:
    """Additive shares of `count` multiplication triples (dealer material): c = a * b mod 2^n."""
    a: tuple
    b: tuple
    c: tuple


def triple_shares(rng: np.random.Generator, n: int, count: int) -> TripleShares:
    m = np.uint64(ring_mask(n))
    a = uniform_ring(rng, n, count).astype(np.uint64)
    b = uniform_ring(rng, n, count).astype(np.uint64)
    return TripleShares(a=additive_shares(rng, n, a), b=additive_shares(rng, n, b), c=additive_shares(rng, n, (a * b) & m))


def maxpool_taps(seed: int, channels: int = 64, hw: int = 112) -> np.ndarray:
    """[9, C*(hw/2)*(hw/2)] int64: the nine taps of every 3x3 stride-2 pad-1 window."""
    rng = np.random.default_rng(seed)
    a = fixed_point_normal(rng, (channels, hw, hw))
    p = np.full((channels, hw + 2, hw + 2), MAXPOOL_PAD, dtype=np.int64)
    p[:, 1:-1, 1:-1] = a
    out = hw // 2
    taps = []
    for dy in range(3):
        for dx in range(3):
            taps.append(p[:, dy:dy + 2 * out:2, dx:dx + 2 * out:2].reshape(-1))
    return np.stack(taps)


def maxpool_round_keys(seed: int, rnd: int, batch: int, n: int = 32) -> GenInputs:
    """Fresh KeyGen arguments for dependent round `rnd` (1..8) of configuration 4."""
    rng = np.random.default_rng([seed, rnd])
    return gen_inputs(rng, n, batch)


def config_workload(cfg: int, seed: Optional[int] = None, batch: Optional[int] = None) -> Workload:
    """The workload of benchmark configuration `cfg` (4 returns the first of its eight comparison batches only; see maxpool_*)."""
    kind, b = CONFIGS[cfg]
    if batch is not None:
        b = batch
    if seed is None:
        seed = BASE_SEED + cfg
    if cfg in (1, 5):
        return uniform_workload("cmp", 32, b, seed, name=f"config{cfg}")
    if cfg == 2:
        w = equality_workload(32, b, seed)
    elif cfg == 3:
        w = relu_workload(b, seed)
    elif cfg == 4:
        w = relu_workload(b, seed)
    else:
        raise ValueError(f"unknown configuration {cfg}")
    w.name = f"config{cfg}"
    return w


def edge_inputs(n: int) -> np.ndarray:
    """Offsets at the ends and the middle of the ring (degenerate special paths)."""
    top = ring_mask(n)
    half = 1 << (n - 1)
    vals = [0, 1, half - 1, half, top - 1, top]
    return np.array(sorted(set(v & top for v in vals)), dtype=np.uint32)
