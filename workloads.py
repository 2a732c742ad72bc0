"""Seeded synthetic workloads for the parameter-exchange path.

This module only describes shapes and draws random inputs.  It holds none of
the arithmetic of the exchange (no conversion, no sum, no update rule), so that
the CPU oracle and the HIP library can both be fed from it without sharing any
code of the method itself.

Shapes follow the models the paper benchmarks (Table 2: AlexNet 60,965,224,
GoogLeNet 13,378,280 and VGGNet 138,357,544 float32 parameters).  The paper
trained on ILSVRC14; gradients and weights here are Gaussian stand-ins of the
same shapes, because the exchange arithmetic only ever sees arrays.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np

# ----------------------------------------------------------------------------
# Tensor shape lists
# ----------------------------------------------------------------------------

# AlexNet in its two-tower form (Table 2: 8 parameter layers, 60,965,224
# float32 parameters).  Each layer contributes a weight tensor and a bias.
ALEXNET_SHAPES: Tuple[Tuple[str, Tuple[int, ...]], ...] = (
    ("conv1.w", (96, 3, 11, 11)), ("conv1.b", (96,)),
    ("conv2.w", (256, 48, 5, 5)), ("conv2.b", (256,)),
    ("conv3.w", (384, 256, 3, 3)), ("conv3.b", (384,)),
    ("conv4.w", (384, 192, 3, 3)), ("conv4.b", (384,)),
    ("conv5.w", (256, 192, 3, 3)), ("conv5.b", (256,)),
    ("fc6.w", (4096, 9216)), ("fc6.b", (4096,)),
    ("fc7.w", (4096, 4096)), ("fc7.b", (4096,)),
    ("fc8.w", (1000, 4096)), ("fc8.b", (1000,)),
)
ALEXNET_PARAMS = 60_965_224  # Table 2

# Thirteen 3x3 convolutions plus three fully connected layers sum to the VGGNet
# count of Table 2 (138,357,544).  The table's depth column says 19, but its
# parameter count is that of the 16-layer network; the count is what the
# exchange sees, so the 16-layer list is used.
_VGG_CONV = ((64, 3), (64, 64), (128, 64), (128, 128), (256, 128), (256, 256),
             (256, 256), (512, 256), (512, 512), (512, 512), (512, 512),
             (512, 512), (512, 512))
VGGNET_SHAPES: Tuple[Tuple[str, Tuple[int, ...]], ...] = tuple(
    item
    for i, (co, ci) in enumerate(_VGG_CONV)
    for item in ((f"conv{i + 1}.w", (co, ci, 3, 3)), (f"conv{i + 1}.b", (co,)))
) + (
    ("fc14.w", (4096, 25088)), ("fc14.b", (4096,)),
    ("fc15.w", (4096, 4096)), ("fc15.b", (4096,)),
    ("fc16.w", (1000, 4096)), ("fc16.b", (1000,)),
)
VGGNET_PARAMS = 138_357_544  # Table 2
GOOGLENET_PARAMS = 13_378_280  # Table 2, auxiliary classifiers included


def counts_of(shapes: Sequence[Tuple[str, Tuple[int, ...]]]) -> List[int]:
    return [int(np.prod(s)) for _, s in shapes]


def alexnet_counts() -> List[int]:
    c = counts_of(ALEXNET_SHAPES)
    assert sum(c) == ALEXNET_PARAMS
    return c


def vggnet_counts() -> List[int]:
    c = counts_of(VGGNET_SHAPES)
    assert sum(c) == VGGNET_PARAMS
    return c


def many_small_counts(seed: int, n_tensors: int = 116, total: int = 7_000_000,
                      lo: int = 64, hi: int = 400_000) -> List[int]:
    """GoogLeNet-scale stand-in: `n_tensors` sizes log-uniform in [lo, hi],
    rescaled to sum to exactly `total`.

    u_t ~ U(0,1); r_t = exp(ln lo + u_t ln(hi/lo)); n_t = max(1, floor(r_t *
    total / sum r)); the deficit left by the floors goes to the largest tensor.
    Counts come out ragged (not multiples of 4 or 8), which is the point.
    """
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0x51235]))
    u = rng.random(n_tensors)
    r = np.exp(math.log(lo) + u * math.log(hi / lo))
    n = np.maximum(1, np.floor(r * (total / r.sum()))).astype(np.int64)
    n[int(np.argmax(n))] += total - int(n.sum())
    assert int(n.sum()) == total and int(n.min()) >= 1
    return [int(x) for x in n]


def googlenet_scale_counts(seed: int, total: int = GOOGLENET_PARAMS,
                           n_tensors: int = 128) -> List[int]:
    """The paper's real GoogLeNet parameter count (Table 2) spread over a
    many-small-tensor list by the same log-uniform recipe (64 weight/bias pairs
    of the 22-layer network with its two auxiliary heads ~ 128 tensors)."""
    return many_small_counts(seed, n_tensors=n_tensors, total=total)


# ----------------------------------------------------------------------------
# Seeded draws
# ----------------------------------------------------------------------------

ROLE = {"grad": 1, "param": 2, "velocity": 3, "worker": 4, "center": 5,
        "order": 6, "misc": 7}


def _rng(seed: int, role: str, worker: int = 0, step: int = 0) -> np.random.Generator:
    return np.random.default_rng(
        np.random.SeedSequence([int(seed), ROLE[role], int(worker), int(step)]))


def gaussian_tensors(counts: Sequence[int], sigma: float, seed: int, role: str,
                     worker: int = 0, step: int = 0) -> List[np.ndarray]:
    """One float32 array per tensor, N(0, sigma^2), reproducible from
    (seed, role, worker, step).  Drawn as one stream and split, so the values
    do not depend on how the caller later groups tensors."""
    rng = _rng(seed, role, worker, step)
    total = int(sum(counts))
    flat = rng.standard_normal(total, dtype=np.float32)
    flat *= np.float32(sigma)
    out, o = [], 0
    for c in counts:
        out.append(flat[o:o + c])
        o += c
    return out


def zeros_tensors(counts: Sequence[int]) -> List[np.ndarray]:
    return [np.zeros(c, dtype=np.float32) for c in counts]


def worker_orders(seed: int, k: int, rounds: int) -> np.ndarray:
    """(rounds, k) int32: a fresh permutation of the k workers per round, the
    order in which they reach the center in the asynchronous exchange."""
    rng = _rng(seed, "order")
    return np.stack([rng.permutation(k) for _ in range(rounds)]).astype(np.int32)


def wide_range_halves(counts: Sequence[int], seed: int, worker: int) -> List[np.ndarray]:
    """float32 values that are exactly representable in binary16, with
    magnitudes log-uniform over 2^-24 .. 2^15 and random signs.  Sums of such
    values depend on the order of addition, unlike sigma=0.01 data."""
    rng = _rng(seed, "misc", worker)
    out = []
    for c in counts:
        e = rng.uniform(-24.0, 15.0, c)
        v = np.exp2(e) * rng.choice(np.array([-1.0, 1.0]), c)
        out.append(v.astype(np.float16).astype(np.float32))
    return out


# ----------------------------------------------------------------------------
# The five benchmark configurations
# ----------------------------------------------------------------------------

@dataclass(frozen=True)
class Config:
    name: str
    counts: Tuple[int, ...]
    k: int
    transfer: str            # "f32" or "f16"
    grad_sigma: float = 0.01
    param_sigma: float = 0.01
    lr: float = 0.01
    mu: float = 0.9
    wd: float = 0.0
    steps: int = 1
    alpha: float = 0.0       # elastic moving rate (async only)
    rounds: int = 0          # elastic rounds (async only)
    seed: int = 0
    extra: Dict[str, object] = field(default_factory=dict)

    @property
    def n(self) -> int:
        return int(sum(self.counts))


BASE_SEED = 20160526


def config(i: int) -> Config:
    """Configuration i in 1..5."""
    s = BASE_SEED + i
    if i == 1:
        return Config("tiny_sync_k2_f32", (1_048_576,), 2, "f32",
                      param_sigma=0.05, seed=s)
    if i == 2:
        return Config("alexnet_sync_k2_f32", tuple(alexnet_counts()), 2, "f32",
                      wd=5e-4, seed=s)
    if i == 3:
        return Config("alexnet_sync_k8_f16", tuple(alexnet_counts()), 8, "f16",
                      steps=10, seed=s)
    if i == 4:
        return Config("many_small_sync_k8_f16", tuple(many_small_counts(s)), 8,
                      "f16", seed=s)
    if i == 5:
        return Config("alexnet_easgd_k8", tuple(alexnet_counts()), 8, "f32",
                      alpha=0.5 / 8, rounds=100, seed=s)
    raise ValueError(f"no configuration {i}")


def gaussian_workers(counts: Sequence[int], sigma: float, seed: int, role: str, k: int,
                     step: int = 0, threads: int = 8) -> List[List[np.ndarray]]:
    """gaussian_tensors for workers 0..k-1, drawn concurrently (each worker has
    its own generator, so the values do not depend on the thread count)."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max(1, min(threads, k))) as ex:
        return list(ex.map(lambda w: gaussian_tensors(counts, sigma, seed, role, w, step), range(k)))
