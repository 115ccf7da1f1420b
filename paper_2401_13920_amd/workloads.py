"""Seeded synthetic inputs for the LocMoE MoE-layer hot path.

This module only draws random numbers and rounds them to the storage dtype.  It
holds none of the method's arithmetic (no gating, routing, capacity, FFN), so the
CPU oracle's tests and the HIP path's tests can both take their inputs from it
without sharing any code of the method itself.

The paper trained on a private corpus with a trained model's activations (its
appendix on datasets); neither is public, so hidden states are stand-ins drawn
from seeded Gaussian mixtures whose cluster structure induces the expert
imbalance the paper's routing section discusses.

Everything is host NumPy ``Generator(PCG64(seed))`` with seed ``1000*cfg + k``
(k=1 tokens, 2 centres / basis, 3 home nodes, 10+e weights of expert e).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Config:
    """Shape of one workload.  Names follow the paper: n experts (here E), d hidden."""

    cfg: int          # 1-based config number
    T: int            # tokens on this GPU
    d: int            # hidden size
    E: int            # experts (the paper's n)
    N: int            # simulated nodes; expert e lives on node e // (E // N)
    h: int            # FFN inner width
    dtype: str        # storage dtype of x / send / out / y: "f32" or "bf16"
    delta: float      # benchmark delta for the capacity lower bound (Theorem 1)
    C: int            # capacity the bound gives at that delta (re-derived in tests)
    clusters: int     # mixture components (0 = not a cluster mixture)
    zipf: float       # cluster weight exponent: weight_k ~ (k+1)^-zipf


CONFIGS = {
    1: Config(1, 512, 128, 8, 2, 256, "f32", 0.2510, 32, 8, 1.0),
    2: Config(2, 8192, 1024, 16, 4, 4096, "bf16", 0.1142, 255, 16, 1.1),
    3: Config(3, 32768, 2048, 32, 4, 8192, "bf16", 0.0884, 512, 0, 0.0),
    4: Config(4, 65536, 4096, 64, 8, 16384, "bf16", 0.0650, 501, 64, 1.2),
    5: Config(5, 131072, 5120, 128, 16, 20480, "bf16", 0.0603, 498, 0, 0.0),
}

#: the measured delta the paper reports from its cosine histograms (Section 4.1)
PAPER_DELTA = 0.03
ALPHA = 0.01      # auxiliary-loss weight, Section 3.2.2
MU = 0.01         # locality-loss weight (the paper leaves it open)


def small_config(T=96, d=48, E=6, N=3, h=40, dtype="bf16", cfg=9, clusters=5, zipf=1.0,
                 delta=0.2, C=8) -> Config:
    """An arbitrary small shape (ragged tails, odd sizes) for parity tests."""
    return Config(cfg, T, d, E, N, h, dtype, delta, C, clusters, zipf)


# ----------------------------------------------------------------------------
# bf16 storage helpers (round-to-nearest-even), pure bit manipulation
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> uint16 bf16 bit patterns, round to nearest even.  Finite inputs."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> the float32 values they represent (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to what the storage dtype can hold; result is float32."""
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    raise ValueError(dtype)


def _rng(cfg: int, k: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(1000 * cfg + k))


# ----------------------------------------------------------------------------
# hidden states and home nodes
# ----------------------------------------------------------------------------
def _mixture(c: Config, T: int) -> np.ndarray:
    """K-cluster isotropic Gaussian mixture: centres ~ N(0, 4 I), unit-variance noise,
    cluster weights proportional to (k+1)^-zipf (skewed, to induce expert imbalance)."""
    centres = (2.0 * _rng(c.cfg, 2).standard_normal((c.clusters, c.d), dtype=np.float32))
    wts = (np.arange(1, c.clusters + 1, dtype=np.float64)) ** (-c.zipf)
    wts /= wts.sum()
    rng = _rng(c.cfg, 1)
    k = rng.choice(c.clusters, size=T, p=wts)
    x = rng.standard_normal((T, c.d), dtype=np.float32)
    x += centres[k]
    return x


def _lowrank(c: Config, T: int) -> np.ndarray:
    """N(0,1) noise plus a rank-32 cluster component with a wide amplitude spread, so the
    angle between a token and the gating directions varies widely (config 3)."""
    B = _rng(c.cfg, 2).standard_normal((32, c.d), dtype=np.float32)
    rng = _rng(c.cfg, 1)
    k = rng.integers(0, 32, size=T)
    a = rng.uniform(0.0, 4.0, size=T).astype(np.float32)
    x = rng.standard_normal((T, c.d), dtype=np.float32)
    x += a[:, None] * B[k]
    return x


def _adversarial(c: Config, T: int):
    """70 % of tokens sit near one of 4 expert directions (experts 0, E/4, E/2, 3E/4): unit
    noise plus a +1 shift of that expert's feature block; their home node is the hot
    expert's node with probability 0.8.  The rest is plain noise with uniform homes."""
    rng = _rng(c.cfg, 1)
    hot = rng.random(T) < 0.7
    which = rng.integers(0, 4, size=T) * (c.E // 4)
    x = rng.standard_normal((T, c.d), dtype=np.float32)
    blk = c.d // c.E
    rows = np.nonzero(hot)[0]
    for e in np.unique(which[rows]):
        r = rows[which[rows] == e]
        x[r, e * blk:(e + 1) * blk] += np.float32(1.0)
    hrng = _rng(c.cfg, 3)
    home = hrng.integers(0, c.N, size=T).astype(np.int32)
    stick = hrng.random(T) < 0.8
    sel = hot & stick
    home[sel] = (which[sel] // (c.E // c.N)).astype(np.int32)
    return x, home


def hidden_states(c: Config, T: int | None = None):
    """Returns (x, home): x float32 [T, d] already rounded to the storage dtype
    (so every value is exactly representable in it), home int32 [T] in [0, N)."""
    T = c.T if T is None else T
    if c.cfg == 5:
        x, home = _adversarial(c, T)
    else:
        x = _lowrank(c, T) if c.cfg == 3 else _mixture(c, T)
        home = _rng(c.cfg, 3).integers(0, c.N, size=T).astype(np.int32)
    # every simulated node owns at least one token (keeps the localized distribution positive)
    if T >= c.N:
        home[:c.N] = np.arange(c.N, dtype=np.int32)
    return round_to_storage(x, c.dtype), home


def upstream_grad(c: Config, T: int | None = None) -> np.ndarray:
    """dL/dy [T, d] that the layers above would hand down: N(0, 1/d) per element (unit-norm rows on
    average), float32 already rounded to the storage dtype."""
    T = c.T if T is None else T
    g = _rng(c.cfg, 7).standard_normal((T, c.d), dtype=np.float32)
    g *= np.float32(1.0 / np.sqrt(c.d))
    return round_to_storage(g, c.dtype)


def expert_to_node(c: Config) -> np.ndarray:
    """Default placement: contiguous groups of E/N experts per node."""
    return (np.arange(c.E, dtype=np.int32) // (c.E // c.N)).astype(np.int32)


# ----------------------------------------------------------------------------
# expert weights: always bf16 storage, one expert at a time
# ----------------------------------------------------------------------------
def expert_weights_bits(c: Config, e: int):
    """(W_in [h,d], W_out [d,h]) of expert e as uint16 bf16 bit patterns; iid N(0, 0.02^2).
    Orientation is Eq. 1's: W_in maps a hidden vector to the inner width (W_in . x), W_out
    maps back, both stored row-major."""
    rng = _rng(c.cfg, 10 + e)
    w_in = rng.standard_normal((c.h, c.d), dtype=np.float32)
    w_in *= np.float32(0.02)
    b_in = f32_to_bf16_bits(w_in)
    del w_in
    w_out = rng.standard_normal((c.d, c.h), dtype=np.float32)
    w_out *= np.float32(0.02)
    b_out = f32_to_bf16_bits(w_out)
    return b_in, b_out


def expert_weights(c: Config, e: int):
    """Same as :func:`expert_weights_bits` but as float32 arrays of bf16-representable values."""
    b_in, b_out = expert_weights_bits(c, e)
    return bf16_bits_to_f32(b_in), bf16_bits_to_f32(b_out)


def dense_gate_weight(c: Config) -> np.ndarray:
    """A learned dense gate weight omega [E, d] for the switch-router comparison: iid N(0, 1/d) (so that the
    gating values of unit-variance features have unit scale), float32 rounded to the storage dtype."""
    w = _rng(c.cfg, 5).standard_normal((c.E, c.d), dtype=np.float32)
    w *= np.float32(1.0 / np.sqrt(c.d))
    return round_to_storage(w, c.dtype)


def token_keys(c: Config, T: int | None = None, vocab: int = 50000) -> np.ndarray:
    """Vocabulary ids for the hash-router comparison: Zipf-like (frequent ids are much more common, as in text),
    int32 in [0, vocab)."""
    T = c.T if T is None else T
    u = _rng(c.cfg, 6).random(T)
    return np.minimum((vocab ** u - 1.0).astype(np.int64), vocab - 1).astype(np.int32)
