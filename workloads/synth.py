"""Seeded draws: plaintext activations, encryption randomness, stand-in residues.

All draws come from numpy's counter-based Philox generator keyed by
(seed, label...), so any consumer can reproduce any buffer independently of
the order in which other buffers were drawn.
"""
from dataclasses import dataclass
from typing import Sequence

import numpy as np

BASE_SEED = 20260208


def Stream(seed: int, *labels: int) -> np.random.Generator:
    """Independent generator for (seed, labels...)."""
    ss = np.random.SeedSequence([int(seed)] + [int(x) for x in labels])
    return np.random.Generator(np.random.Philox(ss))


def ternary_secret(g: np.random.Generator, n: int) -> np.ndarray:
    """Secret key coefficients, uniform in {-1, 0, 1}; int64[n]."""
    return g.integers(-1, 2, size=n, dtype=np.int64)


def gaussian_error(g: np.random.Generator, n: int, sigma: float = 3.2,
                   clip: int = 19) -> np.ndarray:
    """Rounded normal with standard deviation sigma, clipped to +-clip; int64[n]."""
    e = np.rint(g.normal(0.0, sigma, size=n)).astype(np.int64)
    return np.clip(e, -clip, clip)


def uniform_residues(g: np.random.Generator, primes: Sequence[int],
                     n: int) -> np.ndarray:
    """One ring element uniform modulo prod(primes), as residues uint64[len(primes)][n]."""
    out = np.empty((len(primes), n), dtype=np.uint64)
    for i, q in enumerate(primes):
        out[i] = g.integers(0, int(q), size=n, dtype=np.uint64)
    return out


def slot_values(g: np.random.Generator, n: int, lo: int, hi: int) -> np.ndarray:
    """n plaintext slot values uniform in [lo, hi); int64[n]."""
    return g.integers(lo, hi, size=n, dtype=np.int64)


def attention_activations(g: np.random.Generator, heads: int, tokens: int,
                          d: int, lo: int = -128, hi: int = 128) -> np.ndarray:
    """Quantised activations int64[heads][tokens][d], uniform in [lo, hi)."""
    return g.integers(lo, hi, size=(heads, tokens, d), dtype=np.int64)


def pseudo_ciphertexts(g: np.random.Generator, primes: Sequence[int], n: int,
                       batch: int, ncomp: int = 2) -> np.ndarray:
    """Uniform residues shaped like `batch` ciphertexts: uint64[batch][ncomp][k][n].

    A fresh RLWE ciphertext is computationally indistinguishable from a uniform
    ring pair, and every evaluator kernel's control flow and traffic are data
    independent, so these buffers time exactly like real ciphertexts.
    """
    out = np.empty((batch, ncomp, len(primes), n), dtype=np.uint64)
    for i, q in enumerate(primes):
        out[:, :, i, :] = g.integers(0, int(q), size=(batch, ncomp, n),
                                     dtype=np.uint64)
    return out


def pseudo_switch_key(g: np.random.Generator, primes_qp: Sequence[int], n: int,
                      dnum: int) -> np.ndarray:
    """Uniform residues shaped like one switching key: uint64[dnum][2][k+nsp][n]."""
    out = np.empty((dnum, 2, len(primes_qp), n), dtype=np.uint64)
    for i, q in enumerate(primes_qp):
        out[:, :, i, :] = g.integers(0, int(q), size=(dnum, 2, n),
                                     dtype=np.uint64)
    return out


@dataclass(frozen=True)
class Workload:
    """Shape of one benchmark configuration (plaintext-level description)."""
    name: str
    preset: str          # key into params.PRESETS
    seed: int
    heads: int
    d: int               # head dimension d2
    context: int         # tokens already in the encrypted cache
    steps: int = 1       # successive decode steps (cache grows by one per step)
    pairs: int = 0       # C1 only: independent ciphertext pairs
    slot_lo: int = -128
    slot_hi: int = 128


WORKLOADS = {
    # 16 independent mult+relin pairs, slots uniform in [0, t)
    "C1": Workload("C1", "C1", BASE_SEED + 0, heads=0, d=0, context=0,
                   pairs=16, slot_lo=0, slot_hi=65537),
    # one head, one K-cache ciphertext of 128 tokens
    "C2": Workload("C2", "C2", BASE_SEED + 1, heads=1, d=64, context=128),
    # prefill, 12 heads x 128 tokens
    "C3": Workload("C3", "C3", BASE_SEED + 2, heads=12, d=64, context=128),
    # full decode step at 512-token context, 12 heads
    "C4": Workload("C4", "C4", BASE_SEED + 3, heads=12, d=64, context=512),
    # scaled-up: 16 heads, N=16384, 64 steps
    "C5": Workload("C5", "C5", BASE_SEED + 4, heads=16, d=64, context=512,
                   steps=64),
}
