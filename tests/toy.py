"""Tiny parameter sets for brute-force pins (same shape of choices as the presets)."""
from workloads.params import ParamSet

from .bruteforce import ntt_primes


def toy_params(log2n: int, k: int, nsp: int, alpha: int, below: int = 1 << 50,
               t: int = 65537) -> ParamSet:
    ps = ntt_primes(below, 2 << log2n, k + nsp)
    return ParamSet(f"toy_n{1 << log2n}_k{k}", log2n, q=tuple(ps[:k]),
                    p=tuple(ps[k:]), t=t, alpha=alpha)
