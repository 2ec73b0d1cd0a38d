"""Parameter presets of the five benchmark configurations (literal values).

Each preset fixes the ring degree N = 2**log2n, the ciphertext primes q (the
largest primes below 2**50 congruent to 1 mod 2N, descending), the special
key-switching primes p (the next such primes), the plaintext modulus t and the
number of ciphertext primes per key-switching digit (alpha).  The values are
written out; tests re-derive them with an independent primality test.
"""
from dataclasses import dataclass
from typing import Tuple

_B = 1 << 50


@dataclass(frozen=True)
class ParamSet:
    name: str
    log2n: int
    q: Tuple[int, ...]          # ciphertext primes, product Q
    p: Tuple[int, ...]          # special primes, product P
    t: int = 65537              # plaintext modulus (prime, t = 1 mod 2N)
    alpha: int = 1              # ciphertext primes per key-switch digit
    sigma: float = 3.2          # error standard deviation
    err_clip: int = 19          # |error| <= 6 sigma

    @property
    def n(self) -> int:
        return 1 << self.log2n

    @property
    def k(self) -> int:
        return len(self.q)

    @property
    def nsp(self) -> int:
        return len(self.p)

    @property
    def dnum(self) -> int:
        return self.k // self.alpha


_N4096 = ParamSet("n4096_k2", 12,
                  q=(_B - 16383, _B - 212991),
                  p=(_B - 417791,), alpha=1)
_N8192 = ParamSet("n8192_k3", 13,
                  q=(_B - 16383, _B - 212991, _B - 1097727),
                  p=(_B - 1490943,), alpha=1)
_N16384 = ParamSet("n16384_k6", 14,
                   q=(_B - 2162687, _B - 2850815, _B - 3014655,
                      _B - 3047423, _B - 3342335, _B - 3735551),
                   p=(_B - 4718591, _B - 5177343), alpha=2)

# C1..C5 are the five configurations the benchmark description lists.
PRESETS = {"C1": _N4096, "C2": _N8192, "C3": _N8192, "C4": _N8192,
           "C5": _N16384}


def get_params(name: str) -> ParamSet:
    return PRESETS[name]
