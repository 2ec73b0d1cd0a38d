"""Pins for the oracle's arithmetic layers: primes, big integers, CRT, transforms.

Each check compares the C oracle with something it does not contain: sympy's
primality test, Python's arbitrary-precision integers, the O(N^2) schoolbook
convolution, direct polynomial evaluation.
"""
import random
from math import prod

import numpy as np
import pytest
from sympy import isprime

from oracle import bfv
from workloads import PRESETS

from .bruteforce import crt, negacyclic, ntt_primes


def test_presets_are_the_largest_ntt_primes_below_2_50():
    for name, prm in PRESETS.items():
        want = ntt_primes(1 << 50, 2 * prm.n, prm.k + prm.nsp)
        assert list(prm.q) + list(prm.p) == want, name
        assert prm.t == 65537 and (prm.t - 1) % (2 * prm.n) == 0
        assert prm.k % prm.alpha == 0


def test_oracle_primality_matches_sympy():
    rnd = random.Random(1)
    cands = [rnd.getrandbits(50) | 1 for _ in range(300)]
    cands += [p for prm in PRESETS.values() for p in prm.q + prm.p]
    cands += [(1 << 61) - 1, (1 << 61) + 1, 3215031751, 341550071728321]  # strong pseudoprimes
    for c in cands:
        assert bfv.is_prime(c) == isprime(c), c


def test_big_divmod_matches_python():
    rnd = random.Random(2)
    for _ in range(2000):
        abits = rnd.choice([1, 31, 32, 33, 64, 100, 333, 640, 1300])
        bbits = rnd.choice([1, 31, 32, 33, 64, 65, 100, 150, 301, 640])
        a = rnd.getrandbits(abits)
        b = rnd.getrandbits(bbits) | 1
        if rnd.random() < 0.2:                 # stress the quotient-digit correction
            b = (1 << bbits) - rnd.getrandbits(5) - 1 if bbits > 6 else b
            a = b * rnd.getrandbits(max(1, abits - bbits + 1)) + rnd.randrange(b)
        assert bfv.big_divmod(a, b) == divmod(a, b)
    for a, b in [(0, 5), (5, 5), (4, 5), ((1 << 640) - 1, (1 << 320) - 1),
                 (1 << 1000, (1 << 32)), ((1 << 96) - 1, (1 << 64) - 1),
                 (0x8000000000000000_00000000_00000000, 0x80000000_FFFFFFFF)]:
        assert bfv.big_divmod(a, b) == divmod(a, b)


def test_crt_reconstruction_round_trip():
    rnd = random.Random(3)
    for prm in PRESETS.values():
        for mods in (list(prm.q), list(prm.q) + list(prm.p)):
            M = prod(mods)
            for x in [0, 1, M - 1, M // 2, M // 2 + 1] + [rnd.randrange(M) for _ in range(50)]:
                res = [x % m for m in mods]
                assert bfv.crt_words(mods, res) == x
                assert crt(res, mods) == x


@pytest.mark.parametrize("n", [4, 8, 32, 64])
def test_polymul_is_the_schoolbook_negacyclic_convolution(n):
    rnd = random.Random(n)
    for m in ntt_primes(1 << 50, 2 * n, 2) + ntt_primes(1 << 61, 2 * n, 1) + [65537]:
        for _ in range(3):
            a = [rnd.randrange(m) for _ in range(n)]
            b = [rnd.randrange(m) for _ in range(n)]
            want = [x % m for x in negacyclic(a, b)]
            assert [int(x) for x in bfv.polymul(a, b, m)] == want


def test_min_psi_is_the_smallest_primitive_root():
    for n, m in [(8, 17), (8, 97), (16, 97), (32, 193), (64, 257), (8, 65537)]:
        roots = [x for x in range(2, m) if pow(x, n, m) == m - 1]
        assert len(roots) == n
        assert bfv.min_psi(n, m) == min(roots)


@pytest.mark.parametrize("n", [8, 64, 256])
def test_forward_transform_is_evaluation_at_odd_powers_bit_reversed(n):
    rnd = random.Random(100 + n)
    m = ntt_primes(1 << 50, 2 * n, 1)[0]
    psi = bfv.min_psi(n, m)
    assert pow(psi, n, m) == m - 1
    a = [rnd.randrange(m) for _ in range(n)]
    lg = n.bit_length() - 1
    out = bfv.ntt_forward(a, m)
    for i in range(n):
        br = int(format(i, f"0{lg}b")[::-1], 2)
        x = pow(psi, 2 * br + 1, m)
        assert int(out[i]) == sum(c * pow(x, j, m) for j, c in enumerate(a)) % m
    assert [int(x) for x in bfv.ntt_inverse(out, m)] == a


def test_transform_round_trip_and_convolution_theorem_at_full_size():
    for name in ("C1", "C2", "C5"):
        prm = PRESETS[name]
        n, m = prm.n, prm.q[-1]
        rng = np.random.default_rng(5)
        a = rng.integers(0, m, n, dtype=np.uint64)
        b = rng.integers(0, m, n, dtype=np.uint64)
        fa, fb = bfv.ntt_forward(a, m), bfv.ntt_forward(b, m)
        assert np.array_equal(bfv.ntt_inverse(fa, m), a)
        fc = np.array([int(x) * int(y) % m for x, y in zip(fa, fb)], dtype=np.uint64)
        c = bfv.ntt_inverse(fc, m)
        assert np.array_equal(c, bfv.polymul(a, b, m))
        # a few coefficients of the product straight from the definition
        ai, bi = [int(x) for x in a], [int(x) for x in b]
        for idx in (0, 1, n // 2, n - 1):
            s = 0
            for i in range(n):
                j = idx - i
                s += ai[i] * bi[j] if j >= 0 else -ai[i] * bi[j + n]
            assert int(c[idx]) == s % m
