"""Brute-force definitions on tiny rings, in Python integers only.

Nothing here uses a transform, a residue number system or the C oracle: ring
products are the O(N^2) schoolbook negacyclic convolution over the integers,
roundings are exact integer divisions.  The oracle is pinned against these on
small N; they are far too slow for anything else.
"""
from math import prod

from sympy import isprime


def ntt_primes(below: int, two_n: int, count: int):
    """The `count` largest primes < below that are 1 mod two_n, descending."""
    c = below - 1
    c -= (c - 1) % two_n
    out = []
    while len(out) < count:
        if isprime(c):
            out.append(c)
        c -= two_n
    return out


def negacyclic(a, b):
    """a*b in Z[X]/(X^n+1) for integer coefficient lists."""
    n = len(a)
    out = [0] * n
    for i, x in enumerate(a):
        if x == 0:
            continue
        for j, y in enumerate(b):
            k = i + j
            if k >= n:
                out[k - n] -= x * y
            else:
                out[k] += x * y
    return out


def centre(x: int, m: int) -> int:
    x %= m
    return x - m if x > m // 2 else x


def crt(res, mods) -> int:
    M = prod(mods)
    x = 0
    for r, m in zip(res, mods):
        h = M // m
        x += int(r) * pow(h % m, -1, m) * h
    return x % M


def round_div(num: int, den: int) -> int:
    """Nearest integer to num/den (den > 0), halves rounded up."""
    return (2 * num + den) // (2 * den)


def ring_from_rns(rows, mods):
    """rows[i][n] residues -> list of integers in [0, prod mods)."""
    n = len(rows[0])
    return [crt([rows[i][j] for i in range(len(mods))], mods) for j in range(n)]


def bf_mul(a2, b2, q, t):
    """Tensor product scaled by t/Q and rounded; returns [3][k][n] residues."""
    Q = prod(q)
    a = [[centre(x, Q) for x in ring_from_rns(c, q)] for c in a2]
    b = [[centre(x, Q) for x in ring_from_rns(c, q)] for c in b2]
    e0 = negacyclic(a[0], b[0])
    e1 = [x + y for x, y in zip(negacyclic(a[0], b[1]), negacyclic(a[1], b[0]))]
    e2 = negacyclic(a[1], b[1])
    out = []
    for e in (e0, e1, e2):
        d = [round_div(t * x, Q) for x in e]
        out.append([[x % m for x in d] for m in q])
    return out


def bf_mul_sum(pairs, q, t):
    """Sum over the pairs (a2, b2) of the tensor products over the integers, then ONE scaling by t/Q
    with rounding; returns [3][k][n] residues."""
    Q = prod(q)
    n = len(pairs[0][0][0][0])
    e = [[0] * n for _ in range(3)]
    for a2, b2 in pairs:
        a = [[centre(x, Q) for x in ring_from_rns(c, q)] for c in a2]
        b = [[centre(x, Q) for x in ring_from_rns(c, q)] for c in b2]
        terms = (negacyclic(a[0], b[0]),
                 [x + y for x, y in zip(negacyclic(a[0], b[1]), negacyclic(a[1], b[0]))],
                 negacyclic(a[1], b[1]))
        for cc in range(3):
            e[cc] = [x + y for x, y in zip(e[cc], terms[cc])]
    return [[[round_div(t * x, Q) % m for x in e[cc]] for m in q] for cc in range(3)]


def bf_keyswitch(d, ksk, q, p, alpha):
    """Hybrid key switch of d ([k][n]) with ksk ([dnum][2][k+nsp][n]); returns [2][k][n]."""
    k, n = len(q), len(d[0])
    P, Q = prod(p), prod(q)
    PQ = P * Q
    qp = list(q) + list(p)
    dnum = k // alpha
    acc = [[0] * n, [0] * n]
    for j in range(dnum):
        mods = q[j * alpha:(j + 1) * alpha]
        digit = ring_from_rns(d[j * alpha:(j + 1) * alpha], mods)   # in [0, Q_j)
        for c in range(2):
            key = ring_from_rns(ksk[j][c], qp)
            pr = negacyclic(digit, key)
            acc[c] = [(x + y) % PQ for x, y in zip(acc[c], pr)]
    out = []
    for c in range(2):
        u = [((x + P // 2) // P) % Q for x in acc[c]]
        out.append([[x % m for x in u] for m in q])
    return out


def bf_rotate_hoisted(c2, g, ksk, q, p, alpha):
    """Rotation with the digits lifted before the Galois map, all over the integers: digit_j = c1 mod Q_j
    in [0, Q_j); sigma_g moves coefficient x at index i to index i g mod n as x, or as -x when
    i g mod 2n >= n; A_c = sum_j sigma_g(digit_j) key_{j,c} mod PQ; u_c = floor((A_c + floor(P/2)) / P)
    mod Q; result (sigma_g(c0) + u0, u1) as [2][k][n] residues."""
    k, n = len(q), len(c2[0][0])
    P, Q = prod(p), prod(q)
    PQ = P * Q
    qp = list(q) + list(p)
    acc = [[0] * n, [0] * n]
    for j in range(k // alpha):
        mods = q[j * alpha:(j + 1) * alpha]
        digit = ring_from_rns(c2[1][j * alpha:(j + 1) * alpha], mods)
        moved = [0] * n
        for i, x in enumerate(digit):
            e = i * g % (2 * n)
            moved[e - n if e >= n else e] = -x if e >= n else x
        for c in range(2):
            pr = negacyclic(moved, ring_from_rns(ksk[j][c], qp))
            acc[c] = [(x + y) % PQ for x, y in zip(acc[c], pr)]
    u = [[((x + P // 2) // P) % Q for x in acc[c]] for c in range(2)]
    s0 = [bf_galois(c2[0][i], g, m) for i, m in enumerate(q)]
    return [[[(a + x) % m for a, x in zip(s0[i], u[0])] for i, m in enumerate(q)],
            [[x % m for x in u[1]] for m in q]]


def bf_rotate_sum_hoisted(c2, gs, ksks, q, p, alpha):
    """c2 + the sum of its hoisted rotations with one division by P, all over the integers:
    A_c = sum_i sum_j sigma_{g_i}(digit_j) key_{i,j,c} mod PQ with the digits and sigma as in
    bf_rotate_hoisted; u_c = floor((A_c + floor(P/2)) / P) mod Q; result
    (c0 + sum_i sigma_{g_i}(c0) + u0, c1 + u1) as [2][k][n] residues."""
    k, n = len(q), len(c2[0][0])
    P, Q = prod(p), prod(q)
    PQ = P * Q
    qp = list(q) + list(p)
    digits = [ring_from_rns(c2[1][j * alpha:(j + 1) * alpha], q[j * alpha:(j + 1) * alpha]) for j in range(k // alpha)]
    acc = [[0] * n, [0] * n]
    out0 = [[int(x) for x in row] for row in c2[0]]
    for g, ksk in zip(gs, ksks):
        for j, digit in enumerate(digits):
            moved = [0] * n
            for i, x in enumerate(digit):
                e = i * g % (2 * n)
                moved[e - n if e >= n else e] = -x if e >= n else x
            for c in range(2):
                pr = negacyclic(moved, ring_from_rns(ksk[j][c], qp))
                acc[c] = [(x + y) % PQ for x, y in zip(acc[c], pr)]
        for i, m in enumerate(q):
            out0[i] = [(a + b) % m for a, b in zip(out0[i], bf_galois(c2[0][i], g, m))]
    u = [[((x + P // 2) // P) % Q for x in acc[c]] for c in range(2)]
    return [[[(a + x) % m for a, x in zip(out0[i], u[0])] for i, m in enumerate(q)],
            [[(int(a) + x) % m for a, x in zip(c2[1][i], u[1])] for i, m in enumerate(q)]]


def bf_galois(poly, g, m):
    n = len(poly)
    out = [0] * n
    for i, x in enumerate(poly):
        e = i * g % (2 * n)
        if e >= n:
            out[e - n] = (-int(x)) % m
        else:
            out[e] = int(x) % m
    return out


def bf_mul_plain(c2, pt, q, t):
    ptc = [centre(int(x), t) for x in pt]
    out = []
    for comp in c2:
        rows = []
        for i, m in enumerate(q):
            pr = negacyclic([int(x) for x in comp[i]], ptc)
            rows.append([x % m for x in pr])
        out.append(rows)
    return out
