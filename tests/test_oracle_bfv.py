"""Pins for the oracle's evaluator operations.

Three kinds: (i) brute force -- Python-integer schoolbook evaluation of the
definitions on tiny rings, inputs being arbitrary residues; (ii) closed forms
and exact special cases; (iii) decryption semantics with the noise bound, on
the real parameter sets.
"""
import random
from math import prod

import numpy as np
import pytest

from oracle import Client, Oracle
from oracle.client import galois_rot, galois_swap
from workloads import PRESETS, Stream, slot_values

from . import bruteforce as bf
from .toy import toy_params

TOYS = [toy_params(4, 2, 1, 1), toy_params(5, 3, 1, 1), toy_params(4, 4, 2, 2),
        toy_params(3, 6, 2, 2), toy_params(5, 2, 1, 1, below=1 << 30)]


def _rand_ring(rnd, mods, n):
    return [[rnd.randrange(m) for _ in range(n)] for m in mods]


@pytest.mark.parametrize("prm", TOYS, ids=lambda p: f"{p.name}_a{p.alpha}")
def test_mul_matches_brute_force(prm):
    rnd = random.Random(11)
    orc = Oracle(prm)
    q, n = list(prm.q), prm.n
    for trial in range(4):
        a2 = [_rand_ring(rnd, q, n) for _ in range(2)]
        b2 = [_rand_ring(rnd, q, n) for _ in range(2)]
        if trial == 3:   # extreme residues: everything at +-Q/2
            Q = prod(q)
            a2 = [[[(Q // 2 + s) % m for _ in range(n)] for m in q] for s in (0, 1)]
            b2 = a2
        got = orc.mul(np.array(a2, dtype=np.uint64), np.array(b2, dtype=np.uint64))
        assert got.tolist() == bf.bf_mul(a2, b2, q, prm.t)


@pytest.mark.parametrize("prm", TOYS, ids=lambda p: f"{p.name}_a{p.alpha}")
def test_sum_of_products_with_one_scaling_matches_brute_force(prm):
    """Tensor products summed over the integers before the rounding division: brute force for one,
    two and five pairs (one of them at the extreme residues); a single pair is the ordinary product;
    several pairs are NOT the sum of separately scaled products, from which they differ by at most
    (number of pairs + 1) / 2 per coefficient."""
    rnd = random.Random(17)
    orc = Oracle(prm)
    q, n = list(prm.q), prm.n
    Q = prod(q)
    ext = [[[(Q // 2 + s) % m for _ in range(n)] for m in q] for s in (0, 1)]
    pairs = [([_rand_ring(rnd, q, n) for _ in range(2)], [_rand_ring(rnd, q, n) for _ in range(2)]) for _ in range(4)]
    pairs.append((ext, ext))
    arr = lambda x: np.array(x, dtype=np.uint64)
    for cnt in (1, 2, 5):
        sel = pairs[-cnt:]
        got = orc.mul_sum([arr(a) for a, _ in sel], [arr(b) for _, b in sel])
        assert got.tolist() == bf.bf_mul_sum(sel, q, prm.t)
        apart = None
        for a, b in sel:
            m3 = orc.mul(arr(a), arr(b))
            apart = m3 if apart is None else orc.add(apart, m3)
        if cnt == 1:
            assert np.array_equal(got, apart)
        else:
            assert not np.array_equal(got, apart)
            for c in range(3):
                x = bf.ring_from_rns(got[c].tolist(), q)
                y = bf.ring_from_rns(apart[c].tolist(), q)
                assert max(min((u - v) % Q, (v - u) % Q) for u, v in zip(x, y)) <= (cnt + 1) // 2


@pytest.mark.parametrize("prm", TOYS, ids=lambda p: f"{p.name}_a{p.alpha}")
def test_keyswitch_matches_brute_force(prm):
    rnd = random.Random(12)
    orc = Oracle(prm)
    q, p, n = list(prm.q), list(prm.p), prm.n
    for _ in range(3):
        d = _rand_ring(rnd, q, n)
        ksk = [[_rand_ring(rnd, q + p, n) for _ in range(2)] for _ in range(prm.dnum)]
        got = orc.keyswitch(np.array(d, dtype=np.uint64), np.array(ksk, dtype=np.uint64))
        assert got.tolist() == bf.bf_keyswitch(d, ksk, q, p, prm.alpha)


@pytest.mark.parametrize("prm", TOYS[:3], ids=lambda p: p.name)
def test_galois_and_mul_plain_and_add_match_brute_force(prm):
    rnd = random.Random(13)
    orc = Oracle(prm)
    q, n = list(prm.q), prm.n
    poly = _rand_ring(rnd, q, n)
    for g in (1, 3, 9, 2 * n - 1, 5):
        got = orc.galois_poly(np.array(poly, dtype=np.uint64), g)
        assert got.tolist() == [bf.bf_galois(poly[i], g, m) for i, m in enumerate(q)]
    c2 = [_rand_ring(rnd, q, n) for _ in range(2)]
    pt = [rnd.randrange(prm.t) for _ in range(n)]
    pt[0], pt[1] = prm.t // 2, prm.t // 2 + 1          # both sides of the centring threshold
    got = orc.mul_plain(np.array(c2, dtype=np.uint64), np.array(pt, dtype=np.uint64))
    assert got.tolist() == bf.bf_mul_plain(c2, pt, q, prm.t)
    b3 = [_rand_ring(rnd, q, n) for _ in range(3)]
    a3 = [_rand_ring(rnd, q, n) for _ in range(3)]
    got = orc.add(np.array(a3, dtype=np.uint64), np.array(b3, dtype=np.uint64))
    assert got.tolist() == [[[(x + y) % m for x, y in zip(a3[c][i], b3[c][i])]
                             for i, m in enumerate(q)] for c in range(3)]


@pytest.mark.parametrize("prm", TOYS[:3], ids=lambda p: p.name)
def test_relin_and_rotate_compose_as_defined(prm):
    rnd = random.Random(14)
    orc = Oracle(prm)
    q, p, n = list(prm.q), list(prm.p), prm.n
    key = np.array([[_rand_ring(rnd, q + p, n) for _ in range(2)] for _ in range(prm.dnum)],
                   dtype=np.uint64)
    d3 = [_rand_ring(rnd, q, n) for _ in range(3)]
    u = bf.bf_keyswitch(d3[2], key.tolist(), q, p, prm.alpha)
    want = [[[(x + y) % m for x, y in zip(d3[c][i], u[c][i])] for i, m in enumerate(q)]
            for c in range(2)]
    assert orc.relin(np.array(d3, dtype=np.uint64), key).tolist() == want
    c2 = [_rand_ring(rnd, q, n) for _ in range(2)]
    for g in (3, 2 * n - 1):
        s0 = [bf.bf_galois(c2[0][i], g, m) for i, m in enumerate(q)]
        s1 = [bf.bf_galois(c2[1][i], g, m) for i, m in enumerate(q)]
        u = bf.bf_keyswitch(s1, key.tolist(), q, p, prm.alpha)
        want = [[[(x + y) % m for x, y in zip(s0[i], u[0][i])] for i, m in enumerate(q)], u[1]]
        assert orc.rotate(np.array(c2, dtype=np.uint64), g, key).tolist() == want


@pytest.mark.parametrize("prm", TOYS, ids=lambda p: f"{p.name}_a{p.alpha}")
def test_hoisted_rotation_against_the_definition_over_the_integers(prm):
    """Digits lifted from c1 before the Galois map (one decomposition for a series of rotations):
    brute force with Python integers, for block rotations and the row swap; with g = 1 nothing is
    negated and the hoisted form coincides with the ordinary rotation, otherwise it does not."""
    rnd = random.Random(15)
    orc = Oracle(prm)
    q, p, n = list(prm.q), list(prm.p), prm.n
    key = np.array([[_rand_ring(rnd, q + p, n) for _ in range(2)] for _ in range(prm.dnum)], dtype=np.uint64)
    c2 = [_rand_ring(rnd, q, n) for _ in range(2)]
    c2[1][0][1] = 0                      # a zero coefficient: -0 is 0, not q
    ct = np.array(c2, dtype=np.uint64)
    for g in (3, 9, 2 * n - 1, 2 * n - 3):
        got = orc.rotate_hoisted(ct, g, key)
        assert got.tolist() == bf.bf_rotate_hoisted(c2, g, key.tolist(), q, p, prm.alpha)
        assert not np.array_equal(got, orc.rotate(ct, g, key))
    assert np.array_equal(orc.rotate_hoisted(ct, 1, key), orc.rotate(ct, 1, key))
    many = orc.rotate_many(ct, [3, 9], {3: key, 9: key})
    assert np.array_equal(many[0], orc.rotate_hoisted(ct, 3, key)) and np.array_equal(many[1], orc.rotate_hoisted(ct, 9, key))


def test_hoisted_rotations_move_slots_like_ordinary_ones_within_the_noise_bound():
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 32, orc)
    n, h = prm.n, prm.n // 2
    v = slot_values(Stream(32, 1), n, -128, 128)
    ct = cl.encrypt_slots(v)
    vm = v % prm.t
    fresh = cl.noise_budget_bits(ct, cl.codec.encode(v))
    gs = [galois_rot(n, r) for r in (1, 64, 640)] + [galois_swap(n)]
    outs = orc.rotate_many(ct, gs, {g: cl.galois_key(g) for g in gs})
    for r, out in zip((1, 64, 640), outs):
        dec = cl.decrypt_slots(out)
        assert np.array_equal(dec[:h], np.roll(vm[:h], -r)) and np.array_equal(dec[h:], np.roll(vm[h:], -r))
        want = np.concatenate([np.roll(v[:h], -r), np.roll(v[h:], -r)])
        # a key switch adds about dnum N 19 max(Q_j)/P + N/2 to the noise: a few bits off a fresh budget
        assert fresh - cl.noise_budget_bits(out, cl.codec.encode(want)) < 12
    dec = cl.decrypt_slots(outs[3])
    assert np.array_equal(dec[:h], vm[h:]) and np.array_equal(dec[h:], vm[:h])


@pytest.mark.parametrize("prm", TOYS, ids=lambda p: f"{p.name}_a{p.alpha}")
def test_hoisted_rotation_sum_against_the_definition_over_the_integers(prm):
    """One division by P for a whole series: brute force with Python integers for one, two and three
    rotations with different keys; a series of one is the ciphertext plus its hoisted rotation; a
    longer series is NOT the sum of separately rounded rotations (else the single division would
    be untested) but differs from it by less than the number of rotations per coefficient."""
    rnd = random.Random(16)
    orc = Oracle(prm)
    q, p, n = list(prm.q), list(prm.p), prm.n
    keys = {g: np.array([[_rand_ring(rnd, q + p, n) for _ in range(2)] for _ in range(prm.dnum)], dtype=np.uint64)
            for g in (3, 9, 2 * n - 1)}
    c2 = [_rand_ring(rnd, q, n) for _ in range(2)]
    c2[1][0][1] = 0
    ct = np.array(c2, dtype=np.uint64)
    for gs in ([3], [9, 2 * n - 1], [3, 9, 2 * n - 1]):
        got = orc.rotate_sum_hoisted(ct, gs, keys)
        assert got.tolist() == bf.bf_rotate_sum_hoisted(c2, gs, [keys[g].tolist() for g in gs], q, p, prm.alpha)
        apart = ct
        for g in gs:
            apart = orc.add(apart, orc.rotate_hoisted(ct, g, keys[g]))
        if len(gs) == 1:
            assert np.array_equal(got, apart)
        else:
            assert not np.array_equal(got, apart)
            Q = 1
            for m in q:
                Q *= m
            for c in range(2):
                a = bf.ring_from_rns(got[c].tolist(), q)
                b = bf.ring_from_rns(apart[c].tolist(), q)
                assert max(min((x - y) % Q, (y - x) % Q) for x, y in zip(a, b)) < len(gs)
    assert np.array_equal(orc.rotate_sum_hoisted(ct, [], keys), ct)


def test_hoisted_rotation_sum_adds_the_rotated_slots_within_the_noise_bound():
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 33, orc)
    n, h = prm.n, prm.n // 2
    v = slot_values(Stream(33, 1), n, -128, 128)
    ct = cl.encrypt_slots(v)
    fresh = cl.noise_budget_bits(ct, cl.codec.encode(v))
    shifts = (1, 2, 3, 64)
    gs = [galois_rot(n, r) for r in shifts] + [galois_swap(n)]
    out = orc.rotate_sum_hoisted(ct, gs, {g: cl.galois_key(g) for g in gs})
    want = v.copy()
    for r in shifts:
        want = want + np.concatenate([np.roll(v[:h], -r), np.roll(v[h:], -r)])
    want = want + np.concatenate([v[h:], v[:h]])
    assert np.array_equal(cl.decrypt_slots(out), want % prm.t)
    # six ciphertexts' noise and five key switches' noise add up: log2(6) + a few bits
    assert fresh - cl.noise_budget_bits(out, cl.codec.encode(want)) < 15


def test_keyswitch_of_zero_is_zero_and_relin_keeps_two_component_input():
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    rng = np.random.default_rng(3)
    key = np.stack([rng.integers(0, m, (prm.dnum, 2, prm.n), dtype=np.uint64)
                    for m in prm.q + prm.p], axis=2)
    zero = np.zeros((prm.k, prm.n), dtype=np.uint64)
    assert not orc.keyswitch(zero, key).any()
    d3 = np.zeros((3, prm.k, prm.n), dtype=np.uint64)
    for i, m in enumerate(prm.q):
        d3[:2, i] = rng.integers(0, m, (2, prm.n), dtype=np.uint64)
    assert np.array_equal(orc.relin(d3, key), d3[:2])


def test_mul_closed_form_on_noise_free_constant_ciphertexts():
    """(Delta m1, 0) x (Delta m2, 0) with constant polynomials: d0 = round(t c(Delta m1) c(Delta m2) / Q)."""
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 5, orc)
    Q, t = cl.Q, cl.t
    for m1, m2 in [(1, 1), (2, 3), (65536, 65536), (32768, 32769), (12345, 54321)]:
        pt1 = np.zeros(prm.n, dtype=np.uint64); pt1[0] = m1
        pt2 = np.zeros(prm.n, dtype=np.uint64); pt2[0] = m2
        d = orc.mul(cl.trivial(pt1), cl.trivial(pt2))
        x = bf.centre(cl.delta * m1, Q) * bf.centre(cl.delta * m2, Q)
        want0 = bf.round_div(t * x, Q) % Q
        assert [int(d[0, i, 0]) for i in range(prm.k)] == [want0 % m for m in prm.q]
        assert not d[0, :, 1:].any() and not d[1:].any()


def test_decrypted_product_is_the_slotwise_product_within_the_noise_bound():
    """C1 shape: slots uniform in [0,t); Dec(relin(mul)) = m1*m2 mod t with budget left."""
    prm = PRESETS["C1"]
    orc = Oracle(prm)
    cl = Client(prm, 20260208, orc)
    g = Stream(20260208, 50)
    rlk = cl.relin_key()
    logq = sum(np.log2(float(m)) for m in prm.q)
    for _ in range(2):
        v1, v2 = slot_values(g, prm.n, 0, prm.t), slot_values(g, prm.n, 0, prm.t)
        c1, c2 = cl.encrypt_slots(v1), cl.encrypt_slots(v2)
        fresh = cl.noise_budget_bits(c1, cl.codec.encode(v1))
        # fresh: |t e - (Q mod t) m| <= 19 t + t^2
        assert fresh >= logq - 1 - np.log2(19 * prm.t + prm.t ** 2)
        want = v1 * v2 % prm.t
        d3 = orc.mul(c1, c2)
        assert np.array_equal(cl.decrypt_slots(d3), want)
        d2 = orc.relin(d3, rlk)
        assert np.array_equal(cl.decrypt_slots(d2), want)
        left = cl.noise_budget_bits(d2, cl.codec.encode(want))
        # one multiplication costs about log2(t N) plus a few bits
        assert 0 < left and fresh - left < np.log2(prm.t * prm.n) + 8


@pytest.mark.parametrize("name", ["C2", "C5"])
def test_keyswitch_invariant_against_the_secret(name):
    """u0 + u1 s - d s' is small: |.| <= dnum N 19 max(Q_j)/P + (1 + N)/2 + slack."""
    prm = PRESETS[name]
    orc = Oracle(prm)
    cl = Client(prm, 77, orc)
    rng = np.random.default_rng(9)
    d = np.stack([rng.integers(0, m, prm.n, dtype=np.uint64) for m in prm.q])
    s_prime = cl.secret_square()
    key = cl.switch_key(s_prime)
    u = orc.keyswitch(d, key)
    # phase of (u0 - d*s', u1): put d*s' on the c0 side
    ds = np.stack([Client._res(s_prime, m) for m in prm.q])
    from oracle import bfv
    c0 = np.stack([(u[0, i].astype(object) + (m - bfv.polymul(d[i], ds[i], m).astype(object))) % m
                   for i, m in enumerate(prm.q)]).astype(np.uint64)
    ph = cl._phase(np.stack([c0, u[1]]))
    qj = max(prod(prm.q[j * prm.alpha:(j + 1) * prm.alpha]) for j in range(prm.dnum))
    bound = prm.dnum * prm.n * 19 * qj // cl.P + (1 + prm.n) // 2 + 2
    assert max(abs(x) for x in ph) <= bound
    assert max(abs(x) for x in ph) > 0


def test_rotations_move_slots_as_documented():
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 31, orc)
    n, h = prm.n, prm.n // 2
    v = slot_values(Stream(31, 1), n, -128, 128)
    ct = cl.encrypt_slots(v)
    vm = v % prm.t
    for r in (1, 5, 64):
        g = galois_rot(n, r)
        out = cl.decrypt_slots(orc.rotate(ct, g, cl.galois_key(g)))
        assert np.array_equal(out[:h], np.roll(vm[:h], -r))
        assert np.array_equal(out[h:], np.roll(vm[h:], -r))
    g = galois_swap(n)
    out = cl.decrypt_slots(orc.rotate(ct, g, cl.galois_key(g)))
    assert np.array_equal(out[:h], vm[h:]) and np.array_equal(out[h:], vm[:h])
    out = cl.decrypt_slots(orc.rotate(ct, 1, cl.switch_key(cl.s)))
    assert np.array_equal(out, vm)


def test_mul_plain_masks_slots_and_add_adds_them():
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 41, orc)
    n = prm.n
    g = Stream(41, 1)
    v, w = slot_values(g, n, -128, 128), slot_values(g, n, -128, 128)
    mask = np.zeros(n, dtype=np.int64); mask[64:128] = 1; mask[n - 64:] = 1
    out = cl.decrypt_slots(orc.mul_plain(cl.encrypt_slots(v), cl.codec.encode(mask)))
    assert np.array_equal(out, (v * mask) % prm.t)
    out = cl.decrypt_slots(orc.add(cl.encrypt_slots(v), cl.encrypt_slots(w)))
    assert np.array_equal(out, (v + w) % prm.t)


def test_slot_codec_is_evaluation_at_the_documented_points():
    prm = toy_params(5, 2, 1, 1)
    cl = Client(prm, 1)
    n, t = prm.n, prm.t
    v = slot_values(Stream(2, 2), n, 0, t)
    pt = [int(x) for x in cl.codec.encode(v)]
    zeta = cl.codec.zeta
    assert pow(zeta, n, t) == t - 1
    for j in range(n):
        row, pos = divmod(j, n // 2)
        e = pow(3, pos, 2 * n) if row == 0 else (-pow(3, pos, 2 * n)) % (2 * n)
        x = pow(zeta, e, t)
        assert sum(c * pow(x, i, t) for i, c in enumerate(pt)) % t == int(v[j])
    assert np.array_equal(cl.codec.decode(np.array(pt, dtype=np.uint64)), v)
