"""Hoisted rotations (a series of rotations of the same ciphertext from one decomposition of its c1)
and the entry points built on them, bit for bit against the oracle's definition of the hoisted form.
Pseudo-ciphertexts and pseudo-keys: the operations are defined on arbitrary residues."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from workloads import Stream

from .test_gpu_parity import Env, _block_keys, _envs, _fold_keys, say


def _env(name):
    if name not in _envs:
        _envs[name] = Env(name)
    return _envs[name]


@pytest.mark.parametrize("name", ["C1", "C2", "C5"])
def test_rotation_series_matches_oracle(name):
    """Block rotations, the row swap, their product, the identity, a residue pattern with zero
    coefficients; batches that span several workgroups; the output order [b][i]."""
    env = _env(name)
    n = env.n
    gs = [pow(3, 1, 2 * n), pow(3, 64, 2 * n), 2 * n - 1, (2 * n - 1) * pow(3, 5, 2 * n) % (2 * n), 1, 2 * n - 3]
    keys = [env.key(900 + i) for i in range(len(gs))]
    batch = 3
    say(f"rotate_hoisted {name}: batch {batch} x {len(gs)} rotations")
    x = env.cts(95, batch)
    x[1, 1, :, ::3] = 0                                 # -0 stays 0
    got = env.host(env.ctx.rotate_hoisted(env.dev(x), gs, [k[1] for k in keys], batch))
    assert got.shape[:2] == (batch, len(gs))
    for b in range(batch):
        for i, g in enumerate(gs):
            assert np.array_equal(got[b, i], env.orc.rotate_hoisted(x[b], g, keys[i][0])), (name, b, i)
    # not the ordinary rotation (other bits), except for g = 1 where nothing is negated
    plain = env.host(env.ctx.rotate(env.dev(x), gs[0], keys[0][1], batch))
    assert not np.array_equal(plain[0], got[0, 0])
    ident = env.host(env.ctx.rotate(env.dev(x), 1, keys[4][1], batch))
    assert np.array_equal(ident[2], got[2, 4])


def test_rotation_series_longer_than_one_round_and_invalid_arguments():
    """More rotations than one launch's table holds (two rounds over the same digits), sampled
    against the oracle; rejected arguments launch nothing."""
    from paper_2602_08798_amd.binding import CgError
    env = _env("C1")
    n = env.n
    n_rot = 131
    gs = [pow(3, 1 + i, 2 * n) for i in range(n_rot)]
    keys = [env.key(950 + i % 3) for i in range(n_rot)]
    x = env.cts(96, 2)
    say(f"rotate_hoisted C1: 2 x {n_rot} rotations")
    got = env.host(env.ctx.rotate_hoisted(env.dev(x), gs, [k[1] for k in keys], 2))
    for b, i in ((0, 0), (1, 127), (0, 128), (1, 130)):
        assert np.array_equal(got[b, i], env.orc.rotate_hoisted(x[b], gs[i], keys[i][0])), (b, i)
    xd = env.dev(x)
    with pytest.raises(CgError):
        env.ctx.rotate_hoisted(xd, [2], [keys[0][1]], 2)                    # even Galois element
    with pytest.raises(CgError):
        env.ctx.rotate_hoisted(xd, [3, 2 * n + 1], [keys[0][1]] * 2, 2)     # out of range
    with pytest.raises(CgError):
        env.ctx.rotate_hoisted(xd, [3], [keys[0][1]], 2, out=xd)            # output over the input
    with pytest.raises(CgError):
        env.ctx.rotate_hoisted(xd, [], [], 2)                               # an empty series


@pytest.mark.parametrize("name,heads,d2", [("C1", 2, 256), ("C2", 1, 512)])
def test_prompt_products_with_hoisted_copies_match_oracle(name, heads, d2):
    from oracle import attention
    env = _env(name)
    n = env.n
    m = n // d2
    say(f"prefill_qk_hoisted / prefill_av_hoisted {name}, d2 = {d2} (m = {m}), {heads} heads")
    raw_rlk, rlk = env.key(70)
    fold = _fold_keys(env, d2)
    fkeys = {g: env.key(300 + i) for i, g in enumerate(fold)}
    copies = attention.copy_galois(n, d2)[1:]
    ckeys = {g: env.key(700 + i) for i, g in enumerate(copies)}
    raws = {g: fkeys[g][0] for g in fold}
    raws.update({g: ckeys[g][0] for g in copies})
    q, kk = env.cts(91, heads), env.cts(92, heads)
    got = env.host(env.ctx.prefill_qk_hoisted(env.dev(q), env.dev(kk), heads, d2, rlk, [fkeys[g][1] for g in fold],
                                              [ckeys[g][1] for g in copies]))
    for h in range(heads):
        want = attention.prefill_qk_hoisted(env.orc, q[h], kk[h], raw_rlk, raws, d2)
        for i, w in enumerate(want):
            assert np.array_equal(got[h, i], w), ("qk", name, h, i)
    a, v = env.cts(93, heads * m), env.cts(94, heads)
    got = env.host(env.ctx.prefill_av_hoisted(env.dev(a), env.dev(v), heads, d2, rlk, [ckeys[g][1] for g in copies]))
    for h in range(heads):
        want = attention.prefill_av_hoisted(env.orc, list(a[h * m:(h + 1) * m]), v[h], raw_rlk, raws, d2)
        assert np.array_equal(got[h], want), ("av", name, h)


@pytest.mark.parametrize("name,d1,d2,units", [("C1", 1000, 64, 2), ("C2", 768, 64, 3), ("C5", 768, 64, 1)])
def test_cpvm_with_hoisted_token_copies_matches_oracle(name, d1, d2, units):
    from oracle import attention
    from oracle.client import SlotCodec
    env = _env(name)
    n = env.n
    D1, T, C = attention.cpvm_shape(n, d1, d2)
    say(f"cpvm_hoisted {name}: d1 {d1}, d2 {d2}, {C} diagonals, {units} matrices")
    codec = SlotCodec(env.prm)
    g = Stream(1700 + d1, units)
    polys = np.stack([codec.encode(attention.cpvm_weight_values(n, d1, d2, g.integers(-128, 128, (d1, d2)), c))
                      for u in range(units) for c in range(C)])
    x = env.cts(1701 + d1, 1)[0]
    g_copies = [pow(3, c, 2 * n) for c in range(1, C)]
    g_block = _block_keys(env, d2)
    keys = {gal: env.key(1800 + i) for i, gal in enumerate(sorted(set(g_copies + g_block)))}
    got = env.host(env.ctx.cpvm_hoisted(env.dev(x[None]), env.ctx.plain_prepare(env.dev(polys)), units, C, d2,
                                        [keys[gal][1] for gal in g_copies], [keys[gal][1] for gal in g_block]))
    raw = {gal: keys[gal][0] for gal in keys}
    for u in range(units):
        want = attention.cpvm_hoisted(env.orc, x, list(polys[u * C:(u + 1) * C]), raw, d2)
        assert np.array_equal(got[u], want), (name, d1, d2, u)
