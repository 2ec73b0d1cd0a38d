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
    # the folding sums in rounds of 3 bits on top of the hoisted copies (sampled units); the rounds'
    # elements are 3^e with e < d2, the copies' are 3^(d2 r) or row-swapped: the key tables are disjoint
    _, raw_f, dev_f = _round_keys(env, 0, d2, 3, 1100)
    assert not set(copies) & set(raw_f)
    got = env.host(env.ctx.prefill_qk_hoisted(env.dev(q), env.dev(kk), heads, d2, rlk, dev_f,
                                              [ckeys[g][1] for g in copies], fold_round_bits=3))
    rr = {g: ckeys[g][0] for g in copies}
    rr.update(raw_f)
    for h in range(heads):
        want = attention.prefill_qk_hoisted(env.orc, q[h], kk[h], raw_rlk, rr, d2, w=3)
        for i in (0, 1, m // 2, m - 1):
            assert np.array_equal(got[h, i], want[i]), ("qk rounds", name, h, i)
    a, v = env.cts(93, heads * m), env.cts(94, heads)
    got = env.host(env.ctx.prefill_av_hoisted(env.dev(a), env.dev(v), heads, d2, rlk, [ckeys[g][1] for g in copies]))
    for h in range(heads):
        want = attention.prefill_av_hoisted(env.orc, list(a[h * m:(h + 1) * m]), v[h], raw_rlk, raws, d2)
        assert np.array_equal(got[h], want), ("av", name, h)
    got = env.host(env.ctx.prefill_av_hoisted(env.dev(a), env.dev(v), heads, d2, rlk, [ckeys[g][1] for g in copies],
                                              sum_before_scaling=True))
    for h in range(heads):
        want = attention.prefill_av_hoisted(env.orc, list(a[h * m:(h + 1) * m]), v[h], raw_rlk, raws, d2, sum_first=True)
        assert np.array_equal(got[h], want), ("av, products summed before scaling", name, h)


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
    # the sum over residue classes in rounds of 3 bits (elements 3^(d2 j) and the row swap: disjoint
    # from the copies' 3^c, c < C <= d2)
    _, raw_b, dev_b = _round_keys(env, 1, d2, 3, 1300)
    assert not set(g_copies) & set(raw_b)
    got = env.host(env.ctx.cpvm_hoisted(env.dev(x[None]), env.ctx.plain_prepare(env.dev(polys)), units, C, d2,
                                        [keys[gal][1] for gal in g_copies], dev_b, block_round_bits=3))
    rr = {gal: keys[gal][0] for gal in g_copies}
    rr.update(raw_b)
    for u in range(units):
        want = attention.cpvm_hoisted(env.orc, x, list(polys[u * C:(u + 1) * C]), rr, d2, w=3)
        assert np.array_equal(got[u], want), ("rounds", name, d1, d2, u)


@pytest.mark.parametrize("name", ["C1", "C2", "C5"])
def test_rotation_sum_matches_oracle(name):
    """One, three and seven rotations summed under one mod-down; a batch that spans several
    workgroups with a ragged tail; zero coefficients; the identity among the elements."""
    env = _env(name)
    n = env.n
    gs = [pow(3, 1, 2 * n), pow(3, 64, 2 * n), 2 * n - 1, (2 * n - 1) * pow(3, 5, 2 * n) % (2 * n), 1, 2 * n - 3,
          pow(3, 7, 2 * n)]
    keys = [env.key(900 + i) for i in range(len(gs))]
    batch = 5
    x = env.cts(97, batch)
    x[1, :, :, ::3] = 0
    xd = env.dev(x)
    for n_rot in (1, 3, 7):
        say(f"rotate_sum_hoisted {name}: batch {batch}, {n_rot} rotations")
        got = env.host(env.ctx.rotate_sum_hoisted(xd, gs[:n_rot], [k[1] for k in keys[:n_rot]], batch))
        raws = {g: keys[i][0] for i, g in enumerate(gs[:n_rot])}
        for b in range(batch):
            assert np.array_equal(got[b], env.orc.rotate_sum_hoisted(x[b], gs[:n_rot], raws)), (name, n_rot, b)


def test_rotation_sum_of_a_long_series_and_invalid_arguments():
    from paper_2602_08798_amd.binding import CgError
    env = _env("C1")
    n = env.n
    n_rot = 128                                                             # the most one call takes
    gs = [pow(3, 1 + i, 2 * n) for i in range(n_rot)]
    keys = [env.key(950 + i % 3) for i in range(n_rot)]
    x = env.cts(98, 2)
    xd = env.dev(x)
    say(f"rotate_sum_hoisted C1: 2 x {n_rot} rotations")
    got = env.host(env.ctx.rotate_sum_hoisted(xd, gs, [k[1] for k in keys], 2))
    want = env.orc.rotate_sum_hoisted(x[1], gs, {g: keys[i][0] for i, g in enumerate(gs)})
    assert np.array_equal(got[1], want)
    with pytest.raises(CgError):
        env.ctx.rotate_sum_hoisted(xd, gs + [3], [k[1] for k in keys] + [keys[0][1]], 2)   # 129 rotations
    with pytest.raises(CgError):
        env.ctx.rotate_sum_hoisted(xd, [2], [keys[0][1]], 2)                # even Galois element
    with pytest.raises(CgError):
        env.ctx.rotate_sum_hoisted(xd, [3], [keys[0][1]], 2, out=xd)        # output over the input
    with pytest.raises(CgError):
        env.ctx.rotate_sum_hoisted(xd, [], [], 2)                           # an empty series


def _round_keys(env, which, d2, w, seed):
    """Galois elements of all rounds as the library orders them, checked against the oracle's own
    list; -> (elements, raw keys by element, prepared keys in order)."""
    from oracle import attention
    n = env.n
    gens = attention.block_generators(n, d2) if which else attention.fold_generators(n, d2)
    elts = env.ctx.round_galois(which, d2, w)
    assert elts == [e for r in attention.round_galois(n, gens, w) for e in r], (which, d2, w)
    keys = {g: env.key(seed + i % 5) for i, g in enumerate(sorted(set(elts)))}
    return elts, {g: keys[g][0] for g in keys}, [keys[g][1] for g in elts]


@pytest.mark.parametrize("name,w_fold,w_block", [("C1", 2, 3), ("C2", 3, 4), ("C5", 2, 2), ("C1", 1, 1), ("C1", 6, 7)])
def test_decode_products_with_folding_sums_in_rounds_match_oracle(name, w_fold, w_block):
    from oracle import attention
    env = _env(name)
    heads, n_cts, d2 = 2, 2, 64
    say(f"decode_scores_hoisted / decode_context_hoisted {name}: rounds of {w_fold} / {w_block} bits")
    raw_rlk, rlk = env.key(70)
    _, raw_f, dev_f = _round_keys(env, 0, d2, w_fold, 1100)
    _, raw_b, dev_b = _round_keys(env, 1, d2, w_block, 1200)
    q, kc = env.cts(71, heads), env.cts(72, heads * n_cts)
    got = env.host(env.ctx.decode_scores_hoisted(env.dev(q), env.dev(kc), heads, n_cts, d2, w_fold, rlk, dev_f))
    ext = env.ctx.cache_extend(env.dev(kc), heads, n_cts, n_cts, env.ctx.empty_ext(heads * n_cts))
    got_ext = env.host(env.ctx.decode_scores_hoisted(env.dev(q), None, heads, n_cts, d2, w_fold, rlk, dev_f, kext=ext))
    for h in range(heads):
        for c in range(n_cts):
            want = attention.decode_scores_hoisted(env.orc, q[h], kc[h * n_cts + c], raw_rlk, raw_f, d2, w_fold)
            assert np.array_equal(got[h, c], want), (name, h, c)
            assert np.array_equal(got_ext[h, c], want), (name, h, c, "transformed cache")
    a, vc = env.cts(81, heads * n_cts), env.cts(82, heads * n_cts)
    got = env.host(env.ctx.decode_context_hoisted(env.dev(a), env.dev(vc), heads, n_cts, d2, w_block, rlk, dev_b))
    ext = env.ctx.cache_extend(env.dev(vc), heads, n_cts, n_cts, env.ctx.empty_ext(heads * n_cts))
    got_ext = env.host(env.ctx.decode_context_hoisted(env.dev(a), None, heads, n_cts, d2, w_block, rlk, dev_b, vext=ext))
    for h in range(heads):
        sl = slice(h * n_cts, (h + 1) * n_cts)
        want = attention.decode_context_hoisted(env.orc, list(a[sl]), list(vc[sl]), raw_rlk, raw_b, d2, w_block)
        assert np.array_equal(got[h], want), (name, h)
        assert np.array_equal(got_ext[h], want), (name, h, "transformed cache")


@pytest.mark.parametrize("name,with_copy", [("C1", False), ("C2", True)])
def test_decode_step_with_folding_sums_in_rounds_matches_oracle(name, with_copy):
    """The one-call step (three streams) in its hoisted form, with and without the cache's
    transformed copy: the appended cache, every score ciphertext and the context."""
    from oracle import attention
    from paper_2602_08798_amd.binding import CgError, CgSizeError
    env = _env(name)
    n = env.n
    heads, n_cts, stride, d2, w_fold, w_block = 3, 2, 3, 64, 2, 3
    B = n // d2
    raw_rlk, rlk = env.key(70)
    _, raw_f, dev_f = _round_keys(env, 0, d2, w_fold, 1100)
    _, raw_b, dev_b = _round_keys(env, 1, d2, w_block, 1200)
    rng = np.random.default_rng(11)
    taus = (B + 5, 2 * B + 1)                       # appended inside the products' range, then outside it
    masks_pt = np.zeros((6, n), dtype=np.uint64)
    for t in taus:
        masks_pt[t % B] = rng.integers(0, env.prm.t, n, dtype=np.uint64)
    masks = env.ctx.plain_prepare(env.dev(masks_pt))
    cache = env.cts(640, 2 * heads * stride)
    want_cache = cache.copy()
    dcache = env.dev(cache)
    ext = None
    if with_copy:
        ext = env.ctx.cache_extend(dcache, 2 * heads, stride, stride, env.ctx.empty_ext(2 * heads * stride))
    for tau in taus:
        idx, blk = divmod(tau, B)
        say(f"decode_step_hoisted {name}: token {tau}, transformed copy {with_copy}")
        q, a, rows = env.cts(650 + tau, heads), env.cts(660 + tau, heads * n_cts), env.cts(670 + tau, 2 * heads)
        scores, context = env.ctx.decode_step_hoisted(env.dev(q), env.dev(a), dcache, heads, n_cts, stride, d2, tau,
                                                      env.dev(rows), masks, rlk, w_fold, dev_f, w_block, dev_b,
                                                      cache_ext=ext)
        for c in range(2 * heads):
            masked = env.orc.mul_plain(rows[c], masks_pt[blk])
            want_cache[c * stride + idx] = env.orc.add(want_cache[c * stride + idx], masked)
        assert np.array_equal(env.host(dcache), want_cache), tau
        scores, context = env.host(scores), env.host(context)
        for h in range(heads):
            for c in range(n_cts):
                w = attention.decode_scores_hoisted(env.orc, q[h], want_cache[h * stride + c], raw_rlk, raw_f, d2, w_fold)
                assert np.array_equal(scores[h, c], w), (tau, h, c)
            vs = want_cache[(heads + h) * stride:(heads + h) * stride + n_cts]
            w = attention.decode_context_hoisted(env.orc, list(a[h * n_cts:(h + 1) * n_cts]), list(vs), raw_rlk, raw_b,
                                                 d2, w_block)
            assert np.array_equal(context[h], w), (tau, h)
    # wrong key counts and round sizes are refused before any launch
    q, a, rows = env.dev(env.cts(1, heads)), env.dev(env.cts(2, heads * n_cts)), env.dev(env.cts(3, 2 * heads))
    with pytest.raises(CgSizeError):
        env.ctx.decode_step_hoisted(q, a, dcache, heads, n_cts, stride, d2, 0, rows, masks, rlk, w_fold, dev_f[:-1],
                                    w_block, dev_b, cache_ext=ext)
    with pytest.raises(CgError):
        env.ctx.decode_step_hoisted(q, a, dcache, heads, n_cts, stride, d2, 0, rows, masks, rlk, 8, dev_f, w_block, dev_b,
                                    cache_ext=ext)
    with pytest.raises(CgError):
        env.ctx.round_galois(0, d2, 0)
    assert np.array_equal(env.host(dcache), want_cache)


@pytest.mark.parametrize("name", ["C1", "C2", "C5"])
def test_sum_of_products_with_one_scaling_matches_oracle(name):
    """Groups of 1, 3 and 5 pairs (ragged against the kernel's slices), several groups per launch;
    extreme residues in one pair; rejected sizes."""
    from paper_2602_08798_amd.binding import CgError
    env = _env(name)
    for n_groups, group_len in ((1, 1), (2, 3), (3, 5)):
        say(f"mul_sum {name}: {n_groups} groups of {group_len}")
        batch = n_groups * group_len
        a, b = env.cts(1400 + batch, batch), env.cts(1500 + batch, batch)
        for i, m in enumerate(env.prm.q):                      # one pair at the largest residues
            a[batch - 1, :, i, :] = m - 1
            b[batch - 1, :, i, :] = m - 1
        got = env.host(env.ctx.mul_sum(env.dev(a), env.dev(b), n_groups, group_len))
        for g in range(n_groups):
            sl = slice(g * group_len, (g + 1) * group_len)
            assert np.array_equal(got[g], env.orc.mul_sum(list(a[sl]), list(b[sl]))), (name, n_groups, group_len, g)
    with pytest.raises(CgError):
        env.ctx.mul_sum(env.dev(a), env.dev(b), 0, 3)
    with pytest.raises(CgError):
        env.ctx.mul_sum(env.dev(a), env.dev(b), 3, 0)


@pytest.mark.parametrize("name,with_copy", [("C1", True), ("C2", False), ("C5", False)])
def test_decode_context_and_step_with_products_summed_before_scaling_match_oracle(name, with_copy):
    from oracle import attention
    env = _env(name)
    n = env.n
    heads, n_cts, stride, d2, w_fold, w_block = 2, 3, 3, 64, 3, 3
    B = n // d2
    raw_rlk, rlk = env.key(70)
    _, raw_f, dev_f = _round_keys(env, 0, d2, w_fold, 1100)
    _, raw_b, dev_b = _round_keys(env, 1, d2, w_block, 1200)
    say(f"decode_context_hoisted, products summed before scaling, {name}")
    a, vc = env.cts(83, heads * n_cts), env.cts(84, heads * n_cts)
    got = env.host(env.ctx.decode_context_hoisted(env.dev(a), env.dev(vc), heads, n_cts, d2, w_block, rlk, dev_b,
                                                  sum_before_scaling=True))
    ext = env.ctx.cache_extend(env.dev(vc), heads, n_cts, n_cts, env.ctx.empty_ext(heads * n_cts))
    got_ext = env.host(env.ctx.decode_context_hoisted(env.dev(a), None, heads, n_cts, d2, w_block, rlk, dev_b, vext=ext,
                                                      sum_before_scaling=True))
    for h in range(heads):
        sl = slice(h * n_cts, (h + 1) * n_cts)
        want = attention.decode_context_hoisted(env.orc, list(a[sl]), list(vc[sl]), raw_rlk, raw_b, d2, w_block,
                                                sum_first=True)
        assert np.array_equal(got[h], want), (name, h)
        assert np.array_equal(got_ext[h], want), (name, h, "transformed cache")
    say(f"decode_step_hoisted, products summed before scaling, {name}, transformed copy {with_copy}")
    rng = np.random.default_rng(12)
    tau = 2 * B + 7                                  # appended into the third ciphertext, which the products read
    masks_pt = np.zeros((8, n), dtype=np.uint64)
    masks_pt[tau % B] = rng.integers(0, env.prm.t, n, dtype=np.uint64)
    masks = env.ctx.plain_prepare(env.dev(masks_pt))
    cache = env.cts(680, 2 * heads * stride)
    want_cache = cache.copy()
    dcache = env.dev(cache)
    cext = env.ctx.cache_extend(dcache, 2 * heads, stride, stride, env.ctx.empty_ext(2 * heads * stride)) if with_copy else None
    q, rows = env.cts(681, heads), env.cts(682, 2 * heads)
    scores, context = env.ctx.decode_step_hoisted(env.dev(q), env.dev(a), dcache, heads, n_cts, stride, d2, tau,
                                                  env.dev(rows), masks, rlk, w_fold, dev_f, w_block, dev_b,
                                                  cache_ext=cext, sum_before_scaling=True)
    idx, blk = divmod(tau, B)
    for c in range(2 * heads):
        want_cache[c * stride + idx] = env.orc.add(want_cache[c * stride + idx], env.orc.mul_plain(rows[c], masks_pt[blk]))
    assert np.array_equal(env.host(dcache), want_cache)
    scores, context = env.host(scores), env.host(context)
    for h in range(heads):
        for c in (0, n_cts - 1):
            w = attention.decode_scores_hoisted(env.orc, q[h], want_cache[h * stride + c], raw_rlk, raw_f, d2, w_fold)
            assert np.array_equal(scores[h, c], w), (h, c)
        vs = want_cache[(heads + h) * stride:(heads + h) * stride + n_cts]
        w = attention.decode_context_hoisted(env.orc, list(a[h * n_cts:(h + 1) * n_cts]), list(vs), raw_rlk, raw_b, d2,
                                             w_block, sum_first=True)
        assert np.array_equal(context[h], w), h


def test_decode_step_in_rounds_at_the_smallest_and_largest_head_dimension():
    """d2 = 2 (one fold bit, eleven block bits: rounds of 6 and 5 bits at the widest setting) and
    d2 = N/4 (ten fold bits, two block bits), one head, tokens at the first and last block."""
    from oracle import attention
    env = _env("C1")
    n = env.n
    raw_rlk, rlk = env.key(70)
    for d2, tau, w_fold, w_block in ((2, n // 2 - 1, 1, 7), (n // 4, 3, 7, 2), (n // 4, 4, 4, 1)):
        B = n // d2
        say(f"decode_step_hoisted C1: d2 = {d2}, token {tau}, rounds of {w_fold} / {w_block} bits")
        _, raw_f, dev_f = _round_keys(env, 0, d2, w_fold, 1100)
        _, raw_b, dev_b = _round_keys(env, 1, d2, w_block, 1200)
        rng = np.random.default_rng(13 + d2)
        masks_pt = np.zeros((tau % B + 1, n), dtype=np.uint64)
        masks_pt[tau % B] = rng.integers(0, env.prm.t, n, dtype=np.uint64)
        masks = env.ctx.plain_prepare(env.dev(masks_pt))
        heads, stride = 1, 2
        idx, blk = divmod(tau, B)
        n_cts = idx + 1
        cache = env.cts(690 + d2 + tau, 2 * heads * stride)
        want_cache = cache.copy()
        dcache = env.dev(cache)
        q, a, rows = env.cts(691 + tau, heads), env.cts(692 + tau, heads * n_cts), env.cts(693 + tau, 2 * heads)
        scores, context = env.ctx.decode_step_hoisted(env.dev(q), env.dev(a), dcache, heads, n_cts, stride, d2, tau,
                                                      env.dev(rows), masks, rlk, w_fold, dev_f, w_block, dev_b,
                                                      sum_before_scaling=(n_cts > 1))
        for c in range(2 * heads):               # the first token of a ciphertext is stored, later ones are added
            masked = env.orc.mul_plain(rows[c], masks_pt[blk])
            want_cache[c * stride + idx] = masked if blk == 0 else env.orc.add(want_cache[c * stride + idx], masked)
        assert np.array_equal(env.host(dcache), want_cache), (d2, tau)
        scores, context = env.host(scores), env.host(context)
        for c in range(n_cts):
            w = attention.decode_scores_hoisted(env.orc, q[0], want_cache[c], raw_rlk, raw_f, d2, w_fold)
            assert np.array_equal(scores[0, c], w), (d2, tau, c)
        w = attention.decode_context_hoisted(env.orc, list(a), list(want_cache[stride:stride + n_cts]), raw_rlk, raw_b,
                                             d2, w_block, sum_first=(n_cts > 1))
        assert np.array_equal(context[0], w), (d2, tau)


def test_rotation_sums_with_random_series_match_oracle():
    """Seeded random series: 1 to 20 Galois elements drawn from all odd residues (repeats allowed: the
    same rotation may enter a sum twice), batches of 1 to 7."""
    env = _env("C1")
    n = env.n
    rng = np.random.default_rng(20260208)
    pool = [env.key(1000 + i) for i in range(5)]
    for case in range(6):
        n_rot, batch = int(rng.integers(1, 21)), int(rng.integers(1, 8))
        gs = [int(2 * rng.integers(0, n) + 1) for _ in range(n_rot)]
        which = [int(rng.integers(0, len(pool))) for _ in range(n_rot)]
        say(f"rotate_sum_hoisted C1 random case {case}: batch {batch}, {n_rot} rotations")
        x = env.cts(2000 + case, batch)
        got = env.host(env.ctx.rotate_sum_hoisted(env.dev(x), gs, [pool[w][1] for w in which], batch))
        for b in (0, batch - 1):
            want = env.orc.rotate_sum_hoisted(x[b], gs, [pool[w][0] for w in which])
            assert np.array_equal(got[b], want), (case, b)
