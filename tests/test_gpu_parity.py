"""Bit-exact parity of the HIP library (through its C ABI) with the CPU oracle.

Inputs are seeded: mostly uniformly random canonical residues (every evaluator
operation is defined on arbitrary residues, and a fresh ciphertext is
indistinguishable from uniform), plus real encryptions where the decrypted
meaning is checked as well.  Sizes: the three parameter sets of the benchmark
configurations (N = 4096/k = 2, N = 8192/k = 3, N = 16384/k = 6 with two
special primes and alpha = 2), batches spanning several workgroups.
"""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from workloads import PRESETS, Stream, attention_activations, pseudo_ciphertexts, pseudo_switch_key


def say(msg):
    print(f"[gpu-parity] {msg}", flush=True)
    sys.stdout.flush()


class Env:
    def __init__(self, name):
        import paper_2602_08798_amd as P
        from oracle import Oracle
        self.P = P
        self.name = name
        self.prm = PRESETS[name]
        self.ctx = P.Context(self.prm)
        self.orc = Oracle(self.prm)
        self.n, self.k = self.prm.n, self.prm.k
        self.qp = list(self.prm.q) + list(self.prm.p)
        self._keys = {}

    def cts(self, seed, batch, ncomp=2):
        return pseudo_ciphertexts(Stream(seed, 1), self.prm.q, self.n, batch, ncomp)

    def key(self, seed):
        """(raw numpy key, prepared device key)"""
        if seed not in self._keys:
            raw = pseudo_switch_key(Stream(seed, 2), self.qp, self.n, self.prm.dnum)
            self._keys[seed] = (raw, self.ctx.ksk_prepare(self.P.to_device(raw)))
        return self._keys[seed]

    def dev(self, a):
        return self.P.to_device(a)

    def host(self, t):
        import torch
        torch.cuda.synchronize()
        return self.P.to_host(t)


_envs = {}


@pytest.fixture(params=["C1", "C2", "C5"])
def env(request):
    if request.param not in _envs:
        _envs[request.param] = Env(request.param)
    return _envs[request.param]


def test_transform_matches_definition(env):
    say(f"ntt {env.name}")
    from oracle import bfv
    L = env.k + env.prm.nsp
    idx = [i % L for i in range(L + 3)]
    rng = np.random.default_rng(1)
    rows = np.stack([rng.integers(0, env.qp[i], env.n, dtype=np.uint64) for i in idx])
    rows[0, :4] = [0, 1, env.qp[idx[0]] - 1, env.qp[idx[0]] - 2]
    got = env.host(env.ctx.ntt_forward(env.dev(rows), idx))
    for r, i in enumerate(idx):
        assert np.array_equal(got[r], bfv.ntt_forward(rows[r], env.qp[i])), (env.name, r)
    back = env.host(env.ctx.ntt_inverse(env.dev(got), idx))
    assert np.array_equal(back, rows)
    # an arbitrary assignment of primes to rows (goes through the staged index table)
    idx2 = [(L - 1 - i) % L for i in range(L)] + [0, 0, L - 1]
    rows2 = np.stack([rng.integers(0, env.qp[i], env.n, dtype=np.uint64) for i in idx2])
    got2 = env.host(env.ctx.ntt_forward(env.dev(rows2), idx2))
    for r, i in enumerate(idx2):
        assert np.array_equal(got2[r], bfv.ntt_forward(rows2[r], env.qp[i])), (env.name, r)
    assert np.array_equal(env.host(env.ctx.ntt_inverse(env.dev(got2), idx2)), rows2)


def test_mul_matches_oracle(env):
    say(f"mul {env.name}")
    batch = 3
    a, b = env.cts(10, batch), env.cts(11, batch)
    # extreme residues in unit 0: zeros, q-1, and the two values around Q/2
    Q = int(np.prod([int(x) for x in env.prm.q], dtype=object))
    for i, m in enumerate(env.prm.q):
        a[0, 0, i, :4] = [0, m - 1, (Q // 2) % m, (Q // 2 + 1) % m]
        b[0, 1, i, :4] = [m - 1, m - 1, (Q // 2) % m, (Q // 2 + 1) % m]
    got = env.host(env.ctx.mul(env.dev(a), env.dev(b), batch))
    for u in range(batch):
        assert np.array_equal(got[u], env.orc.mul(a[u], b[u])), (env.name, u)
    say(f"mul a_group {env.name}")
    got = env.host(env.ctx.mul(env.dev(a[:1]), env.dev(b), batch, a_group=3))
    for u in range(batch):
        assert np.array_equal(got[u], env.orc.mul(a[0], b[u])), (env.name, u)


def test_relin_and_mul_relin_match_oracle(env):
    say(f"relin {env.name}")
    batch = 2
    raw, rlk = env.key(20)
    d3 = env.cts(21, batch, 3)
    got = env.host(env.ctx.relin(env.dev(d3), rlk, batch))
    for u in range(batch):
        assert np.array_equal(got[u], env.orc.relin(d3[u], raw)), (env.name, u)
    say(f"mul_relin {env.name}")
    a, b = env.cts(22, batch), env.cts(23, batch)
    got = env.host(env.ctx.mul_relin(env.dev(a), env.dev(b), rlk, batch))
    for u in range(batch):
        assert np.array_equal(got[u], env.orc.relin(env.orc.mul(a[u], b[u]), raw)), (env.name, u)


def test_rotate_matches_oracle(env):
    batch = 2
    raw, gk = env.key(30)
    x = env.cts(31, batch)
    x[0, :, :, :3] = 0                                     # zero coefficients: negation of 0 stays 0
    n = env.n
    for g in (3, pow(3, 64, 2 * n), 2 * n - 1, 1, 2 * n - 3):
        for acc in (False, True):
            say(f"rotate {env.name} g={g} acc={acc}")
            got = env.host(env.ctx.rotate(env.dev(x), g, gk, batch, accumulate=acc))
            for u in range(batch):
                want = env.orc.rotate(x[u], g, raw)
                if acc:
                    want = env.orc.add(x[u], want)
                assert np.array_equal(got[u], want), (env.name, g, acc, u)


def test_add_matches_oracle(env):
    say(f"add {env.name}")
    for ncomp in (2, 3):
        a, b = env.cts(40, 2, ncomp), env.cts(41, 2, ncomp)
        got = env.host(env.ctx.add(env.dev(a), env.dev(b), ncomp, 2))
        for u in range(2):
            assert np.array_equal(got[u], env.orc.add(a[u], b[u]))


def test_add_plain_matches_oracle(env):
    """Masking and unmasking of the lazy noise refresh: one plaintext for the whole batch or one per
    ciphertext, both signs, also in place."""
    say(f"add_plain {env.name}")
    n, t = env.n, env.prm.t
    rng = np.random.default_rng(40)
    pts = rng.integers(0, t, (3, n), dtype=np.uint64)
    pts[0, :3] = [0, t - 1, t // 2]
    x = env.cts(41, 3)
    for negative in (False, True):
        got = env.host(env.ctx.add_plain(env.dev(x), env.dev(pts), 3, negative=negative))
        one = env.host(env.ctx.add_plain(env.dev(x), env.dev(pts[:1]), 3, negative=negative))
        for u in range(3):
            assert np.array_equal(got[u], env.orc.add_plain(x[u], pts[u], negative)), (env.name, negative, u)
            assert np.array_equal(one[u], env.orc.add_plain(x[u], pts[0], negative)), (env.name, negative, u)
    dx = env.dev(x)
    env.ctx.add_plain(dx, env.dev(pts), 3, negative=True, out=dx)
    env.ctx.add_plain(dx, env.dev(pts), 3, out=dx)
    assert np.array_equal(env.host(dx), x)


def test_mul_plain_and_append_match_oracle(env):
    say(f"mul_plain {env.name}")
    n, t = env.n, env.prm.t
    rng = np.random.default_rng(50)
    pts = rng.integers(0, t, (3, n), dtype=np.uint64)
    pts[0, :2] = [t // 2, t // 2 + 1]
    plain = env.ctx.plain_prepare(env.dev(pts))
    x = env.cts(51, 3)
    got = env.host(env.ctx.mul_plain(env.dev(x), plain, 3, plain_stride=1))
    for u in range(3):
        assert np.array_equal(got[u], env.orc.mul_plain(x[u], pts[u]))
    got = env.host(env.ctx.mul_plain(env.dev(x), plain, 3, plain_stride=0))
    for u in range(3):
        assert np.array_equal(got[u], env.orc.mul_plain(x[u], pts[0]))

    say(f"kv_append {env.name}")
    # 3 caches of 2 ciphertexts each; "masks" are arbitrary plaintexts here (B of them is too many to
    # transform on the CPU, so the cache geometry uses d2 = N/4, B = 4)
    d2 = n // 4
    masks_pt = rng.integers(0, t, (4, n), dtype=np.uint64)
    masks = env.ctx.plain_prepare(env.dev(masks_pt))
    cache = env.cts(52, 6)                                  # junk contents: first append must ignore them
    want = cache.copy()
    dcache = env.dev(cache)
    for tau in (0, 1, 3, 4, 5):
        rows = env.cts(60 + tau, 3)
        env.ctx.kv_append(dcache, 2, 3, tau, env.dev(rows), masks, d2)
        for c in range(3):
            idx, blk = divmod(tau, 4)
            masked = env.orc.mul_plain(rows[c], masks_pt[blk])
            want[c * 2 + idx] = masked if blk == 0 else env.orc.add(want[c * 2 + idx], masked)
    assert np.array_equal(env.host(dcache), want)


def _fold_keys(env, d2):
    n = env.n
    gs, sh = [], 1
    while sh < d2:
        gs.append(pow(3, sh, 2 * n))
        sh *= 2
    return gs


def _block_keys(env, d2):
    n = env.n
    gs, sh = [], d2
    while sh <= n // 4:
        gs.append(pow(3, sh, 2 * n))
        sh *= 2
    return gs + [2 * n - 1]


def test_decode_scores_match_oracle(env):
    from oracle import attention
    say(f"decode_scores {env.name}")
    heads, n_cts, d2 = 2, 2, 64
    raw_rlk, rlk = env.key(70)
    gs = _fold_keys(env, d2)
    keys = {g: env.key(100 + i) for i, g in enumerate(gs)}
    q, kc = env.cts(71, heads), env.cts(72, heads * n_cts)
    got = env.host(env.ctx.decode_scores(env.dev(q), env.dev(kc), heads, n_cts, d2, rlk,
                                         [keys[g][1] for g in gs]))
    # the same call reading the cache in transformed form (strided: one spare ciphertext per head)
    stride = n_cts + 1
    spaced = np.zeros((heads * stride,) + kc.shape[1:], dtype=kc.dtype)
    for h in range(heads):
        spaced[h * stride:h * stride + n_cts] = kc[h * n_cts:(h + 1) * n_cts]
    ext = env.ctx.empty_ext(heads * stride)
    ext.fill_(float("nan"))                              # entries that are not extended must not be read
    env.ctx.cache_extend(env.dev(spaced), heads, n_cts, stride, ext)
    got_ext = env.host(env.ctx.decode_scores_ext(env.dev(q), ext, heads, n_cts, d2, rlk, [keys[g][1] for g in gs],
                                                 cache_stride_cts=stride))
    raws = {g: keys[g][0] for g in gs}
    for h in range(heads):
        for c in range(n_cts):
            want = attention.decode_scores(env.orc, q[h], kc[h * n_cts + c], raw_rlk, raws, d2)
            assert np.array_equal(got[h, c], want), (env.name, h, c)
            assert np.array_equal(got_ext[h, c], want), (env.name, h, c, "transformed cache")


def test_decode_context_match_oracle(env):
    from oracle import attention
    say(f"decode_context {env.name}")
    heads, n_cts, d2 = 2, 3, 64
    raw_rlk, rlk = env.key(70)
    gs = _block_keys(env, d2)
    keys = {g: env.key(200 + i) for i, g in enumerate(gs)}
    a, vc = env.cts(81, heads * n_cts), env.cts(82, heads * n_cts)
    got = env.host(env.ctx.decode_context(env.dev(a), env.dev(vc), heads, n_cts, d2, rlk,
                                          [keys[g][1] for g in gs]))
    ext = env.ctx.cache_extend(env.dev(vc), heads, n_cts, n_cts, env.ctx.empty_ext(heads * n_cts))
    got_ext = env.host(env.ctx.decode_context_ext(env.dev(a), ext, heads, n_cts, d2, rlk, [keys[g][1] for g in gs]))
    raws = {g: keys[g][0] for g in gs}
    for h in range(heads):
        sl = slice(h * n_cts, (h + 1) * n_cts)
        want = attention.decode_context(env.orc, list(a[sl]), list(vc[sl]), raw_rlk, raws, d2)
        assert np.array_equal(got[h], want), (env.name, h)
        assert np.array_equal(got_ext[h], want), (env.name, h, "transformed cache")


def test_prefill_diagonals_match_oracle():
    from oracle import attention
    env = _envs.setdefault("C1", Env("C1")) if "C1" in _envs else Env("C1")
    _envs["C1"] = env
    say("prefill_qk C1 params, d2 = 256 (m = 16 diagonals), 2 heads")
    heads, d2 = 2, 256
    n = env.n
    raw_rlk, rlk = env.key(70)
    gs = _fold_keys(env, d2)
    keys = {g: env.key(300 + i) for i, g in enumerate(gs)}
    g_blk, g_swap = pow(3, d2, 2 * n), 2 * n - 1
    kb, ks = env.key(320), env.key(321)
    q, kk = env.cts(91, heads), env.cts(92, heads)
    got = env.host(env.ctx.prefill_qk(env.dev(q), env.dev(kk), heads, d2, rlk, [keys[g][1] for g in gs],
                                      kb[1], ks[1]))
    raws = {g: keys[g][0] for g in gs}
    raws[g_blk], raws[g_swap] = kb[0], ks[0]
    for h in range(heads):
        want = attention.prefill_qk(env.orc, q[h], kk[h], raw_rlk, raws, d2)
        assert len(want) == n // d2
        for i, w in enumerate(want):
            assert np.array_equal(got[h, i], w), (h, i)


def test_real_ciphertexts_decrypt_to_attention_scores():
    """End to end at the N = 8192 set: GPU scores on real encryptions decrypt to K q mod t."""
    from oracle import Client, attention
    env = _envs.get("C2") or Env("C2")
    _envs["C2"] = env
    say("semantic decode_scores C2")
    prm, n, d2 = env.prm, env.n, 64
    B = n // d2
    cl = Client(prm, 4242, env.orc)
    act = attention_activations(Stream(4242, 1), 1, B + 1, d2)[0]
    qv, K = act[0], act[1:]
    raw_rlk = cl.relin_key()
    gs = _fold_keys(env, d2)
    raw_g = {g: cl.galois_key(g) for g in gs}
    q_ct = cl.encrypt_slots(np.tile(qv, B))
    k_ct = cl.encrypt_slots(K.reshape(-1))
    rlk = env.ctx.ksk_prepare(env.dev(raw_rlk))
    gks = [env.ctx.ksk_prepare(env.dev(raw_g[g])) for g in gs]
    got = env.host(env.ctx.decode_scores(env.dev(q_ct[None]), env.dev(k_ct[None]), 1, 1, d2, rlk, gks))[0, 0]
    assert np.array_equal(got, attention.decode_scores(env.orc, q_ct, k_ct, raw_rlk, raw_g, d2))
    assert np.array_equal(cl.decrypt_slots(got)[::d2], (K @ qv) % prm.t)


def test_full_decode_step_shape_on_sampled_units():
    """The launch configuration the benchmark times (12 heads x 4 cache ciphertexts at N = 8192):
    a sample of output units is recomputed by the oracle one by one."""
    from oracle import attention
    env = _envs.get("C2") or Env("C2")
    _envs["C2"] = env
    say("full-shape decode step, sampled units")
    heads, n_cts, d2 = 12, 4, 64
    raw_rlk, rlk = env.key(70)
    gs = _fold_keys(env, d2)
    keys = {g: env.key(100 + i) for i, g in enumerate(gs)}
    q, kc = env.cts(401, heads), env.cts(402, heads * n_cts)
    got = env.host(env.ctx.decode_scores(env.dev(q), env.dev(kc), heads, n_cts, d2, rlk,
                                         [keys[g][1] for g in gs]))
    raws = {g: keys[g][0] for g in gs}
    for (h, c) in [(0, 0), (5, 2), (11, 3)]:
        want = attention.decode_scores(env.orc, q[h], kc[h * n_cts + c], raw_rlk, raws, d2)
        assert np.array_equal(got[h, c], want), (h, c)
    gb = _block_keys(env, d2)
    bkeys = {g: env.key(200 + i) for i, g in enumerate(gb)}
    a, vc = env.cts(403, heads * n_cts), env.cts(404, heads * n_cts)
    got = env.host(env.ctx.decode_context(env.dev(a), env.dev(vc), heads, n_cts, d2, rlk,
                                          [bkeys[g][1] for g in gb]))
    braws = {g: bkeys[g][0] for g in gb}
    for h in (0, 7, 11):
        sl = slice(h * n_cts, (h + 1) * n_cts)
        want = attention.decode_context(env.orc, list(a[sl]), list(vc[sl]), raw_rlk, braws, d2)
        assert np.array_equal(got[h], want), h


def test_invalid_arguments_are_rejected_without_launching():
    import torch
    from paper_2602_08798_amd.binding import CgError
    env = _envs.get("C1") or Env("C1")
    _envs["C1"] = env
    say("negative tests")
    x = env.dev(env.cts(1, 1))
    raw, gk = env.key(30)
    with pytest.raises(CgError):
        env.ctx.rotate(x, 2, gk, 1)                     # even Galois element
    with pytest.raises(CgError):
        env.ctx.rotate(x, 2 * env.n + 1, gk, 1)         # out of range
    with pytest.raises(CgError):
        env.ctx.rotate(x, 3, gk, 1, out=x)              # in-place is not supported
    x3 = env.dev(env.cts(1, 3))
    with pytest.raises(CgError):
        env.ctx.rotate(x3[:2], 3, gk, 2, out=x3[1:])    # nor is a partial overlap of the two batches
    with pytest.raises(CgError):
        env.ctx.add(x, x, 4, 1)                         # ncomp must be 2 or 3
    with pytest.raises(CgError):
        env.ctx.add(x, x, 2, 0)                         # an empty batch is an error, not a silent no-op
    with pytest.raises(CgError):
        env.ctx.rotate(x, 3, gk, (1 << 16) + 1, out=env.ctx.empty_ct(1))   # above the largest batch
    with pytest.raises(CgError):
        env.ctx.kv_append(x, 1, 1, env.n, x, gk, env.n // 4)   # token beyond the cache
    # unsupported parameter sets never reach the device
    import dataclasses
    P = env.P
    bad = dataclasses.replace(env.prm, q=(env.prm.q[0], env.prm.q[0]))
    with pytest.raises(CgError):
        P.Context(bad)
    bad = dataclasses.replace(env.prm, q=(env.prm.q[0], (1 << 50) - 27))   # not 1 mod 2N
    with pytest.raises(CgError):
        P.Context(bad)
    for composite in (1125899906818049, 1125899906670593):   # 1 mod 2N, 11 * ... and 1733 * 20129 * 32275949
        bad = dataclasses.replace(env.prm, q=(env.prm.q[0], composite))
        with pytest.raises(CgError):
            P.Context(bad)
    bad = dataclasses.replace(env.prm, alpha=2)          # a two-prime digit against one special prime
    with pytest.raises(CgError):
        P.Context(bad)
    torch.cuda.synchronize()


def test_decode_scores_outer_match_oracle(env):
    from oracle import attention
    heads, d2 = 2, 8
    say(f"decode_scores_outer {env.name} d2={d2}")
    n, t = env.n, env.prm.t
    raw_rlk, rlk = env.key(70)
    gs = _fold_keys(env, d2)
    keys = {g: env.key(100 + i) for i, g in enumerate(gs)}
    rng = np.random.default_rng(77)
    masks_pt = rng.integers(0, t, (d2, n), dtype=np.uint64)      # arbitrary plaintexts stand in for the masks
    masks = env.ctx.plain_prepare(env.dev(masks_pt))
    q, cols = env.cts(501, heads), env.cts(502, heads * d2)
    got = env.host(env.ctx.decode_scores_outer(env.dev(q), env.dev(cols), heads, d2, masks, rlk,
                                               [keys[g][1] for g in gs]))
    raws = {g: keys[g][0] for g in gs}
    for h in range(heads):
        want = attention.decode_scores_outer(env.orc, q[h], list(cols[h * d2:(h + 1) * d2]), list(masks_pt),
                                             raw_rlk, raws, d2)
        assert np.array_equal(got[h], want), (env.name, h)


def test_decode_context_outer_match_oracle(env):
    from oracle import attention
    heads, d2 = 2, 3
    say(f"decode_context_outer {env.name} columns={d2}")
    n = env.n
    raw_rlk, rlk = env.key(70)
    gs, sh = [], 1
    while sh <= n // 4:
        gs.append(pow(3, sh, 2 * n))
        sh *= 2
    gs.append(2 * n - 1)
    keys = {g: env.key(600 + i) for i, g in enumerate(gs)}
    a, cols = env.cts(601, heads), env.cts(602, heads * d2)
    got = env.host(env.ctx.decode_context_outer(env.dev(a), env.dev(cols), heads, d2, rlk,
                                                [keys[g][1] for g in gs]))
    raws = {g: keys[g][0] for g in gs}
    for h in range(heads):
        want = attention.decode_context_outer(env.orc, a[h], list(cols[h * d2:(h + 1) * d2]), raw_rlk, raws)
        for j in range(d2):
            assert np.array_equal(got[h, j], want[j]), (env.name, h, j)


@pytest.mark.parametrize("name,heads,d2", [("C1", 2, 256), ("C2", 2, 512)])
def test_prefill_context_match_oracle(name, heads, d2):
    from oracle import attention
    env = _envs.get(name) or Env(name)
    _envs[name] = env
    n = env.n
    m = n // d2
    say(f"prefill_av {name}, d2 = {d2} (m = {m} units per head), {heads} heads")
    raw_rlk, rlk = env.key(70)
    g_blk, g_swap = pow(3, d2, 2 * n), 2 * n - 1
    kb, ks = env.key(320), env.key(321)
    a, v = env.cts(93, heads * m), env.cts(94, heads)
    got = env.host(env.ctx.prefill_av(env.dev(a), env.dev(v), heads, d2, rlk, kb[1], ks[1]))
    raws = {g_blk: kb[0], g_swap: ks[0]}
    for h in range(heads):
        want = attention.prefill_av(env.orc, list(a[h * m:(h + 1) * m]), v[h], raw_rlk, raws, d2)
        assert np.array_equal(got[h], want), (name, h)


@pytest.mark.parametrize("name,heads,d2", [("C1", 2, 256), ("C2", 1, 512), ("C1", 1, 16)])
def test_prefill_repack_match_oracle(name, heads, d2):
    """Groups of min(d2, H) score ciphertexts are compacted; the inputs stay untouched.  The third case
    has more diagonals per slot row (H = 128) than slots per block (16): eight groups per row."""
    from oracle import attention
    env = _envs.get(name) or Env(name)
    _envs[name] = env
    n, t = env.n, env.prm.t
    m = n // d2
    w = min(d2, m // 2)
    say(f"prefill_repack {name}, d2 = {d2}: {heads} x {m} units in groups of {w}")
    shifts = list(attention.right_shifts(w))
    gs = [pow(3, n // 2 - sh, 2 * n) for sh in shifts]
    keys = [env.key(400 + i) for i in range(len(gs))]
    mask_pt = attention.slot0_mask_values(n, d2).astype(np.uint64)
    # an arbitrary plaintext exercises the same path as the encoded mask, which is not sparse either
    rng = np.random.default_rng(95)
    mask_pt = (mask_pt + rng.integers(0, t, n, dtype=np.uint64)) % t
    mask0 = env.ctx.plain_prepare(env.dev(mask_pt[None, :]))
    x = env.cts(96, heads * m)
    dx = env.dev(x)
    got = env.host(env.ctx.prefill_repack(dx, heads, d2, mask0, [k[1] for k in keys]))
    assert np.array_equal(env.host(dx), x)
    raws = {g: k[0] for g, k in zip(gs, keys)}
    assert got.shape[0] == heads * m // w
    for h in range(heads):
        want = attention.prefill_repack(env.orc, list(x[h * m:(h + 1) * m]), mask_pt, raws, d2)
        for i, wv in enumerate(want):
            assert np.array_equal(got[h * (m // w) + i], wv), (name, h, i)


def test_invalid_arguments_of_the_step_and_prompt_entry_points():
    import torch
    from paper_2602_08798_amd.binding import CgError
    env = _envs.get("C1") or Env("C1")
    _envs["C1"] = env
    say("negative tests, composite entry points")
    n, d2 = env.n, 64
    B = n // d2
    heads, n_cts, stride = 1, 1, 2
    x = env.dev(env.cts(1, 2 * heads * stride))
    q = env.dev(env.cts(2, heads))
    rows = env.dev(env.cts(3, 2 * heads))
    raw, key = env.key(30)
    fold = [key] * 6
    block = [key] * (len(_block_keys(env, d2)))
    masks = env.ctx.plain_prepare(env.dev(np.zeros((B, n), dtype=np.uint64)))
    a3 = env.dev(env.cts(4, 3))                          # large enough for every n_cts tried below
    step = lambda **kw: env.ctx.decode_step(q, a3, x, heads, kw.get("n_cts", n_cts), kw.get("stride", stride),
                                            kw.get("d2", d2), kw.get("tau", 0), rows, kw.get("masks", masks), key, fold, block)
    before = env.host(x).copy()
    with pytest.raises(CgError):
        step(tau=stride * B)                             # token beyond the last cache ciphertext
    with pytest.raises(CgError):
        step(n_cts=3)                                    # more ciphertexts than a cache holds
    with pytest.raises(CgError):
        step(d2=48)                                      # block size must be a power of two
    with pytest.raises(CgError):
        env.ctx.decode_step(q, q, x, 1 << 15, 4, 4, d2, 0, rows, masks, key, fold, block)   # batch too large
    with pytest.raises(CgError, match="masks"):
        step(tau=1, masks=masks[:masks.numel() // B])    # prepared masks end before the block in use
    with pytest.raises(CgError):
        env.ctx.cache_extend(x, 2, 3, 2, env.ctx.empty_ext(4))      # group longer than its stride
    with pytest.raises(CgError):
        env.ctx.prefill_av(x, q, 1, 48, key, key, key)
    with pytest.raises(CgError):
        env.ctx.prefill_repack(x, 1, n // 2, masks, [key])     # d2 above N/4
    assert np.array_equal(env.host(x), before)           # nothing was launched on the cache
    torch.cuda.synchronize()


def test_decode_step_edge_shapes_match_oracle():
    """One head and one cache ciphertext; tokens at the first and the last block of a ciphertext; the
    smallest head dimension the fold accepts (d2 = 2: a single fold rotation, log2(N/4) block rotations)
    and the largest (d2 = N/4: two blocks per slot row)."""
    from oracle import attention
    env = _envs.get("C1") or Env("C1")
    _envs["C1"] = env
    n = env.n
    raw_rlk, rlk = env.key(70)
    for d2, taus in ((2, (0, n // 2 - 1)), (n // 4, (0, 3, 4))):
        B = n // d2
        say(f"decode_step edge shapes C1, d2 = {d2}, tokens {taus}")
        gs_f, gs_b = _fold_keys(env, d2), _block_keys(env, d2)
        kf = {g: env.key(500 + i) for i, g in enumerate(gs_f)}
        kb = {g: env.key(520 + i) for i, g in enumerate(gs_b)}
        rng = np.random.default_rng(7 + d2)
        # only the masks the tokens use are prepared (B can be thousands)
        blocks = sorted({t % B for t in taus})
        masks_pt = np.zeros((max(blocks) + 1, n), dtype=np.uint64)
        for b in blocks:
            masks_pt[b] = rng.integers(0, env.prm.t, n, dtype=np.uint64)
        masks = env.ctx.plain_prepare(env.dev(masks_pt))
        heads, stride = 1, 2
        cache = env.cts(600 + d2, 2 * heads * stride)
        want_cache = cache.copy()
        dcache = env.dev(cache)
        for tau in taus:
            idx, blk = divmod(tau, B)
            n_cts = idx + 1                              # the appended ciphertext is read by the products
            q, a, rows = env.cts(610 + tau, heads), env.cts(620 + tau, heads * n_cts), env.cts(630 + tau, 2 * heads)
            scores, context = env.ctx.decode_step(env.dev(q), env.dev(a), dcache, heads, n_cts, stride, d2, tau,
                                                  env.dev(rows), masks, rlk, [kf[g][1] for g in gs_f],
                                                  [kb[g][1] for g in gs_b])
            for c in range(2 * heads):
                masked = env.orc.mul_plain(rows[c], masks_pt[blk])
                want_cache[c * stride + idx] = masked if blk == 0 else env.orc.add(want_cache[c * stride + idx], masked)
            assert np.array_equal(env.host(dcache), want_cache), (d2, tau)
            scores, context = env.host(scores), env.host(context)
            for c in range(n_cts):
                w = attention.decode_scores(env.orc, q[0], want_cache[c], raw_rlk, {g: kf[g][0] for g in gs_f}, d2)
                assert np.array_equal(scores[0, c], w), (d2, tau, c)
            w = attention.decode_context(env.orc, list(a), list(want_cache[stride:stride + n_cts]), raw_rlk,
                                         {g: kb[g][0] for g in gs_b}, d2)
            assert np.array_equal(context[0], w), (d2, tau)


@pytest.mark.parametrize("batch", [5, 9, 23])
def test_rotate_and_mul_relin_at_ragged_batches(batch):
    """Batches whose row and block counts are not multiples of the XCD-aware launch orders' period
    (full periods are permuted, the ragged tail is not): every unit still gets its own result."""
    env = _envs.get("C1") or Env("C1")
    _envs["C1"] = env
    say(f"ragged batch {batch} C1")
    n = env.n
    raw, key = env.key(30)
    x = env.cts(700 + batch, batch)
    g = pow(3, 5, 2 * n)
    got = env.host(env.ctx.rotate(env.dev(x), g, key, batch, accumulate=True))
    for u in range(batch):
        assert np.array_equal(got[u], env.orc.add(x[u], env.orc.rotate(x[u], g, raw))), (batch, u)
    y = env.cts(800 + batch, batch)
    got = env.host(env.ctx.mul_relin(env.dev(x), env.dev(y), key, batch))
    for u in range(batch):
        assert np.array_equal(got[u], env.orc.relin(env.orc.mul(x[u], y[u]), raw)), (batch, u)


def test_decode_step_random_shapes_match_oracle():
    """Seeded sweep over heads, ciphertexts read, cache stride, head dimension and token position (also
    with the transformed copy of the cache), each compared in full with the oracle's step."""
    from oracle import run_configs
    import torch
    env = _envs.get("C1") or Env("C1")
    _envs["C1"] = env
    n = env.n
    rng = np.random.default_rng(2026)
    raw_rlk, rlk = env.key(70)
    for case in range(6):
        d2 = int(rng.choice([16, 64, 256, 1024]))
        B = n // d2
        heads = int(rng.integers(1, 4))
        n_cts = int(rng.integers(1, 4))
        stride = n_cts + int(rng.integers(0, 3))
        tau = int(rng.integers(0, stride * B))
        use_ext = bool(case % 2)
        say(f"decode_step sweep {case}: heads {heads}, n_cts {n_cts}, stride {stride}, d2 {d2}, tau {tau}, ext {use_ext}")
        gs_f, gs_b = _fold_keys(env, d2), _block_keys(env, d2)
        kf = {g: env.key(900 + i) for i, g in enumerate(gs_f)}
        kb = {g: env.key(930 + i) for i, g in enumerate(gs_b)}
        blk = tau % B
        mask_pt = rng.integers(0, env.prm.t, n, dtype=np.uint64)
        # prepared masks are indexed by block: only the one in use is filled in, at its index
        one = env.ctx.plain_prepare(env.dev(mask_pt[None, :]))          # flat: k * n doubles
        per = one.numel()
        masks_dev = torch.zeros((blk + 1) * per, dtype=one.dtype, device=one.device)
        masks_dev[blk * per:(blk + 1) * per] = one
        q, a = env.cts(1000 + case, heads), env.cts(1100 + case, heads * n_cts)
        rows, cache = env.cts(1200 + case, 2 * heads), env.cts(1300 + case, 2 * heads * stride)
        dcache = env.dev(cache)
        ext = None
        if use_ext:
            ext = env.ctx.empty_ext(2 * heads * stride)
            env.ctx.cache_extend(dcache, 2 * heads, n_cts, stride, ext)
        scores, context = env.ctx.decode_step(env.dev(q), env.dev(a), dcache, heads, n_cts, stride, d2, tau,
                                              env.dev(rows), masks_dev, rlk, [kf[g][1] for g in gs_f],
                                              [kb[g][1] for g in gs_b], cache_ext=ext)
        st = {"heads": heads, "stride": stride, "B": B, "d2": d2, "fold": gs_f, "block": gs_b,
              "masks": {blk: mask_pt}, "rlk": raw_rlk,
              "gk": {**{g: kf[g][0] for g in gs_f}, **{g: kb[g][0] for g in gs_b}}}
        # (when the appended ciphertext lies beyond those read, append and products commute)
        want, wcache = {}, cache.copy()
        run_configs._decode_step(env.orc, st, q, a, wcache, rows, tau, n_cts, want)
        scores, context, got_cache = env.host(scores), env.host(context), env.host(dcache)
        assert np.array_equal(got_cache, wcache), case
        for h in range(heads):
            for c in range(n_cts):
                assert np.array_equal(scores[h, c], want[f"score{h}_{c}"]), (case, h, c)
            assert np.array_equal(context[h], want[f"context{h}"]), (case, h)


def test_binding_rejects_undersized_tensors_before_any_launch():
    """Pointers cross the C ABI without sizes: the binding compares every tensor with what the
    call's arguments imply and raises instead of letting a kernel run off the end of a buffer."""
    from paper_2602_08798_amd.binding import CgSizeError
    env = _envs.get("C1") or Env("C1")
    _envs["C1"] = env
    say("undersized tensors")
    x2 = env.dev(env.cts(5, 2))
    raw, key = env.key(31)
    with pytest.raises(CgSizeError, match="b"):
        env.ctx.mul(x2, x2[:1], 2)
    with pytest.raises(CgSizeError, match="a"):
        env.ctx.mul_relin(x2[:1], x2, key, 2)            # a_group 1: one a operand per product
    env.ctx.mul_relin(x2[:1], x2, key, 2, a_group=2)     # shared a operand: fits
    with pytest.raises(CgSizeError, match="in"):
        env.ctx.rotate(x2, 3, key, 3)
    with pytest.raises(CgSizeError, match="gk"):
        env.ctx.rotate(x2, 3, key[:key.numel() // 2], 2)
    with pytest.raises(CgSizeError, match="out"):
        env.ctx.add(x2, x2, 2, 2, out=env.ctx.empty_ct(1))
    with pytest.raises(CgSizeError, match="cache"):
        env.ctx.decode_scores(x2, x2, 2, 1, 64, key, [key] * 6, cache_stride_cts=2)   # 2 heads, stride 2: 3 cts
    with pytest.raises(CgSizeError, match="ext"):
        env.ctx.cache_extend(x2, 1, 2, 2, env.ctx.empty_ext(1))
    import torch
    torch.cuda.synchronize()


@pytest.mark.parametrize("name,d1,d2,units", [("C1", 200, 64, 3), ("C1", 1000, 64, 2), ("C1", 100, 16, 5),
                                             ("C1", 37, 256, 1), ("C2", 768, 64, 6), ("C5", 1024, 64, 2)])
def test_cpvm_matches_oracle(name, d1, d2, units):
    """The decode step's ciphertext-plaintext vector-matrix product (section 4.2) against the oracle's
    procedure, on pseudo-ciphertexts and pseudo-keys (bit-exactness needs no valid encryption);
    the paper's sizes (768 x 64 at N = 8192) are the C2 case."""
    from oracle import attention
    from oracle.client import SlotCodec
    env = _envs.get(name) or Env(name)
    _envs[name] = env
    n = env.n
    D1, T, C = attention.cpvm_shape(n, d1, d2)
    say(f"cpvm {name}: d1 {d1}, d2 {d2}, tile {D1}, {C} diagonals, {units} matrices")
    codec = SlotCodec(env.prm)
    g = Stream(1500 + d1, units)
    polys = np.stack([codec.encode(attention.cpvm_weight_values(n, d1, d2, g.integers(-128, 128, (d1, d2)), c))
                      for u in range(units) for c in range(C)])
    x = env.cts(1501 + d1, 1)[0]
    g_shift = [pow(3, sh, 2 * n) for sh in attention.cpvm_shifts(C)]
    g_block = _block_keys(env, d2)
    keys = {gal: env.key(1600 + i) for i, gal in enumerate(sorted(set(g_shift + g_block)))}
    got = env.host(env.ctx.cpvm(env.dev(x[None]), env.ctx.plain_prepare(env.dev(polys)), units, C, d2,
                                [keys[gal][1] for gal in g_shift], [keys[gal][1] for gal in g_block]))
    raw = {gal: keys[gal][0] for gal in keys}
    for u in range(units):
        want = attention.cpvm(env.orc, x, list(polys[u * C:(u + 1) * C]), raw, d2)
        assert np.array_equal(got[u], want), (name, d1, d2, u)


def test_cpvm_rejects_invalid_arguments():
    from paper_2602_08798_amd.binding import CgError
    env = _envs.get("C1") or Env("C1")
    _envs["C1"] = env
    say("cpvm negative tests")
    raw, key = env.key(30)
    x = env.dev(env.cts(1, 1))
    plain = env.ctx.plain_prepare(env.dev(np.zeros((4, env.n), dtype=np.uint64)))
    block = [key] * len(_block_keys(env, 64))
    with pytest.raises(CgError):
        env.ctx.cpvm(x, plain, 1, 3, 64, [key, key], block)          # diagonals: a power of two
    with pytest.raises(CgError):
        env.ctx.cpvm(x, plain, 1, 4, 48, [key, key], block)          # d2: a power of two
    with pytest.raises(CgError):
        env.ctx.cpvm(x, plain, 1, 4, 2, [key, key], block)           # more diagonals than outputs
    with pytest.raises(CgError, match="diags"):
        env.ctx.cpvm(x, plain, 2, 4, 64, [key, key], block)          # two matrices need eight diagonals
    import torch
    torch.cuda.synchronize()


def test_one_head_of_a_decode_layer_on_real_encryptions():
    """The pieces in the order a decode layer uses them (section 4.1's workflow), on real encryptions
    at the N = 8192 set: CT x PT projections of the token, append of the new key and value, scores
    against the cache, (client: decrypt, pick integer weights, re-encrypt them broadcast per block),
    context.  What the client decrypts must be the plaintext attention arithmetic modulo t."""
    from oracle import Client, attention
    env = _envs.get("C2") or Env("C2")
    _envs["C2"] = env
    say("semantic decode layer C2 (one head)")
    prm, n, t, d1, d2 = env.prm, env.n, env.prm.t, 768, 64
    B = n // d2
    tau = 5                                             # the cache holds tokens 0..4; the new token is 5
    cl = Client(prm, 777, env.orc)
    g = Stream(777, 1)
    x = g.integers(-8, 8, d1)
    W = [g.integers(-8, 8, (d1, d2)) for _ in range(3)]            # Wq, Wk, Wv
    Kc, Vc = g.integers(-8, 8, (tau, d2)), g.integers(-8, 8, (tau, d2))
    D1, T, C = attention.cpvm_shape(n, d1, d2)
    gals = sorted(set(attention.cpvm_galois(n, C, d2)) | set(attention.required_galois(n, d2)))
    say(f"  {len(gals)} Galois keys")
    raw_g = {gal: cl.galois_key(gal) for gal in gals}
    key = {gal: env.ctx.ksk_prepare(env.dev(raw_g[gal])) for gal in gals}
    rlk = env.ctx.ksk_prepare(env.dev(cl.relin_key()))
    fold = [key[gal] for gal in _fold_keys(env, d2)]
    block = [key[gal] for gal in _block_keys(env, d2)]
    shift = [key[pow(3, sh, 2 * n)] for sh in attention.cpvm_shifts(C)]
    # projections: q, k, v tiled with period d2
    diags = np.stack([cl.codec.encode(attention.cpvm_weight_values(n, d1, d2, Wm, c)) for Wm in W for c in range(C)])
    x_ct = cl.encrypt_slots(attention.cpvm_token_values(n, d1, d2, x))
    qkv = env.ctx.cpvm(env.dev(x_ct[None]), env.ctx.plain_prepare(env.dev(diags)), 3, C, d2, shift, block)
    q_want, k_want, v_want = [(x @ Wm) % t for Wm in W]
    assert np.array_equal(cl.decrypt_slots(env.host(qkv)[0]), np.tile(q_want, B))
    # caches of the head (K then V), tokens 0..tau-1 in blocks 0..tau-1; append the new rows
    pad = lambda M: np.concatenate([M.reshape(-1), np.zeros(n - M.size, dtype=np.int64)])
    cache = env.dev(np.stack([cl.encrypt_slots(pad(Kc)), cl.encrypt_slots(pad(Vc))]))
    per = env.k * n
    import torch
    one = env.ctx.plain_prepare(env.dev(cl.codec.encode(attention.block_mask_values(n, d2, tau))[None, :]))
    masks = torch.zeros((tau + 1) * per, dtype=one.dtype, device=one.device)
    masks[tau * per:] = one
    env.ctx.kv_append(cache, 1, 2, tau, qkv[1:], masks, d2)
    Kn, Vn = np.vstack([Kc, k_want]), np.vstack([Vc, v_want])
    assert np.array_equal(cl.decrypt_slots(env.host(cache)[0]), pad(Kn) % t)
    # scores of the projected query against the cache that now includes the new token
    scores = env.ctx.decode_scores(qkv[:1], cache[:1], 1, 1, d2, rlk, fold)
    s = cl.decrypt_slots(env.host(scores)[0, 0])[::d2]
    assert np.array_equal(s[:tau + 1], (Kn @ q_want) % t)
    # the client's turn: integer weights from the scores (any function will do), broadcast per block
    a = (s[:tau + 1] % 7).astype(np.int64)
    a_ct = cl.encrypt_slots(np.concatenate([np.repeat(a, d2), np.zeros(n - (tau + 1) * d2, dtype=np.int64)]))
    ctxt = env.ctx.decode_context(env.dev(a_ct[None]), cache[1:], 1, 1, d2, rlk, block)
    got = cl.decrypt_slots(env.host(ctxt)[0])
    assert np.array_equal(got, np.tile((a @ Vn) % t, B))
    assert cl.noise_budget_bits(env.host(ctxt)[0], cl.decrypt_poly(env.host(ctxt)[0])) > 10
