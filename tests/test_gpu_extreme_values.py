"""Inputs chosen to push the lazily reduced arithmetic to its bounds: every residue at q - 1, at the
middle of the range, alternating extremes, a single spike -- for ciphertexts and for keys alike.  The
transforms carry values of up to 8 p unreduced, so worst-case magnitudes (which random residues almost
never produce) are where a wrong bound would show."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from workloads import PRESETS


def say(msg):
    print(f"[gpu-extreme] {msg}", flush=True)
    sys.stdout.flush()


def patterns(mods, n, shape_lead):
    """name -> array [*shape_lead][len(mods)][n] of canonical residues"""
    out = {}
    mods = [int(m) for m in mods]

    def fill(f):
        a = np.empty(tuple(shape_lead) + (len(mods), n), dtype=np.uint64)
        for i, m in enumerate(mods):
            a[..., i, :] = f(m)
        return a

    out["all q-1"] = fill(lambda m: np.full(n, m - 1, dtype=np.uint64))
    out["all (q-1)/2"] = fill(lambda m: np.full(n, (m - 1) // 2, dtype=np.uint64))
    out["all (q+1)/2"] = fill(lambda m: np.full(n, (m + 1) // 2, dtype=np.uint64))
    alt = np.arange(n) % 2
    out["alternating 0, q-1"] = fill(lambda m: (alt * (m - 1)).astype(np.uint64))
    out["alternating 1, q-1"] = fill(lambda m: np.where(alt == 1, m - 1, 1).astype(np.uint64))
    spike = np.zeros(n, dtype=np.uint64)
    out["spike q-1 at the last coefficient"] = fill(lambda m: np.concatenate([spike[:-1], [np.uint64(m - 1)]]))
    return out


@pytest.mark.parametrize("name", ["C1", "C2", "C5"])
def test_products_and_key_switches_at_extreme_residues(name):
    import paper_2602_08798_amd as P
    from oracle import Oracle
    prm = PRESETS[name]
    n, k = prm.n, prm.k
    qp = list(prm.q) + list(prm.p)
    ctx, orc = P.Context(prm), Oracle(prm)
    cts = patterns(prm.q, n, (2,))                  # one ciphertext per pattern
    keys = patterns(qp, n, (prm.dnum, 2))           # one switching key per pattern
    g = pow(3, 7, 2 * n)
    for kname, raw in keys.items():
        key = ctx.ksk_prepare(P.to_device(raw))
        names = list(cts)
        a = np.stack([cts[x] for x in names])
        b = np.stack([cts[names[(i + 1) % len(names)]] for i in range(len(names))])
        say(f"{name}: key '{kname}', {len(names)} ciphertext patterns")
        got_mr = P.to_host(ctx.mul_relin(P.to_device(a), P.to_device(b), key, len(names)))
        got_rot = P.to_host(ctx.rotate(P.to_device(a), g, key, len(names), accumulate=True))
        for i, x in enumerate(names):
            want = orc.relin(orc.mul(a[i], b[i]), raw)
            assert np.array_equal(got_mr[i], want), (name, kname, x, "mul_relin")
            want = orc.add(a[i], orc.rotate(a[i], g, raw))
            assert np.array_equal(got_rot[i], want), (name, kname, x, "rotate")
    # transforms of the same patterns, there and back
    L = len(qp)
    allrows = np.concatenate([v.reshape(-1, n) for v in patterns(qp, n, ()).values()])  # [patterns * L][n]
    idx = [i % L for i in range(allrows.shape[0])]
    fwd = ctx.ntt_forward(P.to_device(allrows), idx)
    back = P.to_host(ctx.ntt_inverse(fwd, idx))
    assert np.array_equal(back, allrows)
    from oracle import bfv
    f = P.to_host(fwd)
    for r in (0, L + 1, len(idx) - 1):
        assert np.array_equal(f[r], bfv.ntt_forward(allrows[r], qp[idx[r]])), (name, r)
    ctx.close()
