"""Full-size launch shapes of the prefill (C3) and scaled-up decode (C5) configurations.

The GPU runs the whole batch; the oracle recomputes a sample of output units one by one."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from workloads import PRESETS, Stream, pseudo_ciphertexts, pseudo_switch_key


def say(msg):
    print(f"[gpu-full] {msg}", flush=True)
    sys.stdout.flush()


def _keys(ctx, P, prm, seed, gals):
    qp = list(prm.q) + list(prm.p)
    raw = {g: pseudo_switch_key(Stream(seed, 7, i), qp, prm.n, prm.dnum) for i, g in enumerate(gals)}
    dev = {g: ctx.ksk_prepare(P.to_device(k)) for g, k in raw.items()}
    return raw, dev


def test_prefill_12_heads_128_tokens_sampled():
    import torch
    import paper_2602_08798_amd as P
    from oracle import Oracle
    prm = PRESETS["C3"]
    n, d2, heads = prm.n, 64, 12
    m, H = n // d2, n // d2 // 2
    say(f"prefill C3: {heads} heads x {m} diagonals, workspace {heads * m} units")
    ctx, orc = P.Context(prm), Oracle(prm)
    fold = [pow(3, 1 << j, 2 * n) for j in range(6)]
    g_blk, g_swap = pow(3, d2, 2 * n), 2 * n - 1
    raw, dev = _keys(ctx, P, prm, 33, ["rlk"] + fold + [g_blk, g_swap])
    q = pseudo_ciphertexts(Stream(33, 1), prm.q, n, heads)
    kk = pseudo_ciphertexts(Stream(33, 2), prm.q, n, heads)
    out = ctx.prefill_qk(P.to_device(q), P.to_device(kk), heads, d2, dev["rlk"], [dev[g] for g in fold],
                         dev[g_blk], dev[g_swap])
    torch.cuda.synchronize()
    for (h, sigma, r) in [(0, 0, 0), (5, 1, 3), (11, 0, H - 1), (7, 1, H - 1)]:
        say(f"  oracle unit head={h} sigma={sigma} r={r}")
        kr = kk[h]
        for _ in range(r):
            kr = orc.rotate(kr, g_blk, raw[g_blk])
        if sigma:
            kr = orc.rotate(kr, g_swap, raw[g_swap])
        x = orc.relin(orc.mul(q[h], kr), raw["rlk"])
        for g in fold:
            x = orc.add(x, orc.rotate(x, g, raw[g]))
        got = P.to_host(out[h, sigma * H + r])
        assert np.array_equal(got, x), (h, sigma, r)
    del out
    ctx._ws = None
    torch.cuda.empty_cache()


def test_scaled_decode_steps_with_cache_growth_sampled():
    """C5: 16 heads, N = 16384, 6+2 primes, alpha = 2; three successive steps starting at 512 tokens."""
    import torch
    import paper_2602_08798_amd as P
    from oracle import Oracle, attention
    prm = PRESETS["C5"]
    n, d2, heads = prm.n, 64, 16
    B = n // d2                       # 256 tokens per cache ciphertext
    stride = 3
    say(f"decode steps C5: {heads} heads, B = {B}")
    ctx, orc = P.Context(prm), Oracle(prm)
    fold = [pow(3, 1 << j, 2 * n) for j in range(6)]
    blk, sh = [], d2
    while sh <= n // 4:
        blk.append(pow(3, sh, 2 * n))
        sh *= 2
    blk.append(2 * n - 1)
    raw, dev = _keys(ctx, P, prm, 55, ["rlk"] + fold + blk)
    rng = np.random.default_rng(55)
    masks_pt = rng.integers(0, prm.t, (4, n), dtype=np.uint64)     # blocks 0..3 are the ones used
    masks = ctx.plain_prepare(P.to_device(masks_pt))
    h_cache = pseudo_ciphertexts(Stream(55, 3), prm.q, n, 2 * heads * stride)   # [K|V][head][stride]
    cache = P.to_device(h_cache)
    want_cache = h_cache.copy()
    for step in range(3):
        tau = 512 + step
        idx, b = divmod(tau, B)
        rows = pseudo_ciphertexts(Stream(55, 4, step), prm.q, n, 2 * heads)
        q = pseudo_ciphertexts(Stream(55, 5, step), prm.q, n, heads)
        n_cts = idx + 1
        a = pseudo_ciphertexts(Stream(55, 6, step), prm.q, n, heads * n_cts)
        say(f"  step {step}: tau = {tau}, {n_cts} cache ciphertexts per head")
        ctx.kv_append(cache, stride, 2 * heads, tau, P.to_device(rows), masks, d2)
        scores = ctx.decode_scores(P.to_device(q), cache[:heads * stride], heads, n_cts, d2, dev["rlk"],
                                   [dev[g] for g in fold], cache_stride_cts=stride)
        context = ctx.decode_context(P.to_device(a), cache[heads * stride:], heads, n_cts, d2, dev["rlk"],
                                     [dev[g] for g in blk], cache_stride_cts=stride)
        torch.cuda.synchronize()
        # oracle: the append for every cache (cheap), then sampled attention units
        for c in range(2 * heads):
            masked = orc.mul_plain(rows[c], masks_pt[b])
            tgt = c * stride + idx
            want_cache[tgt] = masked if b == 0 else orc.add(want_cache[tgt], masked)
        assert np.array_equal(P.to_host(cache), want_cache), f"cache after step {step}"
        h, c = (3 * step + 1) % heads, step % n_cts
        wanted = attention.decode_scores(orc, q[h], want_cache[h * stride + c], raw["rlk"],
                                         {g: raw[g] for g in fold}, d2)
        assert np.array_equal(P.to_host(scores[h, c]), wanted), ("scores", step, h, c)
        h = (5 * step + 2) % heads
        v0 = (heads + h) * stride
        wanted = attention.decode_context(orc, list(a[h * n_cts:(h + 1) * n_cts]),
                                          list(want_cache[v0:v0 + n_cts]), raw["rlk"],
                                          {g: raw[g] for g in blk}, d2)
        assert np.array_equal(P.to_host(context[h]), wanted), ("context", step, h)
