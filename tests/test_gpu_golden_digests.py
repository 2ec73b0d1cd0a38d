"""All five benchmark configurations, every output ciphertext, bit for bit.

tests/golden/digests_<config>.json holds SHA-256 digests written by a committed script that calls
only the CPU oracle.  Here the HIP library recomputes the same outputs from the same seeded inputs
(workloads.configs) in the launch configuration bench.py uses, and every digest must match."""
import hashlib
import json
import os
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from workloads import configs

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def say(msg):
    print(f"[gpu-golden] {msg}", flush=True)
    sys.stdout.flush()


def digest(arr) -> str:
    return hashlib.sha256(np.ascontiguousarray(arr, dtype="<u8").tobytes()).hexdigest()


def load(name):
    path = os.path.join(GOLDEN, f"digests_{name}.json")
    if not os.path.exists(path):
        pytest.skip(f"{path} not generated (python -m tests.golden.make_digests {name})")
    return json.load(open(path))["digests"]


def compare(got: dict, want: dict, name):
    assert set(got) == set(want), (name, sorted(set(got) ^ set(want))[:5])
    bad = [k for k in want if got[k] != want[k]]
    assert not bad, (name, len(bad), bad[:5])


class Gpu:
    def __init__(self, prm):
        import paper_2602_08798_amd as P
        import torch
        self.P, self.torch = P, torch
        self.ctx = P.Context(prm)

    def dev(self, a):
        return self.P.to_device(a)

    def host(self, t):
        self.torch.cuda.synchronize()
        return self.P.to_host(t)

    def key(self, raw):
        return self.ctx.ksk_prepare(self.dev(raw))


def test_c1_sixteen_mult_relin_pairs():
    say("C1")
    inp, want = configs.c1_inputs(), load("C1")
    g = Gpu(inp["prm"])
    out = g.host(g.ctx.mul_relin(g.dev(inp["a"]), g.dev(inp["b"]), g.key(inp["rlk"]), len(inp["a"])))
    compare({f"pair{u}": digest(out[u]) for u in range(len(out))}, want, "C1")


def _decode_state(g, st):
    gk = {gal: g.key(k) for gal, k in st["gk"].items()}
    return {"rlk": g.key(st["rlk"]), "fold": [gk[x] for x in st["fold"]], "block": [gk[x] for x in st["block"]],
            "masks": g.ctx.plain_prepare(g.dev(st["masks"]))}


def test_c2_decode_scores_one_head_one_ciphertext():
    say("C2")
    st, want = configs.c2_inputs(), load("C2")
    g = Gpu(st["prm"])
    d = _decode_state(g, st)
    cache = g.dev(st["cache"])
    out = g.host(g.ctx.decode_scores(g.dev(st["q"]), cache, 1, 1, st["d2"], d["rlk"], d["fold"],
                                     cache_stride_cts=st["stride"]))
    compare({"score0_0": digest(out[0, 0])}, want, "C2")


def test_c4_full_decode_step_every_output():
    say("C4")
    st, want = configs.c4_inputs(), load("C4")
    g = Gpu(st["prm"])
    d = _decode_state(g, st)
    H, C, S, d2 = st["heads"], st["n_cts"], st["stride"], st["d2"]
    cache = g.dev(st["cache"])
    scores = g.ctx.decode_scores(g.dev(st["q"]), cache[:H * S], H, C, d2, d["rlk"], d["fold"], cache_stride_cts=S)
    context = g.ctx.decode_context(g.dev(st["a"]), cache[H * S:], H, C, d2, d["rlk"], d["block"], cache_stride_cts=S)
    g.ctx.kv_append(cache, S, 2 * H, st["tau"], g.dev(st["rows"]), d["masks"], d2)
    scores, context, cache_h = g.host(scores), g.host(context), g.host(cache)
    got = {}
    for h in range(H):
        for c in range(C):
            got[f"score{h}_{c}"] = digest(scores[h, c])
        got[f"context{h}"] = digest(context[h])
    idx = st["tau"] // st["B"]
    for c in range(2 * H):
        got[f"cache{c}"] = digest(cache_h[c * S + idx])
    compare(got, want, "C4")


@pytest.mark.parametrize("sum_first", [False, True], ids=["C4H", "C4HS"])
def test_c4_full_decode_step_in_hoisted_form_every_output(sum_first):
    """The step as bench.py's headline runs it: one call, three streams, folding sums in rounds of
    hoisted rotation sums, the products reading the cache's transformed copy; without and with the
    context's products summed before their scaling (the headline has them summed)."""
    name = "C4HS" if sum_first else "C4H"
    say(name)
    st, want = configs.c4_inputs(), load(name)
    g = Gpu(st["prm"])
    d = _decode_state(g, st)
    H, C, S, d2 = st["heads"], st["n_cts"], st["stride"], st["d2"]
    wf, wb = configs.C4_ROUND_BITS
    g_fold, g_block = g.ctx.round_galois(0, d2, wf), g.ctx.round_galois(1, d2, wb)
    raw = configs.galois_keys("C4", sorted(set(g_fold + g_block)))
    keys = {gal: g.key(k) for gal, k in raw.items()}
    cache = g.dev(st["cache"])
    ext = g.ctx.cache_extend(cache, 2 * H, C, S, g.ctx.empty_ext(2 * H * S))
    scores, context = g.ctx.decode_step_hoisted(g.dev(st["q"]), g.dev(st["a"]), cache, H, C, S, d2, st["tau"],
                                                g.dev(st["rows"]), d["masks"], d["rlk"], wf, [keys[x] for x in g_fold],
                                                wb, [keys[x] for x in g_block], cache_ext=ext,
                                                sum_before_scaling=sum_first)
    scores, context, cache_h = g.host(scores), g.host(context), g.host(cache)
    got = {}
    for h in range(H):
        for c in range(C):
            got[f"score{h}_{c}"] = digest(scores[h, c])
        got[f"context{h}"] = digest(context[h])
    idx = st["tau"] // st["B"]
    for c in range(2 * H):
        got[f"cache{c}"] = digest(cache_h[c * S + idx])
    compare(got, want, name)


def test_c3_prefill_appends_diagonals_compaction_and_context():
    say("C3")
    st, want = configs.c3_inputs(), load("C3")
    g = Gpu(st["prm"])
    H, m, d2 = st["heads"], st["m"], st["d2"]
    masks = g.ctx.plain_prepare(g.dev(st["masks"]))
    cache = g.ctx.empty_ct(2 * H)                       # one ciphertext per cache, opened by token 0
    for tau in range(m):
        g.ctx.kv_append(cache, 1, 2 * H, tau, g.dev(st["rows"][tau]), masks, d2)
    gk = {gal: g.key(k) for gal, k in st["gk"].items()}
    out = g.ctx.prefill_qk(g.dev(st["q"]), cache[:H], H, d2, g.key(st["rlk"]), [gk[x] for x in st["fold"]],
                           gk[st["g_blk"]], gk[st["g_swap"]])
    gkr = [g.key(st["gk_right"][x]) for x in st["right"]]
    mask0 = g.ctx.plain_prepare(g.dev(st["mask0"][None, :]))
    packed = g.ctx.prefill_repack(out, H, d2, mask0, gkr)
    av = g.ctx.prefill_av(g.dev(st["a"]), cache[H:], H, d2, g.key(st["rlk"]), gk[st["g_blk"]], gk[st["g_swap"]])
    cache_h, out, packed, av = g.host(cache), g.host(out), g.host(packed), g.host(av)
    got = {f"cache{c}": digest(cache_h[c]) for c in range(2 * H)}
    per_head = packed.shape[0] // H
    for h in range(H):
        for i in range(m):
            got[f"qk{h}_{i}"] = digest(out[h, i])
        for i in range(per_head):
            got[f"packed{h}_{i}"] = digest(packed[h * per_head + i])
        got[f"av{h}"] = digest(av[h])
    compare(got, want, "C3")


def test_c5_scaled_decode_steps_with_cache_growth():
    from tests.golden.make_digests import C5_STEPS
    say("C5")
    st, want = configs.c5_inputs(), load("C5")
    g = Gpu(st["prm"])
    d = _decode_state(g, st)
    H, S, d2, B = st["heads"], st["stride"], st["d2"], st["B"]
    cache = g.dev(st["cache"])
    got = {}
    for i in range(C5_STEPS):
        si = st["step_inputs"](i)
        tau, C = 512 + i, si["n_cts"]
        g.ctx.kv_append(cache, S, 2 * H, tau, g.dev(si["rows"]), d["masks"], d2)
        scores = g.ctx.decode_scores(g.dev(si["q"]), cache[:H * S], H, C, d2, d["rlk"], d["fold"], cache_stride_cts=S)
        context = g.ctx.decode_context(g.dev(si["a"]), cache[H * S:], H, C, d2, d["rlk"], d["block"],
                                       cache_stride_cts=S)
        scores, context, cache_h = g.host(scores), g.host(context), g.host(cache)
        idx = tau // B
        for c in range(2 * H):
            got[f"s{i}_cache{c}"] = digest(cache_h[c * S + idx])
        for h in range(H):
            for c in range(C):
                got[f"s{i}_score{h}_{c}"] = digest(scores[h, c])
            got[f"s{i}_context{h}"] = digest(context[h])
    compare(got, want, "C5")


@pytest.mark.parametrize("transformed_cache", [False, True])
def test_c4_decode_step_entry_point_three_branches(transformed_cache):
    """The one-call step (append of token 512 opens ciphertext 5, so all three branches run
    side by side) against the same digests; also with the cache's transformed copy beside it."""
    say(f"C4 decode_step transformed_cache={transformed_cache}")
    st, want = configs.c4_inputs(), load("C4")
    g = Gpu(st["prm"])
    d = _decode_state(g, st)
    H, C, S, d2 = st["heads"], st["n_cts"], st["stride"], st["d2"]
    cache = g.dev(st["cache"])
    q, a, rows = g.dev(st["q"]), g.dev(st["a"]), g.dev(st["rows"])
    ext = None
    if transformed_cache:
        ext = g.ctx.empty_ext(2 * H * S)
        ext.fill_(float("nan"))
        g.ctx.cache_extend(cache, 2 * H, C, S, ext)      # the ciphertexts the products read
    for rep in range(2):    # the second call reuses streams, events and workspace
        cache.copy_(g.dev(st["cache"]))
        scores, context = g.ctx.decode_step(q, a, cache, H, C, S, d2, st["tau"], rows, d["masks"], d["rlk"],
                                            d["fold"], d["block"], cache_ext=ext)
        scores, context, cache_h = g.host(scores), g.host(context), g.host(cache)
        got = {}
        for h in range(H):
            for c in range(C):
                got[f"score{h}_{c}"] = digest(scores[h, c])
            got[f"context{h}"] = digest(context[h])
        idx = st["tau"] // st["B"]
        for c in range(2 * H):
            got[f"cache{c}"] = digest(cache_h[c * S + idx])
        compare(got, want, f"C4 decode_step call {rep}")


@pytest.mark.parametrize("transformed_cache", [False, True])
def test_c5_decode_step_entry_point_append_feeds_products(transformed_cache):
    """The one-call step where the appended ciphertext is read by the products (append first,
    then two branches), over successive steps with cache growth; with a transformed copy of
    the cache, the copy of the growing ciphertext has to be refreshed by every step."""
    from tests.golden.make_digests import C5_STEPS
    say(f"C5 decode_step transformed_cache={transformed_cache}")
    st, want = configs.c5_inputs(), load("C5")
    g = Gpu(st["prm"])
    d = _decode_state(g, st)
    H, S, d2, B = st["heads"], st["stride"], st["d2"], st["B"]
    cache = g.dev(st["cache"])
    ext = None
    if transformed_cache:
        ext = g.ctx.empty_ext(2 * H * S)
        ext.fill_(float("nan"))
        g.ctx.cache_extend(cache, 2 * H, 512 // B, S, ext)   # the full ciphertexts; the growing one is refreshed per step
    got = {}
    for i in range(C5_STEPS):
        si = st["step_inputs"](i)
        tau, C = 512 + i, si["n_cts"]
        assert tau // B < C
        scores, context = g.ctx.decode_step(g.dev(si["q"]), g.dev(si["a"]), cache, H, C, S, d2, tau,
                                            g.dev(si["rows"]), d["masks"], d["rlk"], d["fold"], d["block"],
                                            cache_ext=ext)
        scores, context, cache_h = g.host(scores), g.host(context), g.host(cache)
        idx = tau // B
        for c in range(2 * H):
            got[f"s{i}_cache{c}"] = digest(cache_h[c * S + idx])
        for h in range(H):
            for c in range(C):
                got[f"s{i}_score{h}_{c}"] = digest(scores[h, c])
            got[f"s{i}_context{h}"] = digest(context[h])
    compare(got, want, "C5 decode_step")


def test_c5_first_steps_in_hoisted_form_with_cache_growth():
    """The scaled configuration through cg_decode_step_hoisted (rounds of hoisted rotation sums, the
    context's products summed before one scaling, the cache's transformed copy refreshed per step):
    the appended ciphertext is read by the same step's products."""
    from tests.golden.make_digests import C5H_STEPS
    say("C5 hoisted")
    st, want = configs.c5_inputs(), load("C5H")
    g = Gpu(st["prm"])
    d = _decode_state(g, st)
    H, S, d2, B = st["heads"], st["stride"], st["d2"], st["B"]
    wf, wb = configs.C4_ROUND_BITS
    g_fold, g_block = g.ctx.round_galois(0, d2, wf), g.ctx.round_galois(1, d2, wb)
    raw = configs.galois_keys("C5", sorted(set(g_fold + g_block)))
    keys = {gal: g.key(k) for gal, k in raw.items()}
    kf, kb = [keys[x] for x in g_fold], [keys[x] for x in g_block]
    cache = g.dev(st["cache"])
    ext = g.ctx.empty_ext(2 * H * S)
    ext.fill_(float("nan"))
    g.ctx.cache_extend(cache, 2 * H, 512 // B, S, ext)
    got = {}
    for i in range(C5H_STEPS):
        si = st["step_inputs"](i)
        tau, C = 512 + i, si["n_cts"]
        scores, context = g.ctx.decode_step_hoisted(g.dev(si["q"]), g.dev(si["a"]), cache, H, C, S, d2, tau,
                                                    g.dev(si["rows"]), d["masks"], d["rlk"], wf, kf, wb, kb,
                                                    cache_ext=ext, sum_before_scaling=configs.C4_SUM_BEFORE_SCALING)
        scores, context, cache_h = g.host(scores), g.host(context), g.host(cache)
        idx = tau // B
        for c in range(2 * H):
            got[f"s{i}_cache{c}"] = digest(cache_h[c * S + idx])
        for h in range(H):
            for c in range(C):
                got[f"s{i}_score{h}_{c}"] = digest(scores[h, c])
            got[f"s{i}_context{h}"] = digest(context[h])
    compare(got, want, "C5H")


def test_c3_prompt_products_in_hoisted_forms_every_output():
    """The prompt configuration at full size through the hoisted calls: 12 x 128 diagonals of Q K^T
    (hoisted copies of K, folding sums in rounds) and 12 contexts A V (hoisted copies of V, the 128
    products of a head summed before one scaling)."""
    from oracle import attention
    say("C3 hoisted")
    st, want = configs.c3_inputs(), load("C3H")
    g = Gpu(st["prm"])
    H, m, d2, n = st["heads"], st["m"], st["d2"], st["prm"].n
    wf = configs.C4_ROUND_BITS[0]
    masks = g.ctx.plain_prepare(g.dev(st["masks"]))
    cache = g.ctx.empty_ct(2 * H)
    for tau in range(m):
        g.ctx.kv_append(cache, 1, 2 * H, tau, g.dev(st["rows"][tau]), masks, d2)
    copies = attention.copy_galois(n, d2)[1:]
    g_fold = g.ctx.round_galois(0, d2, wf)
    raw = configs.galois_keys("C3", sorted(set(copies) | set(g_fold)))
    keys = {gal: g.key(k) for gal, k in raw.items()}
    rlk = g.key(st["rlk"])
    out = g.ctx.prefill_qk_hoisted(g.dev(st["q"]), cache[:H], H, d2, rlk, [keys[x] for x in g_fold],
                                   [keys[x] for x in copies], fold_round_bits=wf)
    av = g.ctx.prefill_av_hoisted(g.dev(st["a"]), cache[H:], H, d2, rlk, [keys[x] for x in copies],
                                  sum_before_scaling=configs.C4_SUM_BEFORE_SCALING)
    out, av = g.host(out), g.host(av)
    got = {}
    for h in range(H):
        for i in range(m):
            got[f"qk{h}_{i}"] = digest(out[h, i])
        got[f"av{h}"] = digest(av[h])
    compare(got, want, "C3H")
