"""The five benchmark configurations evaluated by the oracle (test infrastructure only).

Each function takes the seeded inputs of workloads.configs and returns {name: ciphertext array}
for every output unit, in the order and with the operation sequence the library documents."""
import numpy as np

from . import attention


def run_c1(orc, inp):
    return {f"pair{u}": orc.relin(orc.mul(inp["a"][u], inp["b"][u]), inp["rlk"]) for u in range(len(inp["a"]))}


def _decode_step(orc, st, q, a, cache, rows, tau, n_cts, out, tag="", rounds=None):
    """Append at token tau, then scores and context over n_cts cache ciphertexts per head.
    `cache` is modified in place (numpy array [2*heads*stride] of ciphertexts).
    rounds = (w_fold, w_block, keys by Galois element, sum_first): the hoisted forms of the products."""
    H, S, B, d2 = st["heads"], st["stride"], st["B"], st["d2"]
    idx, blk = divmod(tau, B)
    for c in range(2 * H):
        masked = orc.mul_plain(rows[c], st["masks"][blk])
        tgt = c * S + idx
        cache[tgt] = masked if blk == 0 else orc.add(cache[tgt], masked)
        out[f"{tag}cache{c}"] = cache[tgt].copy()
    fold = {g: st["gk"][g] for g in st["fold"]}
    block = {g: st["gk"][g] for g in st["block"]}
    for h in range(H):
        v0 = (H + h) * S
        a_h, v_h = list(a[h * n_cts:(h + 1) * n_cts]), list(cache[v0:v0 + n_cts])
        if rounds is None:
            for c in range(n_cts):
                out[f"{tag}score{h}_{c}"] = attention.decode_scores(orc, q[h], cache[h * S + c], st["rlk"], fold, d2)
            out[f"{tag}context{h}"] = attention.decode_context(orc, a_h, v_h, st["rlk"], block, d2)
        else:
            wf, wb, keys, sum_first = rounds
            for c in range(n_cts):
                out[f"{tag}score{h}_{c}"] = attention.decode_scores_hoisted(orc, q[h], cache[h * S + c], st["rlk"],
                                                                            keys, d2, wf)
            out[f"{tag}context{h}"] = attention.decode_context_hoisted(orc, a_h, v_h, st["rlk"], keys, d2, wb,
                                                                       sum_first=sum_first)


def run_c2(orc, st):
    """Decode scores of one head against its one cache ciphertext."""
    fold = {g: st["gk"][g] for g in st["fold"]}
    return {"score0_0": attention.decode_scores(orc, st["q"][0], st["cache"][0], st["rlk"], fold, st["d2"])}


def run_c4(orc, st):
    """Scores and context over the 512 cached tokens, then the append of token 512 (which opens the
    fifth ciphertext of every cache and therefore does not feed this step's products)."""
    out = {}
    cache = st["cache"].copy()
    H, S, C, d2 = st["heads"], st["stride"], st["n_cts"], st["d2"]
    fold = {g: st["gk"][g] for g in st["fold"]}
    block = {g: st["gk"][g] for g in st["block"]}
    for h in range(H):
        for c in range(C):
            out[f"score{h}_{c}"] = attention.decode_scores(orc, st["q"][h], cache[h * S + c], st["rlk"], fold, d2)
        v0 = (H + h) * S
        out[f"context{h}"] = attention.decode_context(orc, list(st["a"][h * C:(h + 1) * C]),
                                                      list(cache[v0:v0 + C]), st["rlk"], block, d2)
    idx, blk = divmod(st["tau"], st["B"])
    for c in range(2 * H):
        masked = orc.mul_plain(st["rows"][c], st["masks"][blk])
        out[f"cache{c}"] = masked if blk == 0 else orc.add(cache[c * S + idx], masked)
    return out


def run_c4_hoisted(orc, st, w_fold, w_block, gk_rounds, sum_first=False):
    """run_c4 with both folding sums taken in rounds of hoisted rotation sums (w_fold / w_block bits
    per round); gk_rounds: switching keys by Galois element for attention.hoisted_fold_galois.
    sum_first: the context's products over the cache ciphertexts summed before the one scaling."""
    out = {}
    cache = st["cache"].copy()
    H, S, C, d2 = st["heads"], st["stride"], st["n_cts"], st["d2"]
    for h in range(H):
        for c in range(C):
            out[f"score{h}_{c}"] = attention.decode_scores_hoisted(orc, st["q"][h], cache[h * S + c], st["rlk"],
                                                                   gk_rounds, d2, w_fold)
        v0 = (H + h) * S
        out[f"context{h}"] = attention.decode_context_hoisted(orc, list(st["a"][h * C:(h + 1) * C]),
                                                              list(cache[v0:v0 + C]), st["rlk"], gk_rounds, d2, w_block,
                                                              sum_first=sum_first)
    idx, blk = divmod(st["tau"], st["B"])
    for c in range(2 * H):
        masked = orc.mul_plain(st["rows"][c], st["masks"][blk])
        out[f"cache{c}"] = masked if blk == 0 else orc.add(cache[c * S + idx], masked)
    return out


def run_c3(orc, st, heads=None, progress=None):
    """Build every K and V cache ciphertext from its 128 row ciphertexts, then per head: Q K^T,
    the compaction of its score ciphertexts, and A V."""
    H, m, d2 = st["heads"], st["m"], st["d2"]
    heads = range(H) if heads is None else heads
    out = {}
    caches = {}
    for c in [h for h in heads] + [H + h for h in heads]:
        acc = None
        for tau in range(m):
            masked = orc.mul_plain(st["rows"][tau][c], st["masks"][tau])
            acc = masked if acc is None else orc.add(acc, masked)
        caches[c] = acc
        out[f"cache{c}"] = acc
    for h in heads:
        diag = attention.prefill_qk(orc, st["q"][h], caches[h], st["rlk"], st["gk"], d2)
        for i, x in enumerate(diag):
            out[f"qk{h}_{i}"] = x
        # the scores compacted for hand-over, and the context from the (stand-in) weights
        gkr = dict(st["gk_right"])
        for i, x in enumerate(attention.prefill_repack(orc, diag, st["mask0"], gkr, d2)):
            out[f"packed{h}_{i}"] = x
        out[f"av{h}"] = attention.prefill_av(orc, list(st["a"][h * m:(h + 1) * m]), caches[H + h], st["rlk"],
                                             st["gk"], d2)
        if progress:
            progress(f"C3 head {h} done")
    return out


def run_c3_hoisted(orc, st, heads, keys, w_fold, sum_first):
    """The prompt's Q K^T and A V of the given heads in their hoisted forms: the rotated copies of K
    and V as one series of hoisted rotations each, the folding sums in rounds of w_fold bits, the m
    products of A V summed before one scaling (sum_first).  keys: switching keys by Galois element
    for attention.copy_galois and the rounds' elements.  The caches are built as in run_c3."""
    H, m, d2 = st["heads"], st["m"], st["d2"]
    out = {}
    for h in heads:
        caches = {}
        for c in (h, H + h):
            acc = None
            for tau in range(m):
                masked = orc.mul_plain(st["rows"][tau][c], st["masks"][tau])
                acc = masked if acc is None else orc.add(acc, masked)
            caches[c] = acc
        for i, x in enumerate(attention.prefill_qk_hoisted(orc, st["q"][h], caches[h], st["rlk"], keys, d2, w=w_fold)):
            out[f"qk{h}_{i}"] = x
        out[f"av{h}"] = attention.prefill_av_hoisted(orc, list(st["a"][h * m:(h + 1) * m]), caches[H + h], st["rlk"],
                                                     keys, d2, sum_first=sum_first)
    return out


def run_c5(orc, st, steps, rounds=None):
    """`steps` successive decode steps with cache growth (append first, then attend over the cache
    including the new token's ciphertext); rounds as in _decode_step."""
    out = {}
    cache = st["cache"].copy()
    for i in range(steps):
        si = st["step_inputs"](i)
        _decode_step(orc, st, si["q"], si["a"], cache, si["rows"], 512 + i, si["n_cts"], out, tag=f"s{i}_",
                     rounds=rounds)
    return out
