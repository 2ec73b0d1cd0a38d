"""Seeded input sets of the five benchmark configurations (draws only, no arithmetic).

Every array is a stand-in of the right shape: ciphertexts, switching keys and block masks are
uniformly random canonical residues / plaintexts (see synth.pseudo_ciphertexts).  The same
functions feed the oracle (digest generation, CPU baseline) and the HIP library (tests, bench).
"""
import numpy as np

from .params import PRESETS
from .synth import WORKLOADS, Stream, pseudo_ciphertexts, pseudo_switch_key


def fold_galois(n: int, d2: int):
    """Galois elements of the folding sum over one block: 3^1, 3^2, 3^4, ... 3^(d2/2) mod 2n."""
    gs, sh = [], 1
    while sh < d2:
        gs.append(pow(3, sh, 2 * n))
        sh *= 2
    return gs


def block_galois(n: int, d2: int):
    """Galois elements of the sum over blocks: 3^d2, 3^(2 d2), ... 3^(n/4), then the row swap."""
    gs, sh = [], d2
    while sh <= n // 4:
        gs.append(pow(3, sh, 2 * n))
        sh *= 2
    return gs + [2 * n - 1]


def _keys(prm, seed, label, gals):
    qp = list(prm.q) + list(prm.p)
    return {g: pseudo_switch_key(Stream(seed, label, i), qp, prm.n, prm.dnum) for i, g in enumerate(gals)}


def galois_keys(name: str, gals, label: int = 9):
    """Stand-in switching keys for arbitrary Galois elements of configuration `name`, one seeded draw
    per element (the stream is labelled by the element itself, so whoever asks for element g gets
    the same key whatever list it came in)."""
    w, prm = WORKLOADS[name], PRESETS[name]
    qp = list(prm.q) + list(prm.p)
    return {int(g): pseudo_switch_key(Stream(w.seed, label, int(g)), qp, prm.n, prm.dnum) for g in gals}


def _masks(prm, seed, count):
    rng = np.random.default_rng(seed)
    return rng.integers(0, prm.t, (count, prm.n), dtype=np.uint64)


def c1_inputs():
    """16 independent ciphertext pairs at N = 4096: tensor product + relinearisation of each."""
    w, prm = WORKLOADS["C1"], PRESETS["C1"]
    return {"prm": prm, "a": pseudo_ciphertexts(Stream(w.seed, 1), prm.q, prm.n, w.pairs),
            "b": pseudo_ciphertexts(Stream(w.seed, 2), prm.q, prm.n, w.pairs),
            "rlk": _keys(prm, w.seed, 5, ["rlk"])["rlk"]}


def decode_inputs(name: str, heads: int, context: int, d2: int = 64, spare_cts: int = 1):
    """Decode-step state: q, a, K/V caches ([K|V][head][stride] ciphertexts), new rows, masks, keys."""
    w, prm = WORKLOADS[name], PRESETS[name]
    B = prm.n // d2
    n_cts = context // B
    stride = n_cts + spare_cts
    s = w.seed
    fold, blk = fold_galois(prm.n, d2), block_galois(prm.n, d2)
    return {"prm": prm, "heads": heads, "d2": d2, "B": B, "n_cts": n_cts, "stride": stride, "tau": context,
            "q": pseudo_ciphertexts(Stream(s, 1), prm.q, prm.n, heads),
            "a": pseudo_ciphertexts(Stream(s, 2), prm.q, prm.n, heads * n_cts),
            "cache": pseudo_ciphertexts(Stream(s, 3), prm.q, prm.n, 2 * heads * stride),
            "rows": pseudo_ciphertexts(Stream(s, 4), prm.q, prm.n, 2 * heads),
            "masks": _masks(prm, s, B), "fold": fold, "block": blk,
            "rlk": _keys(prm, s, 5, ["rlk"])["rlk"], "gk": _keys(prm, s, 6, fold + blk)}


def c2_inputs():
    """One head, one K-cache ciphertext of 128 tokens at N = 8192: decode scores."""
    return decode_inputs("C2", heads=1, context=128)


def c4_inputs():
    """Full decode step at 512-token context, 12 heads, N = 8192."""
    return decode_inputs("C4", heads=12, context=512)


# bits per round of the scores' and the context's folding sums when the C4 step is run in its
# hoisted form (two rounds of 7 rotations for the scores; rounds of 7, 3 and 3 for the context)
C4_ROUND_BITS = (3, 3)
# ... and whether the context's products over the cache ciphertexts are summed before the one scaling
C4_SUM_BEFORE_SCALING = True


def c3_inputs(heads: int = 12, d2: int = 64):
    """Prefill: per head a row-packed Q ciphertext, and 128 K rows + 128 V rows (each tiled) that are
    appended into one K and one V cache ciphertext before Q K^T is formed."""
    w, prm = WORKLOADS["C3"], PRESETS["C3"]
    s, m = w.seed, prm.n // d2
    fold = fold_galois(prm.n, d2)
    g_blk, g_swap = pow(3, d2, 2 * prm.n), 2 * prm.n - 1
    right, sh = [], 1
    while sh < min(d2, m // 2):                      # right shifts by 1, 2, 4, ... slots
        right.append(pow(3, prm.n // 2 - sh, 2 * prm.n))
        sh *= 2
    return {"prm": prm, "heads": heads, "d2": d2, "m": m,
            "q": pseudo_ciphertexts(Stream(s, 1), prm.q, prm.n, heads),
            # rows[tau][cache]: caches = K of head 0..heads-1, then V of head 0..heads-1
            "rows": pseudo_ciphertexts(Stream(s, 4), prm.q, prm.n, m * 2 * heads).reshape(
                m, 2 * heads, 2, prm.k, prm.n),
            "masks": _masks(prm, s, m), "fold": fold, "g_blk": g_blk, "g_swap": g_swap,
            "rlk": _keys(prm, s, 5, ["rlk"])["rlk"], "gk": _keys(prm, s, 6, fold + [g_blk, g_swap]),
            # the rest of the prompt's attention: compaction of the scores, then A V with the weights
            # arriving as one ciphertext per (head, diagonal) (stand-ins for re-encrypted softmax output)
            "right": right, "gk_right": _keys(prm, s, 8, right),
            "mask0": np.random.default_rng(s + 1).integers(0, prm.t, prm.n, dtype=np.uint64),
            "a": pseudo_ciphertexts(Stream(s, 7), prm.q, prm.n, heads * m)}


def c5_inputs(heads: int = 16, d2: int = 64, steps: int = 64):
    """Scaled-up decode: N = 16384, 6+2 primes, 512-token cache growing by one token per step."""
    st = decode_inputs("C5", heads=heads, context=512, d2=d2, spare_cts=1)
    w, prm = WORKLOADS["C5"], st["prm"]
    st["steps"] = steps

    def step_inputs(i: int):
        n_cts = (512 + i) // st["B"] + 1
        return {"rows": pseudo_ciphertexts(Stream(w.seed, 10, i), prm.q, prm.n, 2 * heads),
                "q": pseudo_ciphertexts(Stream(w.seed, 11, i), prm.q, prm.n, heads),
                "a": pseudo_ciphertexts(Stream(w.seed, 12, i), prm.q, prm.n, heads * n_cts), "n_cts": n_cts}
    st["step_inputs"] = step_inputs
    return st
