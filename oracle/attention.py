"""Cache append and attention products as plain sequences of evaluator calls.

Test infrastructure only.  Token rows are "inner-packed" (the paper's section
2.4): with head dimension d and B = N/d blocks per ciphertext, block b (flat
slots [b d, (b+1) d)) of a cache ciphertext holds one token's d-vector.

  append          Algorithm 1, steps 2-3 (slot-aware concatenation): the new
                  row arrives tiled into every block, is masked to block
                  tau mod B by a plaintext multiplication and added into cache
                  ciphertext floor(tau / B); tokens are numbered from 0.
  decode_scores   section 4.3, inner-outer mode: one slot-wise product of the
                  tiled query with a cache ciphertext, relinearise, then the
                  folding sum (rotate by 1, 2, 4, ... d/2 and add).  Slot b d
                  then holds <q, K_b> mod t.
  decode_context  section 4.3, inner-inner mode with the attention weight of
                  token b already broadcast over block b by the encryptor:
                  sum of slot-wise products over the cache ciphertexts (three
                  components), one relinearisation, then a sum over blocks
                  (rotate by d, 2d, ... N/4, then swap the two slot rows).
  decode_scores_hoisted, decode_context_hoisted  the same two products with their folding
                  sums regrouped into rounds of several rotations of one ciphertext each
                  (hoisted, one division by P per round); defined above round_chunks.
  decode_scores_outer  section 4.3, inner-inner mode: scores against an outer-packed
                  (column-per-ciphertext) cache segment; each query feature is masked,
                  broadcast by rotations and multiplied with its column ciphertext.
  prefill_qk      the prompt's Q K^T as m "generalised diagonals" (the paper
                  names an outer-outer product and gives no procedure; the one
                  used is stated at the function: K rotated by whole blocks and
                  optionally row-swapped, slot-wise product, folding sum).
  prefill_av      the prompt's A V over the same diagonals: the weights arrive
                  one ciphertext per diagonal, broadcast over each token's block.
  prefill_repack  compaction of the score ciphertexts (useful values in slot 0 of
                  each block) into ciphertexts with d useful values per block.
  cpvm            section 4.2, the decode step's ciphertext-plaintext vector-matrix
                  product ("inner-diagonal"): one token of d1 features in one
                  ciphertext times a plaintext d1 x d2 matrix, the result tiled with
                  period d2 over all slots, which is the layout decode_scores takes
                  its query in and append takes its new row in.  The paper gives the
                  operation, its operand counts (one ciphertext per token, about
                  d1 d2 / N plaintext products, O(log) rotations) and no procedure;
                  the one used is laid out in the comment above cpvm_shape.
"""
import numpy as np

from .client import galois_rot, galois_swap


def block_mask_values(n: int, d: int, b: int) -> np.ndarray:
    v = np.zeros(n, dtype=np.int64)
    v[b * d:(b + 1) * d] = 1
    return v


def append(orc, cache, tau: int, row_ct, mask_polys, d: int):
    """cache: list of ciphertexts (grown in place); mask_polys[b] = encode(block mask b)."""
    B = orc.n // d
    idx, b = divmod(tau, B)
    masked = orc.mul_plain(row_ct, mask_polys[b])
    if idx == len(cache):
        cache.append(np.zeros_like(masked))
    cache[idx] = orc.add(cache[idx], masked)
    return cache


def fold_shifts(d: int):
    sh = 1
    while sh < d:
        yield sh
        sh *= 2


def block_shifts(n: int, d: int):
    sh = d
    while sh <= n // 4:
        yield sh
        sh *= 2


def decode_scores(orc, q_ct, k_ct, rlk, gks, d: int, counts=None):
    x = orc.relin(orc.mul(q_ct, k_ct), rlk)
    if counts is not None:
        counts["mul"] = counts.get("mul", 0) + 1
        counts["relin"] = counts.get("relin", 0) + 1
    for sh in fold_shifts(d):
        g = galois_rot(orc.n, sh)
        x = orc.add(x, orc.rotate(x, g, gks[g]))
        if counts is not None:
            counts["rotate"] = counts.get("rotate", 0) + 1
    return x


def decode_context(orc, a_cts, v_cts, rlk, gks, d: int, counts=None):
    y = None
    for a_ct, v_ct in zip(a_cts, v_cts):
        prod3 = orc.mul(a_ct, v_ct)
        y = prod3 if y is None else orc.add(y, prod3)
        if counts is not None:
            counts["mul"] = counts.get("mul", 0) + 1
    x = orc.relin(y, rlk)
    if counts is not None:
        counts["relin"] = counts.get("relin", 0) + 1
    gs = [galois_rot(orc.n, sh) for sh in block_shifts(orc.n, d)] + [galois_swap(orc.n)]
    for g in gs:
        x = orc.add(x, orc.rotate(x, g, gks[g]))
        if counts is not None:
            counts["rotate"] = counts.get("rotate", 0) + 1
    return x


# ---------------------------------------------------------------------------
# folding sums by rounds of hoisted rotations
#
# A folding sum x -> sum over all products of a subset of the generators g_0 .. g_{B-1}
# (sigma applied to x) is what "rotate by g_b and add" for b = 0 .. B-1 computes in B dependent
# steps.  The Galois maps commute, so the bits can be taken in chunks instead: a round over bits
# [b0, b0 + c) maps x to the sum of sigma_e(x) over the 2^c products e of subsets of g_b0 ..
# g_{b0+c-1}, and the rounds over consecutive chunks compose to the same sum.  Within a round all
# 2^c - 1 rotations act on the same ciphertext, so they are hoisted and their key-switch
# accumulators summed before one division by P (rotate_sum_hoisted): ceil(B / w) dependent steps
# instead of B, for 2^c - 1 keys per round instead of c.  Same slots, other ciphertext bits.
# ---------------------------------------------------------------------------
def round_chunks(n_bits: int, w: int):
    """Chunk lengths: ceil(n_bits / w) rounds, as even as possible, the longer ones first."""
    assert n_bits >= 0 and w >= 1
    if n_bits == 0:
        return []
    rounds = -(-n_bits // w)
    lo, extra = divmod(n_bits, rounds)
    return [lo + 1] * extra + [lo] * (rounds - extra)


def round_galois(n: int, gens, w: int):
    """[[Galois elements of round 0], [of round 1], ...] for the generators gens (bit b -> gens[b]);
    within a round, entry m - 1 is the product of the generators whose bit is set in m = 1 .. 2^c - 1."""
    out, b0 = [], 0
    for c in round_chunks(len(gens), w):
        elts = []
        for m in range(1, 1 << c):
            e = 1
            for i in range(c):
                if (m >> i) & 1:
                    e = e * gens[b0 + i] % (2 * n)
            elts.append(e)
        out.append(elts)
        b0 += c
    return out


def fold_generators(n: int, d: int):
    return [galois_rot(n, sh) for sh in fold_shifts(d)]


def block_generators(n: int, d: int):
    return [galois_rot(n, sh) for sh in block_shifts(n, d)] + [galois_swap(n)]


def fold_by_rounds(orc, x, gens, gks, w: int, counts=None):
    for elts in round_galois(orc.n, gens, w):
        x = orc.rotate_sum_hoisted(x, elts, gks)
        if counts is not None:
            counts["rounds"] = counts.get("rounds", 0) + 1
            counts["rotate"] = counts.get("rotate", 0) + len(elts)
    return x


def decode_scores_hoisted(orc, q_ct, k_ct, rlk, gks, d: int, w: int, counts=None):
    """decode_scores with the folding sum taken in rounds of w bits (hoisted rotation sums)."""
    x = orc.relin(orc.mul(q_ct, k_ct), rlk)
    return fold_by_rounds(orc, x, fold_generators(orc.n, d), gks, w, counts)


def decode_context_hoisted(orc, a_cts, v_cts, rlk, gks, d: int, w: int, counts=None, sum_first: bool = False):
    """decode_context with the sum over blocks (and the two slot rows) taken in rounds of w bits.
    sum_first: the products over the cache ciphertexts are summed as tensor products over the
    integers and scaled by t/Q once (Oracle.mul_sum) instead of scaled one by one and added."""
    if sum_first:
        y = orc.mul_sum(list(a_cts), list(v_cts))
    else:
        y = None
        for a_ct, v_ct in zip(a_cts, v_cts):
            prod3 = orc.mul(a_ct, v_ct)
            y = prod3 if y is None else orc.add(y, prod3)
    x = orc.relin(y, rlk)
    return fold_by_rounds(orc, x, block_generators(orc.n, d), gks, w, counts)


def hoisted_fold_galois(n: int, d: int, w_fold: int, w_block: int):
    """Galois elements the two hoisted decode products need keys for."""
    gs = [e for r in round_galois(n, fold_generators(n, d), w_fold) for e in r]
    gs += [e for r in round_galois(n, block_generators(n, d), w_block) for e in r]
    return sorted(set(gs))


def residue_mask_values(n: int, d: int, j: int) -> np.ndarray:
    """1 on the flat slots congruent to j modulo d, else 0."""
    v = np.zeros(n, dtype=np.int64)
    v[j::d] = 1
    return v


def decode_scores_outer(orc, q_ct, k_cols, mask_polys, rlk, gks, d: int, counts=None):
    """Section 4.3, inner-inner mode against an outer-packed cache segment.

    k_cols[j] holds feature j of every cached token (token tau in flat slot tau); q_ct holds the
    query tiled with period d.  Each feature of the query is isolated by a plaintext mask,
    broadcast to every slot by the folding rotations, multiplied with its column ciphertext,
    and the three-component products are summed before one relinearisation."""
    y = None
    for j in range(d):
        x = orc.mul_plain(q_ct, mask_polys[j])
        for sh in fold_shifts(d):
            g = galois_rot(orc.n, sh)
            x = orc.add(x, orc.rotate(x, g, gks[g]))
            if counts is not None:
                counts["rotate"] = counts.get("rotate", 0) + 1
        prod3 = orc.mul(x, k_cols[j])
        y = prod3 if y is None else orc.add(y, prod3)
        if counts is not None:
            counts["mul"] = counts.get("mul", 0) + 1
    return orc.relin(y, rlk)


def all_slot_shifts(n: int):
    sh = 1
    while sh <= n // 4:
        yield sh
        sh *= 2


def decode_context_outer(orc, a_ct, v_cols, rlk, gks):
    """Section 4.3, inner-outer mode on an outer-packed value segment: one slot-wise product of
    the weight ciphertext (a_tau in flat slot tau) with each column ciphertext, relinearise,
    then a folding sum over all slots (rotate by 1, 2, ..., N/4, then swap the rows)."""
    n = orc.n
    gs = [galois_rot(n, sh) for sh in all_slot_shifts(n)] + [galois_swap(n)]
    outs = []
    for v_ct in v_cols:
        x = orc.relin(orc.mul(a_ct, v_ct), rlk)
        for g in gs:
            x = orc.add(x, orc.rotate(x, g, gks[g]))
        outs.append(x)
    return outs


def prefill_qk(orc, q_ct, k_ct, rlk, gks, d: int):
    """All m = N/d generalised diagonals of S = Q K^T for one head.

    Q and K are token-major row-packed (token i in block i).  With H = m/2
    tokens per slot row, output (sigma, r) holds at slot i*d the entry
    S[i][j], j = (row_i xor sigma) * H + ((pos_i + r) mod H), i = row_i*H + pos_i.
    Order of the returned list: sigma-major, r ascending.
    """
    n = orc.n
    m = n // d
    H = m // 2
    g_blk, g_swap = galois_rot(n, d), galois_swap(n)
    rot = [k_ct]
    for _ in range(1, H):
        rot.append(orc.rotate(rot[-1], g_blk, gks[g_blk]))
    out = []
    for sigma in (0, 1):
        for r in range(H):
            kk = rot[r] if sigma == 0 else orc.rotate(rot[r], g_swap, gks[g_swap])
            x = orc.relin(orc.mul(q_ct, kk), rlk)
            for sh in fold_shifts(d):
                g = galois_rot(n, sh)
                x = orc.add(x, orc.rotate(x, g, gks[g]))
            out.append(x)
    return out


def rotated_copies(orc, ct, gks, d: int):
    """[sigma*H + r] -> ct rotated left by r blocks (sequentially, one key), row-swapped for sigma = 1."""
    n = orc.n
    H = n // d // 2
    g_blk, g_swap = galois_rot(n, d), galois_swap(n)
    rot = [ct]
    for _ in range(1, H):
        rot.append(orc.rotate(rot[-1], g_blk, gks[g_blk]))
    return rot + [orc.rotate(x, g_swap, gks[g_swap]) for x in rot]


def prefill_av(orc, a_cts, v_ct, rlk, gks, d: int):
    """O = A V for one head.  a_cts[sigma*H + r] holds A[i][j(i, sigma, r)] in every slot of block i
    (j as in prefill_qk); v_ct is token-major.  Sum of the m slot-wise products (three components,
    unit order ascending), one relinearisation: block i of the result holds sum_j A[i][j] V[j][:]."""
    vs = rotated_copies(orc, v_ct, gks, d)
    y = orc.mul(a_cts[0], vs[0])
    for u in range(1, len(vs)):
        y = orc.add(y, orc.mul(a_cts[u], vs[u]))
    return orc.relin(y, rlk)


def copy_galois(n: int, d: int):
    """Galois elements that take a token-major ciphertext straight to its m = N/d rotated copies:
    unit sigma*H + r -> 3^(d r), times 2N - 1 for the row-swapped half (unit 0: the identity)."""
    H = n // d // 2
    g_swap = galois_swap(n)
    return [galois_rot(n, d * r) * (g_swap if sigma else 1) % (2 * n) for sigma in (0, 1) for r in range(H)]


def rotated_copies_hoisted(orc, ct, gks, d: int):
    """The same m copies as rotated_copies, every one of them rotated out of the source ciphertext
    itself as a series of hoisted rotations (one decomposition of its c1, one key per copy)."""
    gs = copy_galois(orc.n, d)
    return [ct] + orc.rotate_many(ct, gs[1:], gks)


def prefill_qk_hoisted(orc, q_ct, k_ct, rlk, gks, d: int, w: int = 0):
    """prefill_qk with the rotated copies of K made by hoisted rotations (same slots, other bits);
    w >= 1: the folding sum of every product in rounds of w bits (fold_by_rounds)."""
    n = orc.n
    out = []
    for kk in rotated_copies_hoisted(orc, k_ct, gks, d):
        x = orc.relin(orc.mul(q_ct, kk), rlk)
        if w:
            x = fold_by_rounds(orc, x, fold_generators(n, d), gks, w)
        else:
            for sh in fold_shifts(d):
                g = galois_rot(n, sh)
                x = orc.add(x, orc.rotate(x, g, gks[g]))
        out.append(x)
    return out


def prefill_av_hoisted(orc, a_cts, v_ct, rlk, gks, d: int, sum_first: bool = False):
    """prefill_av with the rotated copies of V made by hoisted rotations; sum_first: the m products
    summed as tensor products and scaled once (Oracle.mul_sum)."""
    vs = rotated_copies_hoisted(orc, v_ct, gks, d)
    if sum_first:
        return orc.relin(orc.mul_sum(list(a_cts), vs), rlk)
    y = orc.mul(a_cts[0], vs[0])
    for u in range(1, len(vs)):
        y = orc.add(y, orc.mul(a_cts[u], vs[u]))
    return orc.relin(y, rlk)


def slot0_mask_values(n: int, d: int) -> np.ndarray:
    v = np.zeros(n, dtype=np.int64)
    v[::d] = 1
    return v


def right_shifts(w: int):
    sh = 1
    while sh < w:
        yield sh
        sh *= 2


def prefill_repack(orc, x_cts, mask0_poly, gks, d: int):
    """x_cts: the m score ciphertexts of one head (unit order of prefill_qk).  Groups of
    w = min(d, H) consecutive units; each unit is masked to slot 0 of every block, then a pairwise
    tree adds unit r' of the group shifted right by r' slots: at level l,
    y[j 2^(l+1)] += rotate_right(y[j 2^(l+1) + 2^l], 2^l).  Returns the m / w group sums."""
    n = orc.n
    H = n // d // 2
    w = min(d, H)
    y = [orc.mul_plain(x, mask0_poly) for x in x_cts]
    for sh in right_shifts(w):
        g = galois_rot(n, n // 2 - sh)
        for j in range(0, len(y), 2 * sh):
            y[j] = orc.add(y[j], orc.rotate(y[j + sh], g, gks[g]))
    return [y[j] for j in range(0, len(y), w)]


def required_galois(n: int, d: int):
    """Galois elements the decode and prefill products use."""
    gs = [galois_rot(n, sh) for sh in fold_shifts(d)]
    gs += [galois_rot(n, sh) for sh in block_shifts(n, d)]
    gs.append(galois_swap(n))
    return sorted(set(gs))


# ---------------------------------------------------------------------------
# ciphertext-plaintext vector-matrix product of the decode step (section 4.2)
#
# Layout.  D1 = the tile length: a power of two, at least d1, d2 and N/d2 and at most N/2; the N
# slots are T = N/D1 tiles (T/2 per slot row).  C = d2 / T "diagonals".  The token x (zero-padded
# to D1) sits in tile r shifted by C r features: flat slot r D1 + i holds x[(i + C r) mod D1].
# Diagonal c of the weights holds, at flat slot s, W[f][s mod d2] with f the feature that the
# token's ciphertext shows at s once it has been rotated left by c (zero for f >= d1).
# Then y = sum_c rotate(x, c) * P_c has, at slot s, C terms of output s mod d2, every pair
# (feature, output) exactly once over the slots of one residue class modulo d2; the sum over those
# classes (rotate by d2, 2 d2, ... N/4 and add, then the row swap) leaves output j in every slot
# congruent to j.
# ---------------------------------------------------------------------------
def cpvm_shape(n: int, d1: int, d2: int):
    """-> (D1, T, C)."""
    D1 = 1
    while D1 < max(d1, d2, n // d2):
        D1 *= 2
    assert D1 <= n // 2 and d2 >= 2 and d2 & (d2 - 1) == 0, "token longer than a slot row, or d2 not a power of two"
    T = n // D1
    return D1, T, d2 // T


def cpvm_feature_of_slot(n: int, d1: int, d2: int) -> np.ndarray:
    """Feature index shown by every flat slot of the token's ciphertext (>= d1: padding)."""
    D1, T, C = cpvm_shape(n, d1, d2)
    s = np.arange(n)
    return (s % D1 + C * (s // D1)) % D1


def cpvm_token_values(n: int, d1: int, d2: int, x) -> np.ndarray:
    f = cpvm_feature_of_slot(n, d1, d2)
    xp = np.zeros(cpvm_shape(n, d1, d2)[0], dtype=np.int64)
    xp[:d1] = x
    return xp[f]


def cpvm_weight_values(n: int, d1: int, d2: int, W, c: int) -> np.ndarray:
    """Slot values of diagonal c of the d1 x d2 matrix W."""
    f = cpvm_feature_of_slot(n, d1, d2)
    half = n // 2
    s = np.arange(n)
    shown = f[(s // half) * half + (s % half + c) % half]     # feature at s after a left rotation by c
    Wp = np.zeros((cpvm_shape(n, d1, d2)[0], d2), dtype=np.int64)
    Wp[:d1] = W
    return Wp[shown, s % d2]


def cpvm_shifts(c_count: int):
    sh = 1
    while sh < c_count:
        yield sh
        sh *= 2


def cpvm(orc, x_ct, diag_polys, gks, d2: int, counts=None):
    """y = x W for one token and one weight matrix given as its C diagonal plaintexts.

    The C rotated copies of the token come from a doubling tree (copy 2^l + i = copy i rotated by
    2^l: log2 C levels, C - 1 rotations, shared by every matrix applied to this token), then C
    plaintext products are summed and the residue classes modulo d2 folded together."""
    n = orc.n
    copies = [x_ct]
    for sh in cpvm_shifts(len(diag_polys)):
        g = galois_rot(n, sh)
        copies += [orc.rotate(copies[i], g, gks[g]) for i in range(sh)]
    y = orc.mul_plain(copies[0], diag_polys[0])
    for c in range(1, len(diag_polys)):
        y = orc.add(y, orc.mul_plain(copies[c], diag_polys[c]))
    gs = [galois_rot(n, sh) for sh in block_shifts(n, d2)] + [galois_swap(n)]
    for g in gs:
        y = orc.add(y, orc.rotate(y, g, gks[g]))
    if counts is not None:
        counts.update(mul_plain=len(diag_polys), rotate_shared=len(diag_polys) - 1, rotate=len(gs))
    return y


def cpvm_hoisted(orc, x_ct, diag_polys, gks, d2: int, counts=None, w: int = 0):
    """cpvm with the C - 1 rotated copies of the token made as one series of hoisted rotations of the
    token itself (copy c = token rotated by c, key for 3^c) instead of a doubling tree; w >= 1: the
    sum over residue classes in rounds of w bits (fold_by_rounds)."""
    n = orc.n
    C = len(diag_polys)
    copies = [x_ct] + orc.rotate_many(x_ct, [galois_rot(n, c) for c in range(1, C)], gks)
    y = orc.mul_plain(copies[0], diag_polys[0])
    for c in range(1, C):
        y = orc.add(y, orc.mul_plain(copies[c], diag_polys[c]))
    gs = block_generators(n, d2)
    if w:
        y = fold_by_rounds(orc, y, gs, gks, w)
    else:
        for g in gs:
            y = orc.add(y, orc.rotate(y, g, gks[g]))
    if counts is not None:
        counts.update(mul_plain=C, rotate_shared=C - 1, rotate=len(gs))
    return y


def cpvm_hoisted_galois(n: int, c_count: int, d2: int):
    """Galois elements cpvm_hoisted needs keys for."""
    return sorted(set([galois_rot(n, c) for c in range(1, c_count)] +
                      [galois_rot(n, sh) for sh in block_shifts(n, d2)] + [galois_swap(n)]))


def cpvm_galois(n: int, c_count: int, d2: int):
    gs = [galois_rot(n, sh) for sh in cpvm_shifts(c_count)]
    gs += [galois_rot(n, sh) for sh in block_shifts(n, d2)] + [galois_swap(n)]
    return sorted(set(gs))
