"""Pins for the composite operations: decrypted results equal plaintext attention
arithmetic mod t, and the operation counts are the ones the paper states
(one slot-wise product per cache ciphertext and log2(d) rotations for the
decode scores, section 4.3 and its complexity table; B = N/d tokens per cache
ciphertext, Algorithm 1)."""
import numpy as np
import pytest

from oracle import Client, Oracle, attention
from oracle.client import galois_rot
from workloads import PRESETS, Stream, attention_activations

from .toy import toy_params


def _keys(cl, n, d):
    return {g: cl.galois_key(g) for g in attention.required_galois(n, d)}


def test_append_builds_the_packed_cache():
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 61, orc)
    n, d, t = prm.n, 64, prm.t
    B = n // d
    assert B == 128                                    # Algorithm 1: B = ceil(n / d2)
    rows = attention_activations(Stream(61, 1), 1, B + 2, d)[0]
    masks = {b: cl.codec.encode(attention.block_mask_values(n, d, b)) for b in (0, 1, 2, B - 1)}
    cache = []
    taus = [0, 1, 2, B - 1, B, B + 1]
    for tau in taus:
        row_ct = cl.encrypt_slots(np.tile(rows[tau], B))
        attention.append(orc, cache, tau, row_ct, masks, d)
    assert len(cache) == 2                             # token B opens a new ciphertext
    want0 = np.zeros(n, dtype=np.int64)
    for tau in (0, 1, 2, B - 1):
        want0[tau * d:(tau + 1) * d] = rows[tau]
    want1 = np.zeros(n, dtype=np.int64)
    for tau in (B, B + 1):
        want1[(tau - B) * d:(tau - B + 1) * d] = rows[tau]
    assert np.array_equal(cl.decrypt_slots(cache[0]), want0 % t)
    assert np.array_equal(cl.decrypt_slots(cache[1]), want1 % t)


def test_decode_scores_are_the_dot_products_with_log_d_rotations():
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 62, orc)
    n, d, t = prm.n, 64, prm.t
    B = n // d
    act = attention_activations(Stream(62, 1), 1, B + 1, d)[0]
    q, K = act[0], act[1:]
    rlk, gks = cl.relin_key(), _keys(cl, n, d)
    counts = {}
    out = attention.decode_scores(orc, cl.encrypt_slots(np.tile(q, B)),
                                  cl.encrypt_slots(K.reshape(-1)), rlk, gks, d, counts)
    assert counts == {"mul": 1, "relin": 1, "rotate": 6}       # log2(64) rotations
    dec = cl.decrypt_slots(out)
    assert np.array_equal(dec[::d], (K @ q) % t)
    assert cl.noise_budget_bits(out, cl.decrypt_poly(out)) > 20


def test_decode_context_is_the_weighted_sum_of_value_rows():
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 63, orc)
    n, d, t = prm.n, 64, prm.t
    B = n // d
    g = Stream(63, 1)
    V = attention_activations(g, 1, 2 * B, d)[0]
    a = attention_activations(g, 1, 2 * B, 1)[0, :, 0]
    rlk, gks = cl.relin_key(), _keys(cl, n, d)
    a_cts = [cl.encrypt_slots(np.repeat(a[c * B:(c + 1) * B], d)) for c in range(2)]
    v_cts = [cl.encrypt_slots(V[c * B:(c + 1) * B].reshape(-1)) for c in range(2)]
    counts = {}
    out = attention.decode_context(orc, a_cts, v_cts, rlk, gks, d, counts)
    assert counts == {"mul": 2, "relin": 1, "rotate": 7}
    dec = cl.decrypt_slots(out)
    want = (a @ V) % t
    assert np.array_equal(dec, np.tile(want, B))
    assert cl.noise_budget_bits(out, cl.decrypt_poly(out)) > 20


def test_round_chunks_and_round_elements_cover_every_subset_of_generators_once():
    assert attention.round_chunks(6, 2) == [2, 2, 2] and attention.round_chunks(7, 3) == [3, 2, 2]
    assert attention.round_chunks(7, 4) == [4, 3] and attention.round_chunks(6, 1) == [1] * 6
    assert attention.round_chunks(3, 8) == [3] and attention.round_chunks(0, 2) == []
    n, d = 1 << 12, 32
    for gens, w in ((attention.fold_generators(n, d), 2), (attention.block_generators(n, d), 3),
                    (attention.block_generators(n, d), 1)):
        rounds = attention.round_galois(n, gens, w)
        assert [len(r) for r in rounds] == [(1 << c) - 1 for c in attention.round_chunks(len(gens), w)]
        # composing the rounds reaches each of the 2^B subset products exactly once
        reached = [1]
        for elts in rounds:
            reached = [a * b % (2 * n) for a in reached for b in [1] + elts]
        want = [1]
        for g in gens:
            want = want + [a * g % (2 * n) for a in want]
        assert sorted(reached) == sorted(want) and len(set(reached)) == 1 << len(gens)
    # one bit per round: the rotate-and-add chain's own elements, in its order
    assert attention.round_galois(n, attention.fold_generators(n, d), 1) == [[g] for g in attention.fold_generators(n, d)]


@pytest.mark.parametrize("w", [1, 2, 3, 6])
def test_decode_scores_by_rounds_of_hoisted_rotations_are_the_same_dot_products(w):
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 62, orc)
    n, d, t = prm.n, 64, prm.t
    B = n // d
    act = attention_activations(Stream(62, 1), 1, B + 1, d)[0]
    q, K = act[0], act[1:]
    rlk = cl.relin_key()
    gks = {g: cl.galois_key(g) for g in attention.hoisted_fold_galois(n, d, w, 1)}
    counts = {}
    out = attention.decode_scores_hoisted(orc, cl.encrypt_slots(np.tile(q, B)), cl.encrypt_slots(K.reshape(-1)),
                                          rlk, gks, d, w, counts)
    assert counts == {1: {"rounds": 6, "rotate": 6}, 2: {"rounds": 3, "rotate": 9}, 3: {"rounds": 2, "rotate": 14},
                      6: {"rounds": 1, "rotate": 63}}[w]
    dec = cl.decrypt_slots(out)
    assert np.array_equal(dec[::d], (K @ q) % t)
    # every slot of a block holds the sum over the block's d slots rotated to it: the full fold
    prod = (np.tile(q, B) * K.reshape(-1)).reshape(2, n // 2)
    want = sum(np.roll(prod, -s, axis=1) for s in range(d)).reshape(-1)
    assert np.array_equal(dec, want % t)
    assert cl.noise_budget_bits(out, cl.decrypt_poly(out)) > 20


def test_rounds_of_hoisted_rotation_sums_leave_the_noise_budget_of_the_chain():
    """Same noise growth law either way (the sum of 64 rotated copies of the input's noise plus 63
    key switches' worth): the budgets of the chain form and of the rounds differ by about a bit."""
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 65, orc)
    n, d = prm.n, 64
    B = n // d
    act = attention_activations(Stream(65, 1), 1, B + 1, d)[0]
    q_ct, k_ct = cl.encrypt_slots(np.tile(act[0], B)), cl.encrypt_slots(act[1:].reshape(-1))
    rlk = cl.relin_key()
    gks = {g: cl.galois_key(g) for g in set(attention.required_galois(n, d)) | set(attention.hoisted_fold_galois(n, d, 3, 1))}
    chain = attention.decode_scores(orc, q_ct, k_ct, rlk, gks, d)
    rounds = attention.decode_scores_hoisted(orc, q_ct, k_ct, rlk, gks, d, 3)
    assert np.array_equal(cl.decrypt_slots(chain), cl.decrypt_slots(rounds))
    b_chain = cl.noise_budget_bits(chain, cl.decrypt_poly(chain))
    b_rounds = cl.noise_budget_bits(rounds, cl.decrypt_poly(rounds))
    assert abs(b_chain - b_rounds) <= 2 and min(b_chain, b_rounds) > 20


@pytest.mark.parametrize("w", [2, 3, 4, -3])
def test_decode_context_by_rounds_of_hoisted_rotations_is_the_same_weighted_sum(w):
    """w < 0: rounds of -w bits and the cache ciphertexts' products summed before the one scaling."""
    sum_first, w = w < 0, abs(w)
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 63, orc)
    n, d, t = prm.n, 64, prm.t
    B = n // d
    g = Stream(63, 1)
    V = attention_activations(g, 1, 2 * B, d)[0]
    a = attention_activations(g, 1, 2 * B, 1)[0, :, 0]
    rlk = cl.relin_key()
    gks = {e: cl.galois_key(e) for e in attention.hoisted_fold_galois(n, d, 1, w)}
    a_cts = [cl.encrypt_slots(np.repeat(a[c * B:(c + 1) * B], d)) for c in range(2)]
    v_cts = [cl.encrypt_slots(V[c * B:(c + 1) * B].reshape(-1)) for c in range(2)]
    counts = {}
    out = attention.decode_context_hoisted(orc, a_cts, v_cts, rlk, gks, d, w, counts, sum_first=sum_first)
    assert counts == {2: {"rounds": 4, "rotate": 3 + 3 + 3 + 1}, 3: {"rounds": 3, "rotate": 7 + 3 + 3},
                      4: {"rounds": 2, "rotate": 15 + 7}}[w]
    assert np.array_equal(cl.decrypt_slots(out), np.tile((a @ V) % t, B))
    assert cl.noise_budget_bits(out, cl.decrypt_poly(out)) > 20
    if sum_first:
        other = attention.decode_context_hoisted(orc, a_cts, v_cts, rlk, gks, d, w)
        assert not np.array_equal(out, other)
        # one rounding instead of two: never a smaller budget
        assert cl.noise_budget_bits(out, cl.decrypt_poly(out)) >= cl.noise_budget_bits(other, cl.decrypt_poly(other)) - 1


@pytest.mark.parametrize("hoisted", [False, True, 2])
def test_prefill_generalised_diagonals_on_a_small_ring(hoisted):
    """Also with the copies of K made by hoisted rotations of K itself, and (2) with the folding sum
    of every product in rounds of two bits on top: other ciphertexts, same slots."""
    prm = toy_params(8, 3, 1, 1)
    orc = Oracle(prm)
    cl = Client(prm, 64, orc)
    n, d, t = prm.n, 8, prm.t
    m = n // d
    H = m // 2
    g = Stream(64, 1)
    Qm = attention_activations(g, 1, m, d)[0]
    Km = attention_activations(g, 1, m, d)[0]
    rlk, gks = cl.relin_key(), _keys(cl, n, d)
    if hoisted:
        assert len(set(attention.copy_galois(n, d))) == m and attention.copy_galois(n, d)[0] == 1
        gks.update({g: cl.galois_key(g) for g in attention.copy_galois(n, d)[1:]})
    q_ct, k_ct = cl.encrypt_slots(Qm.reshape(-1)), cl.encrypt_slots(Km.reshape(-1))
    if hoisted == 2:
        gks.update({g: cl.galois_key(g) for g in attention.hoisted_fold_galois(n, d, 2, 1) if g not in gks})
        outs = attention.prefill_qk_hoisted(orc, q_ct, k_ct, rlk, gks, d, w=2)
        assert not np.array_equal(outs[1], attention.prefill_qk_hoisted(orc, q_ct, k_ct, rlk, gks, d)[1])
    else:
        outs = (attention.prefill_qk_hoisted if hoisted else attention.prefill_qk)(orc, q_ct, k_ct, rlk, gks, d)
    assert len(outs) == m
    S = (Qm @ Km.T) % t
    seen = np.zeros((m, m), dtype=bool)
    for idx, ct in enumerate(outs):
        sigma, r = divmod(idx, H)
        dec = cl.decrypt_slots(ct)
        for i in range(m):
            row, pos = divmod(i, H)
            j = (row ^ sigma) * H + (pos + r) % H
            assert dec[i * d] == S[i, j]
            seen[i, j] = True
    assert seen.all()


def test_galois_elements_needed_by_the_decode_step():
    n, d = 8192, 64
    gs = attention.required_galois(n, d)
    assert len(gs) == 13          # 6 fold shifts + 6 block shifts + row swap
    assert galois_rot(n, 1) == 3 and 2 * n - 1 in gs


def test_scores_against_an_outer_packed_segment_are_the_dot_products():
    """Inner-inner mode on a small ring: column ciphertexts, masked and broadcast query features."""
    prm = toy_params(8, 3, 1, 1)
    orc = Oracle(prm)
    cl = Client(prm, 65, orc)
    n, d, t = prm.n, 8, prm.t
    m = 40                                              # cached tokens (any number up to n)
    g = Stream(65, 1)
    K = attention_activations(g, 1, m, d)[0]
    q = attention_activations(g, 1, 1, d)[0, 0]
    rlk, gks = cl.relin_key(), _keys(cl, n, d)
    cols = []
    for j in range(d):
        v = np.zeros(n, dtype=np.int64)
        v[:m] = K[:, j]
        cols.append(cl.encrypt_slots(v))
    masks = [cl.codec.encode(attention.residue_mask_values(n, d, j)) for j in range(d)]
    counts = {}
    out = attention.decode_scores_outer(orc, cl.encrypt_slots(np.tile(q, n // d)), cols, masks, rlk, gks, d, counts)
    assert counts == {"mul": d, "rotate": d * 3}        # log2(8) rotations per feature
    dec = cl.decrypt_slots(out)
    assert np.array_equal(dec[:m], (K @ q) % t)
    assert not dec[m:].any()
    assert cl.noise_budget_bits(out, cl.decrypt_poly(out)) > 10


def test_context_against_an_outer_packed_segment_is_the_weighted_sum():
    prm = toy_params(8, 3, 1, 1)
    orc = Oracle(prm)
    cl = Client(prm, 66, orc)
    n, d, t = prm.n, 4, prm.t
    m = 50
    g = Stream(66, 1)
    V = attention_activations(g, 1, m, d)[0]
    a = attention_activations(g, 1, m, 1)[0, :, 0]
    rlk = cl.relin_key()
    gals = [galois_rot(n, sh) for sh in attention.all_slot_shifts(n)] + [2 * n - 1]
    gks = {g_: cl.galois_key(g_) for g_ in gals}
    cols = []
    for j in range(d):
        v = np.zeros(n, dtype=np.int64)
        v[:m] = V[:, j]
        cols.append(cl.encrypt_slots(v))
    av = np.zeros(n, dtype=np.int64)
    av[:m] = a
    outs = attention.decode_context_outer(orc, cl.encrypt_slots(av), cols, rlk, gks)
    want = (a @ V) % t
    for j in range(d):
        assert np.array_equal(cl.decrypt_slots(outs[j]), np.full(n, want[j]))


def _diag_col(i, sigma, r, H):
    row, pos = divmod(i, H)
    return (row ^ sigma) * H + (pos + r) % H


@pytest.mark.parametrize("hoisted", [False, True])
def test_prefill_context_is_the_matrix_product_on_a_small_ring(hoisted):
    """O = A V over the generalised diagonals: block i of the result is row i of A V mod t."""
    prm = toy_params(8, 3, 1, 1)
    orc = Oracle(prm)
    cl = Client(prm, 66, orc)
    n, d, t = prm.n, 8, prm.t
    m = n // d
    H = m // 2
    g = Stream(66, 1)
    Vm = attention_activations(g, 1, m, d)[0]
    Am = attention_activations(g, 1, m, m)[0]
    rlk, gks = cl.relin_key(), _keys(cl, n, d)
    a_cts = []
    for u in range(m):
        sigma, r = divmod(u, H)
        slots = np.zeros(n, dtype=np.int64)
        for i in range(m):
            slots[i * d:(i + 1) * d] = Am[i, _diag_col(i, sigma, r, H)]
        a_cts.append(cl.encrypt_slots(slots))
    if hoisted:
        gks.update({g: cl.galois_key(g) for g in attention.copy_galois(n, d)[1:]})
    fn = attention.prefill_av_hoisted if hoisted else attention.prefill_av
    v_ct = cl.encrypt_slots(Vm.reshape(-1))
    out = fn(orc, a_cts, v_ct, rlk, gks, d)
    dec = cl.decrypt_slots(out).reshape(m, d)
    assert np.array_equal(dec, (Am @ Vm) % t)
    if hoisted:     # and with the m products summed before their one scaling: other bits, same rows
        out2 = attention.prefill_av_hoisted(orc, a_cts, v_ct, rlk, gks, d, sum_first=True)
        assert not np.array_equal(out2, out)
        assert np.array_equal(cl.decrypt_slots(out2).reshape(m, d), (Am @ Vm) % t)


def _repack_case(log2n, d, seed):
    prm = toy_params(log2n, 3, 1, 1)
    orc = Oracle(prm)
    cl = Client(prm, seed, orc)
    n, t = prm.n, prm.t
    m = n // d
    H = m // 2
    w = min(d, H)
    g = Stream(seed, 1)
    Qm = attention_activations(g, 1, m, d)[0]
    Km = attention_activations(g, 1, m, d)[0]
    rlk, gks = cl.relin_key(), _keys(cl, n, d)
    for sh in attention.right_shifts(w):
        gr = galois_rot(n, n // 2 - sh)
        gks[gr] = cl.galois_key(gr)
    xs = attention.prefill_qk(orc, cl.encrypt_slots(Qm.reshape(-1)), cl.encrypt_slots(Km.reshape(-1)), rlk, gks, d)
    mask0 = cl.codec.encode(attention.slot0_mask_values(n, d))
    packed = attention.prefill_repack(orc, xs, mask0, gks, d)
    assert len(packed) == m // w
    S = (Qm @ Km.T) % t
    for gi, ct in enumerate(packed):
        dec = cl.decrypt_slots(ct)
        for i in range(m):
            for rp in range(d):
                if rp < w:
                    sigma, r = divmod(gi * w + rp, H)
                    assert dec[i * d + rp] == S[i, _diag_col(i, sigma, r, H)], (gi, i, rp)
                else:
                    assert dec[i * d + rp] == 0


def test_score_repacking_compacts_d_diagonals_per_ciphertext():
    _repack_case(8, 8, 67)      # H = 16 > d = 8: two groups per slot row


def test_score_repacking_when_a_slot_row_has_fewer_diagonals_than_slots_per_block():
    _repack_case(7, 16, 68)     # m = 8, H = 4 < d = 16: one group of 4 per slot row


def test_a_whole_decode_step_attends_over_the_cache_including_the_new_token():
    """The step as the configurations run it (append first, then scores and context over the cache):
    on a small ring with real encryptions the new token's key and value take part in both products."""
    from oracle import run_configs
    prm = toy_params(8, 3, 1, 1)
    orc = Oracle(prm)
    cl = Client(prm, 69, orc)
    n, d, t = prm.n, 8, prm.t
    B = n // d
    heads, stride, tau = 1, 2, 5                         # five tokens cached, token 5 arrives
    g = Stream(69, 1)
    K = attention_activations(g, 1, tau + 1, d)[0]
    V = attention_activations(g, 1, tau + 1, d)[0]
    q = attention_activations(g, 1, 1, d)[0, 0]
    a = attention_activations(g, 1, tau + 1, 1)[0, :, 0]
    packed = lambda M: np.concatenate([M[:tau].reshape(-1), np.zeros(n - tau * d, dtype=np.int64)])
    zero = np.zeros_like(cl.encrypt_slots(np.zeros(n, dtype=np.int64)))
    cache = np.stack([cl.encrypt_slots(packed(K)), zero, cl.encrypt_slots(packed(V)), zero])
    fold = [galois_rot(n, sh) for sh in attention.fold_shifts(d)]
    block = [galois_rot(n, sh) for sh in attention.block_shifts(n, d)] + [2 * n - 1]
    st = {"heads": heads, "stride": stride, "B": B, "d2": d, "fold": fold, "block": block,
          "masks": {b: cl.codec.encode(attention.block_mask_values(n, d, b)) for b in (tau,)},
          "rlk": cl.relin_key(), "gk": {x: cl.galois_key(x) for x in fold + block}}
    weights = np.zeros(n, dtype=np.int64)
    weights[:(tau + 1) * d] = np.repeat(a, d)
    out = {}
    run_configs._decode_step(orc, st, [cl.encrypt_slots(np.tile(q, B))], [cl.encrypt_slots(weights)], cache,
                             [cl.encrypt_slots(np.tile(K[tau], B)), cl.encrypt_slots(np.tile(V[tau], B))],
                             tau, 1, out)
    scores = cl.decrypt_slots(out["score0_0"])
    assert np.array_equal(scores[:(tau + 1) * d:d], (K @ q) % t)          # six dot products, the new token's last
    assert np.array_equal(cl.decrypt_slots(out["context0"])[:d], (a @ V) % t)
    grown = cl.decrypt_slots(out["cache0"])
    assert np.array_equal(grown[tau * d:(tau + 1) * d], K[tau] % t)


def test_lazy_noise_refresh_restores_the_budget_and_keeps_the_cache():
    """Algorithm 1 step 1 emulated end to end on the C2 parameters: a cache ciphertext that has taken
    many appends is masked by the server (ciphertext - r), refreshed by the client (decrypt, encrypt),
    unmasked (+ r): same contents, the noise budget of a fresh ciphertext.  The client never sees the
    cache (only cache - r), and a step after the refresh still attends correctly."""
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 70, orc)
    n, d, t = prm.n, 64, prm.t
    B = n // d
    g = Stream(70, 1)
    rows = attention_activations(g, 1, 6, d)[0]
    masks = {b: cl.codec.encode(attention.block_mask_values(n, d, b)) for b in range(6)}
    cache = []
    for tau in range(5):
        attention.append(orc, cache, tau, cl.encrypt_slots(np.tile(rows[tau], B)), masks, d)
    contents = cl.decrypt_poly(cache[0])
    worn = cl.noise_budget_bits(cache[0], contents)
    fresh = cl.noise_budget_bits(cl.encrypt_poly(contents), contents)
    assert worn < fresh - 20                            # each append costs a plaintext product

    r = np.random.default_rng(70).integers(0, t, n, dtype=np.uint64)       # the server's random mask
    share = orc.add_plain(cache[0], r, negative=True)
    seen_by_client = cl.decrypt_poly(share)
    assert np.array_equal(seen_by_client, (contents.astype(np.int64) - r.astype(np.int64)) % t)
    refreshed = orc.add_plain(cl.refresh(share), r)
    assert np.array_equal(cl.decrypt_poly(refreshed), contents)
    assert cl.noise_budget_bits(refreshed, contents) > fresh - 2

    cache[0] = refreshed
    attention.append(orc, cache, 5, cl.encrypt_slots(np.tile(rows[5], B)), masks, d)
    want = np.zeros(n, dtype=np.int64)
    want[:6 * d] = rows.reshape(-1)
    assert np.array_equal(cl.decrypt_slots(cache[0]), want % t)


def test_add_plain_is_addition_of_plaintexts_under_encryption():
    prm = toy_params(7, 2, 1, 1)
    orc = Oracle(prm)
    cl = Client(prm, 71, orc)
    rng = np.random.default_rng(71)
    a = rng.integers(0, prm.t, prm.n, dtype=np.uint64)
    b = rng.integers(0, prm.t, prm.n, dtype=np.uint64)
    ct = cl.encrypt_poly(a)
    assert np.array_equal(cl.decrypt_poly(orc.add_plain(ct, b)), (a + b) % prm.t)
    assert np.array_equal(cl.decrypt_poly(orc.add_plain(ct, b, negative=True)), (a + prm.t - b) % prm.t)
    # against the key-free encryption of b: ct + trivial(b) is the same ciphertext, bit for bit
    assert np.array_equal(orc.add_plain(ct, b), orc.add(ct, cl.trivial(b)))
    back = orc.add_plain(orc.add_plain(ct, b, negative=True), b)
    assert np.array_equal(back, ct)


def test_a_full_cache_ciphertext_stays_far_from_the_refresh_threshold():
    """Multi-step noise: 128 appends fill one cache ciphertext at the C2 parameters; its budget falls by
    a few bits only (the noise of the masked rows adds up like a random walk), and the scores computed
    against it still decrypt with tens of bits to spare -- the lazy refresh is rarely due, as the paper
    reports (its overhead stays below one per cent up to 512 tokens)."""
    prm = PRESETS["C2"]
    orc = Oracle(prm)
    cl = Client(prm, 72, orc)
    n, d, t = prm.n, 64, prm.t
    B = n // d
    g = Stream(72, 1)
    K = attention_activations(g, 1, B, d)[0]
    q = attention_activations(g, 1, 1, d)[0, 0]
    cache = []
    budgets = {}
    for tau in range(B):
        mask = cl.codec.encode(attention.block_mask_values(n, d, tau))
        attention.append(orc, cache, tau, cl.encrypt_slots(np.tile(K[tau], B)), {tau: mask}, d)
        if tau in (0, B - 1):
            budgets[tau] = cl.noise_budget_bits(cache[0], cl.decrypt_poly(cache[0]))
    assert len(cache) == 1
    assert np.array_equal(cl.decrypt_slots(cache[0]), K.reshape(-1) % t)
    assert budgets[0] - 6 < budgets[B - 1] < budgets[0]
    rlk, gks = cl.relin_key(), _keys(cl, n, d)
    out = attention.decode_scores(orc, cl.encrypt_slots(np.tile(q, B)), cache[0], rlk, gks, d)
    assert np.array_equal(cl.decrypt_slots(out)[::d], (K @ q) % t)
    assert cl.noise_budget_bits(out, cl.decrypt_poly(out)) > 20


def _cpvm_case(prm, d1, d2, seed, want_shape, hoisted=False, rounds=0):
    """Decrypts to x W mod t, tiled with period d2 (the layout the decode scores take a query in)."""
    orc = Oracle(prm)
    cl = Client(prm, seed, orc)
    n, t = prm.n, prm.t
    D1, T, C = attention.cpvm_shape(n, d1, d2)
    assert (D1, T, C) == want_shape
    g = Stream(seed, 1)
    x = attention_activations(g, 1, 1, d1)[0, 0]
    W = attention_activations(g, 1, d1, d2)[0]
    need = attention.cpvm_hoisted_galois(n, C, d2) if hoisted else attention.cpvm_galois(n, C, d2)
    if rounds:
        need = sorted(set(need) | set(attention.hoisted_fold_galois(n, d2, 1, rounds)))
    gks = {gal: cl.galois_key(gal) for gal in need}
    diags = [cl.codec.encode(attention.cpvm_weight_values(n, d1, d2, W, c)) for c in range(C)]
    x_ct = cl.encrypt_slots(attention.cpvm_token_values(n, d1, d2, x))
    counts = {}
    if rounds:
        y = attention.cpvm_hoisted(orc, x_ct, diags, gks, d2, counts, w=rounds)
    else:
        y = (attention.cpvm_hoisted if hoisted else attention.cpvm)(orc, x_ct, diags, gks, d2, counts)
    levels = (n // d2).bit_length() - 1
    assert counts == {"mul_plain": C, "rotate_shared": C - 1, "rotate": levels}
    want = (x.astype(object) @ W.astype(object)) % t
    assert np.array_equal(cl.decrypt_slots(y), np.tile(np.array(want, dtype=np.int64), n // d2))
    assert cl.noise_budget_bits(y, cl.decrypt_poly(y)) > 20
    return counts


def test_cpvm_layout_shows_every_feature_output_pair_once_per_residue_class():
    """The counting argument behind the procedure, checked on the slot values alone: summing
    token * diagonal_c over the diagonals and over the slots of one residue class modulo d2
    gives x W exactly (integers, no encryption)."""
    for n, d1, d2 in ((128, 20, 8), (256, 100, 16), (4096, 200, 64), (8192, 768, 64), (4096, 1000, 64), (256, 5, 64)):
        D1, T, C = attention.cpvm_shape(n, d1, d2)
        assert T * C == d2 and D1 * T == n
        g = Stream(70, n, d1)
        x = g.integers(-128, 128, d1)
        W = g.integers(-128, 128, (d1, d2))
        tok = attention.cpvm_token_values(n, d1, d2, x)
        half = n // 2
        acc = np.zeros(n, dtype=np.int64)
        for c in range(C):
            rot = np.concatenate([np.roll(tok[:half], -c), np.roll(tok[half:], -c)])   # rows rotate left by c
            acc += rot * attention.cpvm_weight_values(n, d1, d2, W, c)
        assert np.array_equal(acc.reshape(-1, d2).sum(axis=0), x @ W), (n, d1, d2)


def test_cpvm_on_small_rings():
    _cpvm_case(toy_params(7, 3, 1, 1), 20, 8, 71, (32, 4, 2))
    _cpvm_case(toy_params(8, 3, 1, 1), 100, 16, 72, (128, 2, 8))
    _cpvm_case(toy_params(8, 2, 1, 1), 5, 64, 73, (64, 4, 16))     # a token much shorter than a tile


def test_cpvm_with_hoisted_token_copies_on_small_rings():
    """The token's copies as one series of hoisted rotations of the token: same plaintext result."""
    _cpvm_case(toy_params(7, 3, 1, 1), 20, 8, 76, (32, 4, 2), hoisted=True)
    _cpvm_case(toy_params(8, 3, 1, 1), 100, 16, 77, (128, 2, 8), hoisted=True)
    # and the sum over residue classes in rounds of 2 and 3 bits
    _cpvm_case(toy_params(7, 3, 1, 1), 20, 8, 76, (32, 4, 2), hoisted=True, rounds=2)
    _cpvm_case(toy_params(8, 3, 1, 1), 100, 16, 77, (128, 2, 8), hoisted=True, rounds=3)


def test_cpvm_at_the_paper_sizes_takes_eight_products_and_seven_rotations_per_matrix():
    """d1 = 768, d2 = 64, N = 8192 (the sizes of the paper's CT x PT complexity table): one
    ciphertext per token, 8 plaintext products (768 padded to 1024: 1024 * 64 / 8192) and
    log2(N / d2) = 7 rotations per matrix, plus 7 rotations of the token shared by all matrices."""
    counts = _cpvm_case(PRESETS["C2"], 768, 64, 74, (1024, 8, 8))
    assert counts == {"mul_plain": 8, "rotate_shared": 7, "rotate": 7}


def test_cpvm_output_is_the_layout_the_attention_products_and_the_append_take():
    """Section 4.2's claim that the projection's result feeds the CT x CT kernels without
    re-encoding, on a small ring: q = x Wq goes straight into decode_scores as the tiled query,
    k = x Wk straight into append as the tiled new row."""
    prm = toy_params(8, 3, 1, 1)
    orc = Oracle(prm)
    cl = Client(prm, 75, orc)
    n, t, d1, d2 = prm.n, prm.t, 40, 8
    B = n // d2
    D1, T, C = attention.cpvm_shape(n, d1, d2)
    g = Stream(75, 1)
    x = g.integers(-8, 8, d1)
    Wq, Wk = g.integers(-8, 8, (d1, d2)), g.integers(-8, 8, (d1, d2))
    K = g.integers(-8, 8, (B, d2))
    gals = set(attention.cpvm_galois(n, C, d2)) | set(attention.required_galois(n, d2))
    gks = {gal: cl.galois_key(gal) for gal in gals}
    rlk = cl.relin_key()
    x_ct = cl.encrypt_slots(attention.cpvm_token_values(n, d1, d2, x))
    enc = lambda W: [cl.codec.encode(attention.cpvm_weight_values(n, d1, d2, W, c)) for c in range(C)]
    q_ct = attention.cpvm(orc, x_ct, enc(Wq), gks, d2)
    k_ct = attention.cpvm(orc, x_ct, enc(Wk), gks, d2)
    # scores of the projected query against a cache of B tokens
    scores = attention.decode_scores(orc, q_ct, cl.encrypt_slots(K.reshape(-1)), rlk, gks, d2)
    assert np.array_equal(cl.decrypt_slots(scores)[::d2], (K @ (x @ Wq)) % t)
    # the projected key appended as token 3 of an empty cache
    masks = {3: cl.codec.encode(attention.block_mask_values(n, d2, 3))}
    cache = attention.append(orc, [], 3, k_ct, masks, d2)
    want = np.zeros(n, dtype=np.int64)
    want[3 * d2:4 * d2] = (x @ Wk) % t
    assert np.array_equal(cl.decrypt_slots(cache[0]), want)
