"""The one-call decode step under HIP graph capture: the side streams join the capture through the
fork and join events.  Every replay (with eager work of the same library in between) must give the
eager result bit for bit."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from workloads import PRESETS, Stream, pseudo_ciphertexts, pseudo_switch_key


def say(msg):
    print(f"[gpu-graph] {msg}", flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("hoisted", [False, True], ids=["chains", "rounds"])
def test_captured_decode_step_replays_to_the_eager_result(hoisted):
    import torch
    import paper_2602_08798_amd as P
    prm = PRESETS["C1"]
    n, d2 = prm.n, 64
    B = n // d2
    heads, n_cts, stride = 2, 1, 2
    ctx = P.Context(prm)
    qp = list(prm.q) + list(prm.p)
    ct = lambda seed, cnt: P.to_device(pseudo_ciphertexts(Stream(seed, 1), prm.q, n, cnt))
    key = lambda seed: ctx.ksk_prepare(P.to_device(pseudo_switch_key(Stream(seed, 2), qp, n, prm.dnum)))
    q, a, rows = ct(1, heads), ct(2, heads * n_cts), ct(3, 2 * heads)
    cache0 = ct(4, 2 * heads * stride)
    cache = cache0.clone()
    rng = np.random.default_rng(5)
    masks = ctx.plain_prepare(P.to_device(rng.integers(0, prm.t, (1, n), dtype=np.uint64)))
    rlk = key(10)
    n_fold = 6
    n_block = len([s for s in range(20) if d2 << s <= n // 4]) + 1
    fold = [key(20 + i) for i in range(n_fold)]
    block = [key(40 + i) for i in range(n_block)]
    tau = B                                               # opens the second ciphertext: replays are idempotent
    scores, context = ctx.empty_ct(heads, n_cts), ctx.empty_ct(heads)
    step = lambda: ctx.decode_step(q, a, cache, heads, n_cts, stride, d2, tau, rows, masks, rlk, fold, block,
                                   scores=scores, context=context)
    if hoisted:                                           # folding sums in rounds of hoisted rotation sums
        rf = [key(60 + i % 4) for i in range(len(ctx.round_galois(0, d2, 3)))]
        rb = [key(70 + i % 4) for i in range(len(ctx.round_galois(1, d2, 2)))]
        step = lambda: ctx.decode_step_hoisted(q, a, cache, heads, n_cts, stride, d2, tau, rows, masks, rlk, 3, rf,
                                               2, rb, scores=scores, context=context)
    say("eager step")
    step()
    torch.cuda.synchronize()
    want = (scores.clone(), context.clone(), cache.clone())

    say("capture")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                            # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for rep in range(3):
        say(f"replay {rep}")
        scores.zero_(); context.zero_(); cache.copy_(cache0)
        tmp = ctx.add(q, q, 2, heads)                     # eager work of the library between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(scores, want[0]) and torch.equal(context, want[1]) and torch.equal(cache, want[2]), rep
        del tmp
