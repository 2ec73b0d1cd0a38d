"""Micro-benchmarks of the library's building blocks (run on a GPU machine).

    python -m paper_2602_08798_amd.microbench modmul   FP64-FMA vs 32-bit-integer Barrett modular multiply
    python -m paper_2602_08798_amd.microbench exchange wave-local regrouping through LDS vs v_permlane32_swap
    python -m paper_2602_08798_amd.microbench ntt      forward/inverse transform throughput vs number of rows
    python -m paper_2602_08798_amd.microbench copy     plain device copy of known size (counter calibration)
    python -m paper_2602_08798_amd.microbench c5curve  the scaled configuration: per-step time over its 64 decode steps
    python -m paper_2602_08798_amd.microbench prefill  the prompt configuration: appends, Q K^T, score compaction, A V
    python -m paper_2602_08798_amd.microbench mulrelin mult+relin rate against batch size, whole and in chunks
    python -m paper_2602_08798_amd.microbench cpvm     one token times the 36 plaintext 768 x 64 matrices of a layer's Q, K, V

Kernel durations printed by `ntt` include the host-side staging of the prime-index table that the
public transform entry point performs; use `rocprofv3 --kernel-trace` around it for kernel-only times.
"""
import sys

import torch

from workloads import PRESETS

from . import Context


def _time(fn, reps):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps      # microseconds


def modmul(preset="C2"):
    ctx = Context(PRESETS[preset])
    cus, lanes_per_cu_cycle, clk = 256, 64, 2.4e9
    for waves in (1, 2, 4, 8):
        lanes = cus * 4 * 64 * waves
        for kind, name in ((0, "fp64-fma"), (1, "int-barrett")):
            out = torch.empty(lanes, dtype=torch.int64, device="cuda")
            iters = 2048
            us = _time(lambda: ctx.bench_modmul(kind, lanes, iters, out), 3)
            rate = lanes * iters * 2 / (us * 1e-6)
            slots = cus * lanes_per_cu_cycle * clk / rate
            print(f"waves/SIMD={waves} {name:12s} {us:9.1f} us  {rate / 1e12:6.3f} T modmul/s  "
                  f"{slots:5.1f} lane-cycles/modmul", flush=True)
    a, b = ctx.bench_modmul(0, 4096, 64), ctx.bench_modmul(1, 4096, 64)
    torch.cuda.synchronize()
    assert torch.equal(a, b), "the two arithmetic kinds disagree"
    print("both kinds produce identical residues")


def exchange(preset="C2"):
    """The regrouping of 8 doubles per lane between lanes 32 apart: LDS round trip against
    v_permlane32_swap, in clocks per exchange and compute unit (16 waves per unit, 2.4 GHz)."""
    ctx = Context(PRESETS[preset])
    blocks, iters = 256 * 4, 4096
    res = []
    for kind, name in ((0, "LDS (8 ds_write_b64 + 8 ds_read_b64 per lane)"), (1, "v_permlane32_swap (16 per lane)")):
        out = torch.empty(blocks * 1024, dtype=torch.float64, device="cuda")
        us = _time(lambda: ctx.bench_exchange(kind, blocks, iters, out), 3)
        clk = us * 1e-6 * 2.4e9 / (iters * (blocks / 256))       # per exchange of one workgroup's 16 waves
        print(f"{name:48s} {us:9.1f} us  {clk:7.1f} clk per exchange of a 1024-thread workgroup "
              f"({clk / 16:5.1f} per wave)", flush=True)
        res.append(out.clone())
    torch.cuda.synchronize()
    assert torch.equal(res[0], res[1]), "the two exchanges disagree"
    print("both kinds leave identical values")


def ntt(preset="C2", sizes=(512, 4096), reps=5):
    prm = PRESETS[preset]
    ctx = Context(prm)
    L = prm.k + prm.nsp
    for n in sizes:
        idx = [i % L for i in range(n)]
        x = torch.randint(0, 1 << 49, (n, prm.n), dtype=torch.int64, device="cuda")
        y = torch.empty_like(x)
        for inv in (False, True):
            f = (lambda: ctx.ntt_inverse(x, idx, out=y)) if inv else (lambda: ctx.ntt_forward(x, idx, out=y))
            us = _time(f, reps)
            print(f"{preset} {'inv' if inv else 'fwd'} rows={n:5d} {us:9.2f} us/call (host staging included)  "
                  f"{us * 1e3 / n:7.1f} ns/row", flush=True)


def copy(mib=256):
    n = mib * 1024 * 1024 // 8
    x = torch.randint(0, 1 << 49, (n,), dtype=torch.int64, device="cuda")
    y = torch.empty_like(x)
    us = _time(lambda: y.copy_(x), 10)
    print(f"copy of {mib} MiB (read {mib} MiB + write {mib} MiB): {us:.1f} us  {2 * n * 8 / us / 1e3:.0f} GB/s")


def c5curve(steps=64):
    """16 heads, N = 16384, cache growing from token 512 to 575 (the third ciphertext of every cache
    fills up; the number of ciphertexts read stays at 3, so the curve is flat by construction)."""
    import time
    from workloads import configs
    from .binding import to_device
    st = configs.c5_inputs()
    ctx = Context(st["prm"])
    H, S, d2 = st["heads"], st["stride"], st["d2"]
    cache = to_device(st["cache"])
    masks = ctx.plain_prepare(to_device(st["masks"]))
    rlk = ctx.ksk_prepare(to_device(st["rlk"]))
    gk = {g: ctx.ksk_prepare(to_device(k)) for g, k in st["gk"].items()}
    fold, block = [gk[g] for g in st["fold"]], [gk[g] for g in st["block"]]
    times = []
    for i in range(steps):
        si = st["step_inputs"](i)
        C = si["n_cts"]
        q, a, rows = to_device(si["q"]), to_device(si["a"]), to_device(si["rows"])
        scores, context = ctx.empty_ct(H, C), ctx.empty_ct(H)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.decode_step(q, a, cache, H, C, S, d2, 512 + i, rows, masks, rlk, fold, block, scores=scores,
                        context=context)
        torch.cuda.synchronize()
        times.append((time.perf_counter() - t0) * 1e3)
        print(f"step {i:2d} token {512 + i} ciphertexts read per cache {C}: {times[-1]:.3f} ms", flush=True)
    warm = times[2:]
    print(f"steps 2..{steps - 1}: mean {sum(warm) / len(warm):.3f} ms, min {min(warm):.3f}, max {max(warm):.3f} "
          f"(single launches, host-timed with a synchronisation per step)")


def prefill():
    """12 heads, 128 prompt tokens, N = 8192: the four parts of the prompt's attention, each timed as a
    whole (host clock around three repetitions, inputs resident)."""
    import time
    from workloads import configs
    from .binding import to_device as dev
    st = configs.c3_inputs()
    ctx = Context(st["prm"])
    H, m, d2 = st["heads"], st["m"], st["d2"]
    masks = ctx.plain_prepare(dev(st["masks"]))
    rows = [dev(st["rows"][tau]) for tau in range(m)]
    key = lambda k: ctx.ksk_prepare(dev(k))
    gk = {g: key(k) for g, k in st["gk"].items()}
    rlk, gkr = key(st["rlk"]), [key(st["gk_right"][x]) for x in st["right"]]
    mask0 = ctx.plain_prepare(dev(st["mask0"][None, :]))
    q, a = dev(st["q"]), dev(st["a"])
    cache, out = ctx.empty_ct(2 * H), ctx.empty_ct(H, m)

    def timed(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / reps

    def appends():
        for tau in range(m):
            ctx.kv_append(cache, 1, 2 * H, tau, rows[tau], masks, d2)

    fold = [gk[x] for x in st["fold"]]
    parts = [
        (f"{2 * H * m} appends ({m} calls of {2 * H} caches)", appends),
        (f"Q K^T: {H} heads x {m} diagonals", lambda: ctx.prefill_qk(q, cache[:H], H, d2, rlk, fold, gk[st["g_blk"]],
                                                                      gk[st["g_swap"]], out=out)),
        (f"score compaction: {H * m} -> {H * m // min(d2, m // 2)} ciphertexts",
         lambda: ctx.prefill_repack(out, H, d2, mask0, gkr)),
        (f"A V: {H} heads x {m} products", lambda: ctx.prefill_av(a, cache[H:], H, d2, rlk, gk[st["g_blk"]],
                                                                  gk[st["g_swap"]])),
    ]
    total = 0.0
    part_ms = []
    for name, fn in parts:
        ms = timed(fn)
        total += ms
        part_ms.append(ms)
        print(f"{name:58s} {ms:8.2f} ms", flush=True)
    print(f"{'prompt attention of one layer':58s} {total:8.2f} ms")
    # the same with the rotated copies of K and V made by hoisted rotation series (one decomposition
    # per cache ciphertext, m - 1 = 127 keys of uniform residues: timing does not depend on them)
    n = st["prm"].n
    L = st["prm"].k + st["prm"].nsp
    copies = [ctx.ksk_prepare(torch.randint(0, 1 << 49, (st["prm"].dnum, 2, L, n), dtype=torch.int64, device="cuda"))
              for _ in range(m - 1)]
    qk_h = timed(lambda: ctx.prefill_qk_hoisted(q, cache[:H], H, d2, rlk, fold, copies, out=out))
    av_h = timed(lambda: ctx.prefill_av_hoisted(a, cache[H:], H, d2, rlk, copies))
    print(f"{'Q K^T with hoisted copies of K':58s} {qk_h:8.2f} ms", flush=True)
    print(f"{'A V with hoisted copies of V':58s} {av_h:8.2f} ms", flush=True)
    print(f"{'prompt attention of one layer, hoisted copies':58s} {part_ms[0] + qk_h + part_ms[2] + av_h:8.2f} ms")
    av_s = timed(lambda: ctx.prefill_av_hoisted(a, cache[H:], H, d2, rlk, copies, sum_before_scaling=True))
    print(f"{'A V, hoisted copies, products summed before one scaling':58s} {av_s:8.2f} ms", flush=True)
    av_h = av_s
    # and with the folding sum of every product in rounds of hoisted rotation sums
    for w in (2, 3):
        rk = [copies[i % len(copies)] for i in range(len(ctx.round_galois(0, d2, w)))]
        qk_r = timed(lambda: ctx.prefill_qk_hoisted(q, cache[:H], H, d2, rlk, rk, copies, out=out, fold_round_bits=w))
        print(f"{'Q K^T, hoisted copies, folding sums in rounds of %d bits' % w:58s} {qk_r:8.2f} ms", flush=True)
        print(f"{'prompt attention of one layer, that form':58s} {part_ms[0] + qk_r + part_ms[2] + av_h:8.2f} ms")


def mulrelin(preset="C2", batches=(12, 24, 48, 96, 192, 384, 768), chunks=(24, 48, 96, 192)):
    """Products per second against batch size: one call over the whole batch, and the same batch as
    back-to-back calls over chunks (whose intermediates stay in the 256 MiB last-level cache)."""
    prm = PRESETS[preset]
    ctx = Context(prm)
    top = max(batches)
    lim = min(prm.q + prm.p)                     # below every prime: valid residues in every row
    a = torch.randint(0, lim, (top, 2, prm.k, prm.n), dtype=torch.int64, device="cuda")
    b = torch.randint(0, lim, (top, 2, prm.k, prm.n), dtype=torch.int64, device="cuda")
    rlk = ctx.ksk_prepare(torch.randint(0, lim, (ctx.dnum, 2, ctx.L, prm.n), dtype=torch.int64, device="cuda"))
    out = ctx.empty_ct(top)
    for batch in batches:
        whole = _time(lambda: ctx.mul_relin(a, b, rlk, batch, out=out), 5)
        line = f"{preset} batch {batch:4d}: whole {batch / whole * 1e6:9.0f}/s ({whole:8.1f} us)"
        for c in chunks:
            if c >= batch:
                continue

            def chunked():
                for o in range(0, batch, c):
                    m = min(c, batch - o)
                    ctx.mul_relin(a[o:o + m], b[o:o + m], rlk, m, out=out[o:o + m])
            us = _time(chunked, 5)
            line += f"  | by {c}: {batch / us * 1e6:9.0f}/s"
        print(line, flush=True)
    # where the time of a saturating batch goes (every launch bracketed by events: sequential, kernel time)
    ctx.profile_begin()
    for _ in range(3):
        ctx.mul_relin(a, b, rlk, top, out=out)
    torch.cuda.synchronize()
    stats = ctx.profile_end()
    total = sum(s["total_ms"] for s in stats)
    for s in sorted(stats, key=lambda s: -s["total_ms"]):
        if s["launches"]:
            us = s["total_ms"] * 1e3 / s["launches"]
            print(f"  {s['name']:24s} {us:8.1f} us/launch  {s['algo_bytes'] / s['launches'] / us / 1e3:7.0f} GB/s"
                  f"  {100 * s['total_ms'] / total:5.1f} % of the batch of {top}", flush=True)


def cpvm(preset="C2", d2=64, n_diag=8, heads=12):
    """Ciphertext-plaintext vector-matrix product of the decode step at the sizes of the paper's
    CT x PT table (d1 = 768, d2 = 64, N = 8192: tiles of 1024 slots, 8 diagonals per matrix), for the
    3 * heads matrices of one layer's Q, K and V projections (random residues: timing only)."""
    prm = PRESETS[preset]
    ctx = Context(prm)
    units = 3 * heads
    lim = min(prm.q + prm.p)
    x = torch.randint(0, lim, (1, 2, prm.k, prm.n), dtype=torch.int64, device="cuda")
    diags = ctx.plain_prepare(torch.randint(0, prm.t, (units * n_diag, prm.n), dtype=torch.int64, device="cuda"))
    key = lambda: ctx.ksk_prepare(torch.randint(0, lim, (ctx.dnum, 2, ctx.L, prm.n), dtype=torch.int64,
                                                device="cuda"))
    shift = [key() for _ in range(n_diag.bit_length() - 1)]
    block = [key() for _ in range((prm.n // d2).bit_length() - 1)]
    out = ctx.empty_ct(units)
    fn = lambda: ctx.cpvm(x, diags, units, n_diag, d2, shift, block, out=out)
    us = _time(fn, 20)
    print(f"{preset}: one token x {units} matrices (768 x {d2}, {n_diag} diagonals each): {us:8.1f} us "
          f"= {us / units:6.2f} us per matrix", flush=True)
    ctx.profile_begin()
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    for s in sorted(ctx.profile_end(), key=lambda s: -s["total_ms"]):
        if s["launches"]:
            print(f"  {s['name']:24s} {s['launches'] // 3:3d} launches  {s['total_ms'] * 1e3 / 3:8.1f} us per call", flush=True)
    copies = [key() for _ in range(n_diag - 1)]
    us_h = _time(lambda: ctx.cpvm_hoisted(x, diags, units, n_diag, d2, copies, block, out=out), 20)
    print(f"{preset}: the same with the token's {n_diag - 1} copies as one hoisted rotation series: {us_h:8.1f} us", flush=True)
    for w in (2, 3, 4):
        rk = [key() for _ in range(len(ctx.round_galois(1, d2, w)))]
        us_r = _time(lambda: ctx.cpvm_hoisted(x, diags, units, n_diag, d2, copies, rk, out=out, block_round_bits=w), 20)
        print(f"{preset}: hoisted copies and the sum over residue classes in rounds of {w} bits: {us_r:8.1f} us", flush=True)


if __name__ == "__main__":
    what = sys.argv[1] if len(sys.argv) > 1 else "modmul"
    if what == "mulrelin" and len(sys.argv) > 2:      # e.g. `mulrelin 768`: that batch only
        mulrelin(batches=tuple(int(a) for a in sys.argv[2:]))
    else:
        {"modmul": modmul, "exchange": exchange, "ntt": ntt, "copy": copy, "c5curve": c5curve, "prefill": prefill,
         "mulrelin": mulrelin, "cpvm": cpvm}[what]()
