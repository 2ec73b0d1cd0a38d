#!/usr/bin/env python3
"""Benchmark of the encrypted decode step at 512-token context on one MI355X.

One step = the whole ciphertext x ciphertext hot path of one Transformer layer
for one generated token (GPT-2-small shape: 12 heads x d = 64, N = 8192, three
50-bit ciphertext primes + one special prime):
    scores   q . K^T  over 12 x 4 cache ciphertexts (mul, relin, 6 rotate-and-add each)
    context  a . V    over 12 x 4 cache ciphertexts (48 mul, 12 relin, 7 rotate-and-add each)
    append   the new K and V rows into 24 caches at token 512 (opens ciphertext 5)
Inputs are seeded uniform residues (stand-ins for ciphertexts and keys; see
workloads.synth) already resident in HBM when the timed region starts.  The
timed step is one cg_decode_step_ext call (the three parts side by side on three
streams, the products reading the transformed copy of the cache that earlier
steps maintain, this step refreshing the copy of the ciphertexts it appends to);
--serial times three plain calls in sequence instead.

Prints ONE JSON line.  `roofline` is for the kernel class with the largest
share of the step, timed with HIP events by the library itself in a further
pass over the same work issued as three calls in sequence (so that each
kernel has the device to itself while it is timed); `cpu_baseline` times the
CPU oracle on the whole step of the same workload (a few seconds on the host's
cores) and checks every output ciphertext of the GPU step against it.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
FP64_VALU_PEAK_TFLOPS = 78.6   # MI355X published vector FP64


class DecodeStep:
    """Device-resident state of the C4 workload and the calls of one step."""

    def __init__(self):
        import torch
        import paper_2602_08798_amd as P
        from workloads import configs
        self.torch, self.P = torch, P
        st = configs.c4_inputs()            # seeded stand-ins; host copies are kept for the oracle sample
        self.st = st
        self.prm = prm = st["prm"]
        self.heads, self.d2, self.n = st["heads"], st["d2"], prm.n
        self.B, self.n_cts, self.stride, self.tau = st["B"], st["n_cts"], st["stride"], st["tau"]
        self.ctx = ctx = P.Context(prm)
        H, C = self.heads, self.n_cts
        self.h_q, self.h_a, self.h_cache, self.h_rows = st["q"], st["a"], st["cache"], st["rows"]
        self.h_masks, self.h_rlk, self.h_gk = st["masks"], st["rlk"], st["gk"]
        self.g_fold, self.g_block = st["fold"], st["block"]
        dev = P.to_device
        self.q, self.a, self.rows = dev(self.h_q), dev(self.h_a), dev(self.h_rows)
        self.cache = dev(self.h_cache)                  # [K|V][head][stride] ciphertexts
        self.kcache = self.cache[:H * self.stride]
        self.vcache = self.cache[H * self.stride:]
        self.masks = ctx.plain_prepare(dev(self.h_masks))
        self.rlk = ctx.ksk_prepare(dev(self.h_rlk))
        self.gk = {gal: ctx.ksk_prepare(dev(k)) for gal, k in self.h_gk.items()}
        self.scores = ctx.empty_ct(H, C)
        self.context = ctx.empty_ct(H)
        ctx.workspace(H * C)
        # the cache's transformed copy (what earlier steps leave behind): every ciphertext the products read
        self.ext = ctx.empty_ext(2 * H * self.stride)
        ctx.cache_extend(self.cache, 2 * H, C, self.stride, self.ext)
        torch.cuda.synchronize()

    def step(self, transformed_cache=True):
        """One call: the three branches run side by side on the library's streams.  With the
        transformed copy of the cache the products skip the lift and forward transforms of the
        cache operands, and the step refreshes the copy of the ciphertext it appended to."""
        self.ctx.decode_step(self.q, self.a, self.cache, self.heads, self.n_cts, self.stride, self.d2, self.tau,
                             self.rows, self.masks, self.rlk, [self.gk[g] for g in self.g_fold],
                             [self.gk[g] for g in self.g_block], scores=self.scores, context=self.context,
                             cache_ext=self.ext if transformed_cache else None)

    def step_plain_cache(self):
        self.step(transformed_cache=False)

    def step_serial(self):
        """The same work as three calls in sequence (used for per-kernel timing: a kernel's
        duration only describes the kernel when it has the device to itself)."""
        c, H, C = self.ctx, self.heads, self.n_cts
        c.decode_scores(self.q, self.kcache, H, C, self.d2, self.rlk, [self.gk[g] for g in self.g_fold],
                        out=self.scores, cache_stride_cts=self.stride)
        c.decode_context(self.a, self.vcache, H, C, self.d2, self.rlk, [self.gk[g] for g in self.g_block],
                         out=self.context, cache_stride_cts=self.stride)
        c.kv_append(self.cache, self.stride, 2 * H, self.tau, self.rows, self.masks, self.d2)

    # per step: 96 mul, 60 relin, 372 rotations, 24 appends
    def op_counts(self):
        H, C = self.heads, self.n_cts
        return {"mul": 2 * H * C, "relin": H * C + H,
                "rotate": H * C * len(self.g_fold) + H * len(self.g_block), "append": 2 * H}


def timed(torch, fn, steps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def transform_rate(torch, ws, rows=16384, reps=5):
    """The transform kernel in its throughput regime: cg_ntt_forward over `rows` residue rows of
    N = 8192 (uint64 in, uint64 out: 2 x 64 KiB of algorithmic traffic per row), kernel time from
    the library's HIP-event bracketing."""
    prm = ws.prm
    L = prm.k + prm.nsp
    idx = [i % L for i in range(rows)]
    x = torch.randint(0, 1 << 49, (rows, prm.n), dtype=torch.int64, device="cuda")
    y = torch.empty_like(x)
    ws.ctx.ntt_forward(x, idx, out=y)
    torch.cuda.synchronize()
    ws.ctx.profile_begin(reps + 1)
    for _ in range(reps):
        ws.ctx.ntt_forward(x, idx, out=y)
    st = [s for s in ws.ctx.profile_end() if s["name"] == "ntt_fwd<rows>"][0]
    ms = st["total_ms"] / st["launches"]
    gbs = rows * prm.n * 16 / (ms * 1e-3) / 1e9
    return {"metric": "negacyclic NTT rows/s at N=8192 (%d rows per launch, kernel time)" % rows,
            "value": round(rows / (ms * 1e-3), 1), "unit": "1/s", "avg_launch_us": round(ms * 1e3, 1),
            "algo_GBps": round(gbs, 1), "hbm_frac": round(gbs / HBM_PEAK_GBS, 4)}


def c5_step_ms(torch, P, steps):
    """The scaled configuration (16 heads, N = 16384, 6+2 primes): first of its 64 decode steps, where
    the appended ciphertext is among those the products read."""
    from workloads import configs
    st = configs.c5_inputs()
    ctx = P.Context(st["prm"])
    H, S, d2 = st["heads"], st["stride"], st["d2"]
    dev = P.to_device
    cache = dev(st["cache"])
    masks = ctx.plain_prepare(dev(st["masks"]))
    rlk = ctx.ksk_prepare(dev(st["rlk"]))
    gk = {g: ctx.ksk_prepare(dev(k)) for g, k in st["gk"].items()}
    fold, block = [gk[g] for g in st["fold"]], [gk[g] for g in st["block"]]
    si = st["step_inputs"](0)
    C = si["n_cts"]
    q, a, rows = dev(si["q"]), dev(si["a"]), dev(si["rows"])
    scores, context = ctx.empty_ct(H, C), ctx.empty_ct(H)
    step = lambda: ctx.decode_step(q, a, cache, H, C, S, d2, 512, rows, masks, rlk, fold, block,
                                   scores=scores, context=context)
    for _ in range(3):
        step()
    ms = timed(torch, step, steps)
    ctx.close()
    return {"metric": "C5 scaled decode step ms/token (one layer: 16 heads, N=16384, 6+2 primes, step 0 of 64)",
            "value": round(ms, 4), "unit": "ms"}


def cpvm_layer_us(torch, ws, reps=20):
    """The decode step's CT x PT side at the sizes of the paper's CT x PT table: one token times the
    36 plaintext 768 x 64 matrices of a layer's Q, K and V projections (8 diagonals each at N = 8192)."""
    ctx, prm = ws.ctx, ws.prm
    units, n_diag, d2 = 3 * ws.heads, 8, ws.d2
    lim = min(prm.q + prm.p)
    rnd = lambda hi, *shape: torch.randint(0, hi, shape, dtype=torch.int64, device="cuda")
    x = rnd(lim, 1, 2, prm.k, prm.n)
    diags = ctx.plain_prepare(rnd(prm.t, units * n_diag, prm.n))
    shift = [ws.gk[g] for g in ws.g_fold[:3]]                  # keys for 3^1, 3^2, 3^4
    block = [ws.gk[g] for g in ws.g_block]
    out = ctx.empty_ct(units)
    fn = lambda: ctx.cpvm(x, diags, units, n_diag, d2, shift, block, out=out)
    fn()
    ms = timed(torch, fn, reps)
    return {"metric": "decode-step CT x PT projections of one layer (one token x 36 matrices of 768 x 64)",
            "value": round(ms * 1e3, 1), "unit": "us"}


def cpu_baseline(ws: DecodeStep):
    """Time the oracle on the whole step (same seeded inputs) and compare every output ciphertext
    of the GPU step with it."""
    from oracle import Oracle, run_configs
    orc = Oracle(ws.prm)
    H, C, S = ws.heads, ws.n_cts, ws.stride
    gpu_scores = ws.P.to_host(ws.scores)
    gpu_context = ws.P.to_host(ws.context)
    gpu_cache = ws.P.to_host(ws.cache)
    t0 = time.perf_counter()
    want = run_configs.run_c4(orc, ws.st)
    step_s = time.perf_counter() - t0
    idx = ws.tau // ws.B
    ok = all(np.array_equal(gpu_scores[h, c], want[f"score{h}_{c}"]) for h in range(H) for c in range(C))
    ok = ok and all(np.array_equal(gpu_context[h], want[f"context{h}"]) for h in range(H))
    ok = ok and all(np.array_equal(gpu_cache[c * S + idx], want[f"cache{c}"]) for c in range(2 * H))
    counts = ws.op_counts()
    return {
        "value": round(step_s * 1e3, 1), "unit": "ms/token (one layer)",
        "cores": orc.threads, "kind": "oracle",
        "sample": f"the whole step of the same seeded workload ({counts['mul']} products, {counts['relin']} "
                  f"relinearisations, {counts['rotate']} rotations, {counts['append']} appends): "
                  f"{round(step_s * orc.threads, 1)} core-seconds",
        "gpu_matches_oracle_on_every_output": bool(ok),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--serial", action="store_true",
                    help="time the three calls in sequence instead of the one-call step (profiling runs)")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the mult+relin/sec loops (used when profiling the step alone)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards by head with no "
              "collectives: heads are independent and keys replicated); rerun with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)

    ws = DecodeStep()
    step = ws.step_serial if args.serial else ws.step
    for _ in range(args.warmup):
        step()
    ms = timed(torch, step, args.steps)
    ms_serial = ms if args.serial else timed(torch, ws.step_serial, args.steps)
    ms_plain = timed(torch, ws.step_plain_cache, args.steps)

    # second pass over the same work, one call after the other, with the library's event
    # bracketing for per-kernel figures
    ws.ctx.profile_begin(200 * args.steps)
    for _ in range(args.steps):
        ws.step_serial()
    stats = ws.ctx.profile_end()
    kernels = []
    for s in stats:
        avg_us = s["total_ms"] * 1e3 / s["launches"]
        gbs = s["algo_bytes"] / (s["total_ms"] * 1e-3) / 1e9
        kernels.append({"name": s["name"], "launches_per_step": s["launches"] / args.steps,
                        "avg_us": round(avg_us, 2), "ms_per_step": round(s["total_ms"] / args.steps, 4),
                        "algo_GBps": round(gbs, 1), "hbm_frac": round(gbs / HBM_PEAK_GBS, 4)})
    kernels.sort(key=lambda k: -k["ms_per_step"])
    dom = kernels[0]
    dom_stat = next(s for s in stats if s["name"] == dom["name"])
    traffic = None
    tpath = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(dom["name"])
    roofline = {"bound": "hbm", "kernel": dom["name"], "achieved": dom["algo_GBps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(dom["algo_GBps"] / HBM_PEAK_GBS, 4),
                "traffic": traffic,
                "algo_bytes_per_launch": dom_stat["algo_bytes"] / dom_stat["launches"],
                "avg_launch_us": dom["avg_us"]}

    secondary = None
    if not args.no_secondary:
        # secondary metric: ct-ct mult+relin per second at N = 8192, batch 48
        H, C = ws.heads, ws.n_cts
        out2 = ws.ctx.empty_ct(H * C)
        b_dense = ws.cache[:H * C]
        mr = lambda: ws.ctx.mul_relin(ws.a, b_dense, ws.rlk, H * C, out=out2)
        mr()
        mr_ms = timed(torch, mr, max(5, args.steps))

        # same metric at a batch large enough to keep every compute unit busy for several rows
        big = 16 * H * C
        a_big = ws.a.repeat(16, 1, 1, 1)
        b_big = b_dense.repeat(16, 1, 1, 1)
        out_big = ws.ctx.empty_ct(big)
        mrb = lambda: ws.ctx.mul_relin(a_big, b_big, ws.rlk, big, out=out_big)
        for _ in range(3):
            mrb()
        mrb_ms = timed(torch, mrb, 5)
        del a_big, b_big, out_big
        secondary = {"metric": "ct-ct mult+relin/sec at N=8192", "value": round(H * C / (mr_ms * 1e-3), 1),
                     "unit": "1/s", "batch": H * C,
                     "value_at_batch_%d" % big: round(big / (mrb_ms * 1e-3), 1),
                     "transform": transform_rate(torch, ws),
                     "ct_pt_projections": cpvm_layer_us(torch, ws),
                     "scaled_config": c5_step_ms(torch, ws.P, 10)}

    result = {
        "metric": "encrypted decode-step ms/token at 512 ctx",
        "value": round(ms, 4), "unit": "ms/token (one layer: 12 heads, CT x CT path)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": "C4: decode step, 12 heads x d=64, 512-token encrypted KV cache, N=8192, "
                               "3+1 primes < 2^50, t=65537", "ops_per_step": ws.op_counts(),
                   "arithmetic": "exact integer residues < 2^50 carried in FP64 registers; uint64 at the ABI",
                   "derived_12_layers_ms_per_token": round(12 * ms, 3),
                   "launch": "three calls in sequence" if args.serial else
                             "cg_decode_step_ext: scores, context and append side by side on three streams; the "
                             "products read the cache's transformed copy and the step refreshes the copy of the "
                             "24 ciphertexts it appends to",
                   "ms_per_step_without_transformed_cache_copy": round(ms_plain, 4),
                   "ms_per_step_three_calls_in_sequence": round(ms_serial, 4)},
        "secondary": secondary,
        "roofline": roofline,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(ws)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
