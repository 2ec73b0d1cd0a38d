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
step is timed as one call in four forms, K steps each: cg_decode_step (plain
cache), cg_decode_step_ext (the products read a transformed copy of the cache,
which the step keeps up to date), and cg_decode_step_hoisted without and with
that copy (the same products with both folding sums regrouped into rounds of
hoisted rotation sums: 2 + 3 dependent key switches after the
relinearisations instead of 6 + 7, for 14 + 13 rotation keys instead of 6 + 7;
the context's 4 products per head are summed as tensor products and scaled
once; the results decrypt to the same slots and each form is checked against
the oracle's definition of that form).  The fastest is the headline `value`, the
others are listed beside it.  --serial times three calls in sequence instead
and nothing else (profiling runs; with --hoisted the hoisted calls).

Prints ONE JSON line.  `roofline` describes the kernel class with the largest
share of the step, timed with HIP events by the library itself in a further
pass over the same work issued as three calls in sequence (so that each
kernel has the device to itself while it is timed): its algorithmic bytes per
second against the HBM peak and its FP64 vector instructions per second
against the FP64 vector peak, `bound` naming the larger fraction; `roofline.step`
gives the same two fractions for the whole step (compulsory bytes: the step's
input and output ciphertexts and its keys, once each).  `cpu_baseline` times
the CPU oracle on the whole step of the same workload (a few seconds on the
host's cores) and checks every output ciphertext of the GPU step against it.
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0               # MI355X published HBM3E bandwidth
FP64_VALU_PEAK_TFLOPS = 78.6        # MI355X published vector FP64 (an FMA counts as two operations)
FP64_PEAK_LANE_INSTR = FP64_VALU_PEAK_TFLOPS * 1e12 / 2.0   # lane-instructions per second

# FP64 vector instructions (per lane) that one work item of each kernel class executes at N = 8192
# with three ciphertext primes: instructions per thread counted in the generated code of each
# instantiation, times the threads of a workgroup (transform kernels: one item = one residue row);
# for the pointwise kernels instructions per thread on the path taken, times the threads per batch
# unit.  The table and its derivation are in profiles/fp64_instruction_counts.txt.
FP64_LANE_INSTR_PER_ITEM = {
    "ntt_fwd<mul,q-rows>": 472 * 1024,
    "ntt_fwd<mul,aux-rows>": 936 * 1024,
    "ntt_fwd<modup>": 528 * 1024,
    "ntt_fwd<rows>": 472 * 1024,
    "ntt_fwd<plain>": 514 * 1024,
    "ntt_inv<tensor>": 760 * 1024,
    # tensor products of the n units of a group summed on the way in: 560 outside the loop over the units,
    # per unit 136 (components 0 and 2) or 232 (component 1), 168 on average
    "ntt_inv<tensor_sum>": 560 * 1024,
    "ntt_inv<tensor_sum> per unit": 168 * 1024,
    "ntt_inv<u64>": 616 * 1024,
    "ntt_inv<mul_plain>": 688 * 1024,
    "ntt_inv<ks_inner>": 728 * 1024,
    # summed inner product of n_rot rotations: 560 per thread outside the rotation loop, 200 per rotation
    "ntt_inv<ks_sum>": 560 * 1024,
    "ntt_inv<ks_sum> per rotation": 200 * 1024,
    "scale": 373 * 3 * 8192,
    "moddown": 320 * 8192,
    # one thread per pair of coefficients and prime: about 100 outside the rotation loop, 10 per rotation
    # on the c0 half
    "moddown<sum>": 100 * 3 * 8192,
    "moddown<sum> per rotation": 10 * 3 * 4096,
    "sum_groups": 16 * 9 * 8192,
    "add": 6 * 8192,
}

ROOT = os.path.dirname(os.path.abspath(__file__))

FORMS = ("plain", "ext", "hoisted", "hoisted_ext")


def kernel_sources_digest():
    """SHA-256 over the device code (the kernel headers): stored counter readings are only quoted for
    the kernels they were taken on."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2602_08798_amd", "csrc")
    for f in ("kernels.hpp", "modarith.hpp", "tables.hpp"):
        h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()


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
        # the folding sums in rounds: elements in the library's key order, stand-in keys drawn per element
        # bits per round (scores: 6 bits, context: 7): the measured optimum on MI355X
        self.w_fold, self.w_block = configs.C4_ROUND_BITS
        self.sum_first = configs.C4_SUM_BEFORE_SCALING
        self.g_fold_rounds = ctx.round_galois(0, self.d2, self.w_fold)
        self.g_block_rounds = ctx.round_galois(1, self.d2, self.w_block)
        self.h_gk_rounds = configs.galois_keys("C4", sorted(set(self.g_fold_rounds + self.g_block_rounds)))
        self.gk_rounds = {gal: ctx.ksk_prepare(dev(k)) for gal, k in self.h_gk_rounds.items()}
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

    def step_hoisted(self, transformed_cache=True):
        """The step with both folding sums in rounds of hoisted rotation sums."""
        self.ctx.decode_step_hoisted(self.q, self.a, self.cache, self.heads, self.n_cts, self.stride, self.d2,
                                     self.tau, self.rows, self.masks, self.rlk, self.w_fold,
                                     [self.gk_rounds[g] for g in self.g_fold_rounds], self.w_block,
                                     [self.gk_rounds[g] for g in self.g_block_rounds], scores=self.scores,
                                     context=self.context, cache_ext=self.ext if transformed_cache else None,
                                     sum_before_scaling=self.sum_first)

    def step_hoisted_plain_cache(self):
        self.step_hoisted(transformed_cache=False)

    def step_serial_hoisted(self):
        c, H, C = self.ctx, self.heads, self.n_cts
        c.decode_scores_hoisted(self.q, self.kcache, H, C, self.d2, self.w_fold, self.rlk,
                                [self.gk_rounds[g] for g in self.g_fold_rounds], out=self.scores,
                                cache_stride_cts=self.stride)
        c.decode_context_hoisted(self.a, self.vcache, H, C, self.d2, self.w_block, self.rlk,
                                 [self.gk_rounds[g] for g in self.g_block_rounds], out=self.context,
                                 cache_stride_cts=self.stride, sum_before_scaling=self.sum_first)
        c.kv_append(self.cache, self.stride, 2 * H, self.tau, self.rows, self.masks, self.d2)

    def round_sizes(self, which):
        """Rotations per round, by the rule the library states for its rounds (as even as possible,
        longer rounds first); checked against the number of elements the library lists."""
        n_bits = len(self.g_block) if which else len(self.g_fold)
        w = self.w_block if which else self.w_fold
        rounds = -(-n_bits // w)
        lo, extra = divmod(n_bits, rounds)
        sizes = [(1 << (lo + (1 if r < extra else 0))) - 1 for r in range(rounds)]
        assert sum(sizes) == len(self.g_block_rounds if which else self.g_fold_rounds)
        return sizes

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
    def op_counts(self, hoisted=False):
        H, C = self.heads, self.n_cts
        if hoisted:
            mul = {"mul": H * C, "tensor_products_summed_before_one_scaling": H * C} if self.sum_first else {"mul": 2 * H * C}
            return {**mul, "relin": H * C + H,
                    "rotation_sums": H * C * len(self.round_sizes(0)) + H * len(self.round_sizes(1)),
                    "rotate": H * C * len(self.g_fold_rounds) + H * len(self.g_block_rounds), "append": 2 * H}
        return {"mul": 2 * H * C, "relin": H * C + H,
                "rotate": H * C * len(self.g_fold) + H * len(self.g_block), "append": 2 * H}

    def compulsory_bytes(self, hoisted=False):
        """What one step has to move whatever the implementation: every input ciphertext (K and V
        caches, queries, weights, new rows), every key and block mask it uses, once each, and every
        output ciphertext (scores, contexts, the ciphertext each cache was appended to)."""
        H, C = self.heads, self.n_cts
        ct = 2 * self.prm.k * self.n * 8
        key = self.prm.dnum * 2 * (self.prm.k + self.prm.nsp) * self.n * 8
        cts_in = 2 * H * C + H + H * C + 2 * H
        cts_out = H * C + H + 2 * H
        n_keys = 1 + (len(self.g_fold_rounds) + len(self.g_block_rounds) if hoisted
                      else len(self.g_fold) + len(self.g_block))
        return (cts_in + cts_out) * ct + n_keys * key + self.n * 8


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
    fp64 = rows * 520 * 1024 / (ms * 1e-3)          # the uint64-out storer: 520 instructions per thread
    return {"metric": "negacyclic NTT rows/s at N=8192 (%d rows per launch, kernel time)" % rows,
            "value": round(rows / (ms * 1e-3), 1), "unit": "1/s", "avg_launch_us": round(ms * 1e3, 1),
            "algo_GBps": round(gbs, 1), "hbm_frac": round(gbs / HBM_PEAK_GBS, 4),
            "fp64_valu_frac": round(fp64 / FP64_PEAK_LANE_INSTR, 4)}


def mult_relin_rates(torch, P, ws, steps):
    """ct-ct mult+relin per second: N = 8192 (three primes) at batch 16, 48 and 768, and the small
    configuration (C1: N = 4096, two primes, its 16 seeded pairs)."""
    from workloads import configs
    out = {}
    H, C = ws.heads, ws.n_cts
    b_dense = ws.cache[:H * C]
    for batch in (16, H * C, 16 * H * C):
        reps = -(-batch // (H * C))
        a = ws.a.repeat(reps, 1, 1, 1)[:batch].contiguous()
        b = b_dense.repeat(reps, 1, 1, 1)[:batch].contiguous()
        o = ws.ctx.empty_ct(batch)
        fn = lambda: ws.ctx.mul_relin(a, b, ws.rlk, batch, out=o)
        for _ in range(3):
            fn()
        ms = timed(torch, fn, max(5, steps) if batch <= H * C else 5)
        out["n8192_batch_%d" % batch] = round(batch / (ms * 1e-3), 1)
        del a, b, o
    st = configs.c1_inputs()
    ctx = P.Context(st["prm"])
    a, b = P.to_device(st["a"]), P.to_device(st["b"])
    rlk = ctx.ksk_prepare(P.to_device(st["rlk"]))
    batch = a.shape[0]
    o = ctx.empty_ct(batch)
    fn = lambda: ctx.mul_relin(a, b, rlk, batch, out=o)
    for _ in range(3):
        fn()
    ms = timed(torch, fn, max(5, steps))
    out["n4096_k2_batch_%d" % batch] = round(batch / (ms * 1e-3), 1)
    ctx.close()
    return out


def c5_curve(torch, P):
    """The scaled configuration (16 heads, N = 16384, 6+2 primes): all 64 successive decode steps
    with cache growth (token 512 + i goes into the third ciphertext of every cache, which the
    products read), each step timed on its own.  Step 0's seeded inputs are reused for the later
    steps (kernel time does not depend on the residues); the append position is the real one."""
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
    step = lambda tau: ctx.decode_step(q, a, cache, H, C, S, d2, tau, rows, masks, rlk, fold, block,
                                       scores=scores, context=context)
    for _ in range(3):
        step(512)
    per = []
    for i in range(st["steps"]):
        per.append(timed(torch, lambda: step(512 + i), 1))
    # the same steps with the folding sums in rounds of hoisted rotation sums (stand-in keys per element)
    wf, wb = configs.C4_ROUND_BITS
    g_fold, g_block = ctx.round_galois(0, d2, wf), ctx.round_galois(1, d2, wb)
    rk = {g: ctx.ksk_prepare(dev(k)) for g, k in configs.galois_keys("C5", sorted(set(g_fold + g_block))).items()}
    kf, kb = [rk[g] for g in g_fold], [rk[g] for g in g_block]
    hstep = lambda tau: ctx.decode_step_hoisted(q, a, cache, H, C, S, d2, tau, rows, masks, rlk, wf, kf, wb, kb,
                                                scores=scores, context=context,
                                                sum_before_scaling=configs.C4_SUM_BEFORE_SCALING)
    for _ in range(3):
        hstep(512)
    per_h = []
    for i in range(st["steps"]):
        per_h.append(timed(torch, lambda: hstep(512 + i), 1))
    ctx.close()
    return {"metric": "C5 scaled decode step ms/token (one layer: 16 heads, N=16384, 6+2 primes), "
                      "64 successive steps with cache growth",
            "value": round(float(np.mean(per)), 4), "unit": "ms", "min": round(min(per), 4),
            "max": round(max(per), 4), "first": round(per[0], 4), "last": round(per[-1], 4),
            "hoisted_rounds": {"round_bits": [wf, wb], "value": round(float(np.mean(per_h)), 4),
                               "min": round(min(per_h), 4), "max": round(max(per_h), 4)}}


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
    # the token's copies as one hoisted series and the final sums in rounds of 3 bits (stand-in keys)
    key = lambda: ctx.ksk_prepare(rnd(lim, ctx.dnum, 2, ctx.L, prm.n))
    copies = [key() for _ in range(n_diag - 1)]
    rounds = [key() for _ in range(len(ctx.round_galois(1, d2, 3)))]
    fh = lambda: ctx.cpvm_hoisted(x, diags, units, n_diag, d2, copies, rounds, out=out, block_round_bits=3)
    fh()
    ms_h = timed(torch, fh, reps)
    return {"metric": "decode-step CT x PT projections of one layer (one token x 36 matrices of 768 x 64)",
            "value": round(ms * 1e3, 1), "unit": "us",
            "hoisted_copies_and_rounds_of_3_bits": round(ms_h * 1e3, 1)}


def cpu_baseline(ws: DecodeStep, hoisted: bool):
    """Time the oracle on the whole step in the headline's form (same seeded inputs) and compare
    every output ciphertext of the GPU step with it; then run the step once in the other family of
    forms and compare that with the oracle's definition of it as well."""
    from oracle import Oracle, run_configs
    torch = ws.torch
    orc = Oracle(ws.prm)
    H, C, S = ws.heads, ws.n_cts, ws.stride
    idx = ws.tau // ws.B

    def check(form_hoisted):
        (ws.step_hoisted if form_hoisted else ws.step)()
        torch.cuda.synchronize()
        gpu_scores, gpu_context, gpu_cache = (ws.P.to_host(t) for t in (ws.scores, ws.context, ws.cache))
        t0 = time.perf_counter()
        if form_hoisted:
            want = run_configs.run_c4_hoisted(orc, ws.st, ws.w_fold, ws.w_block, ws.h_gk_rounds, sum_first=ws.sum_first)
        else:
            want = run_configs.run_c4(orc, ws.st)
        sec = time.perf_counter() - t0
        ok = all(np.array_equal(gpu_scores[h, c], want[f"score{h}_{c}"]) for h in range(H) for c in range(C))
        ok = ok and all(np.array_equal(gpu_context[h], want[f"context{h}"]) for h in range(H))
        ok = ok and all(np.array_equal(gpu_cache[c * S + idx], want[f"cache{c}"]) for c in range(2 * H))
        return sec, bool(ok)

    step_s, ok = check(hoisted)
    other_s, other_ok = check(not hoisted)
    counts = ws.op_counts(hoisted)
    work = ", ".join(f"{v} {k}" for k, v in counts.items())
    return {
        "value": round(step_s * 1e3, 1), "unit": "ms/token (one layer)",
        "cores": orc.threads, "kind": "oracle",
        "sample": f"the whole step of the same seeded workload in the timed form ({work}): "
                  f"{round(step_s * orc.threads, 1)} core-seconds",
        "gpu_matches_oracle_on_every_output": ok,
        "other_form": {"form": "rotate-and-add chains" if hoisted else "folding sums in rounds of hoisted rotations",
                       "oracle_ms": round(other_s * 1e3, 1), "gpu_matches_oracle_on_every_output": other_ok},
    }


def stored_traffic(kernel_name):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter runs
    (profiles/hbm_traffic.json), or None when they were taken on other kernel sources."""
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(tpath):
        return None, "no counter file"
    doc = json.load(open(tpath))
    if doc.get("kernel_sources_sha256") != kernel_sources_digest():
        return None, "the committed counter readings were taken on other kernel sources"
    return doc.get("bytes_per_launch", {}).get(kernel_name), None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--serial", action="store_true",
                    help="issue the step as three calls in sequence and nothing else: every kernel has the "
                         "device to itself (profiling runs)")
    ap.add_argument("--hoisted", action="store_true", help="with --serial: the hoisted calls")
    ap.add_argument("--one-call", choices=list(FORMS), default=None,
                    help="time only this form of the one-call step and nothing else (profiling runs)")
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
    fns = {"plain": ws.step_plain_cache, "ext": ws.step, "hoisted": ws.step_hoisted_plain_cache,
           "hoisted_ext": ws.step_hoisted}
    profiling_run = args.serial or args.one_call is not None
    per_form, ms_serial = {}, None
    if args.serial:
        fn = ws.step_serial_hoisted if args.hoisted else ws.step_serial
        for _ in range(args.warmup):
            fn()
        ms = ms_serial = timed(torch, fn, args.steps)
        form = "serial_hoisted" if args.hoisted else "serial"
    elif args.one_call:
        fn = fns[args.one_call]
        for _ in range(args.warmup):
            fn()
        ms = timed(torch, fn, args.steps)
        form = args.one_call
    else:
        for _ in range(args.warmup):
            for fn in fns.values():
                fn()
        for name, fn in fns.items():
            per_form[name] = timed(torch, fn, args.steps)
        form = min(per_form, key=per_form.get)
        ms = per_form[form]
    hoisted = "hoisted" in form
    serial_fn = ws.step_serial_hoisted if hoisted else ws.step_serial
    if not profiling_run:
        ms_serial = timed(torch, serial_fn, args.steps)

    kernels, roofline = [], None
    if args.one_call is None:
        # a pass over the same work, one call after the other, with the library's event
        # bracketing for per-kernel figures
        ws.ctx.profile_begin(200 * args.steps)
        for _ in range(args.steps):
            serial_fn()
        stats = ws.ctx.profile_end()
        H, C, L2 = ws.heads, ws.n_cts, 2 * (ws.prm.k + ws.prm.nsp)
        # rotation-rows and rotation-units of the summed kernels, per step
        rot_rows = sum(H * C * L2 * r for r in ws.round_sizes(0)) + sum(H * L2 * r for r in ws.round_sizes(1))
        rot_units = sum(H * C * r for r in ws.round_sizes(0)) + sum(H * r for r in ws.round_sizes(1))
        fp64_step = 0.0
        for s in stats:
            sec = s["total_ms"] * 1e-3
            gbs = s["algo_bytes"] / sec / 1e9
            fp64 = s["work_items"] * FP64_LANE_INSTR_PER_ITEM.get(s["name"], 0)
            if s["name"] == "ntt_inv<ks_sum>":
                fp64 += args.steps * rot_rows * FP64_LANE_INSTR_PER_ITEM["ntt_inv<ks_sum> per rotation"]
            if s["name"] == "ntt_inv<tensor_sum>":     # its rows each take in the n_cts units of a head
                fp64 += s["work_items"] * C * FP64_LANE_INSTR_PER_ITEM["ntt_inv<tensor_sum> per unit"]
            if s["name"] == "moddown<sum>":
                fp64 += args.steps * rot_units * FP64_LANE_INSTR_PER_ITEM["moddown<sum> per rotation"]
            fp64_step += fp64 / args.steps
            kernels.append({"name": s["name"], "launches_per_step": s["launches"] / args.steps,
                            "avg_us": round(s["total_ms"] * 1e3 / s["launches"], 2),
                            "ms_per_step": round(s["total_ms"] / args.steps, 4),
                            "algo_GBps": round(gbs, 1), "hbm_frac": round(gbs / HBM_PEAK_GBS, 4),
                            "fp64_valu_frac": round(fp64 / sec / FP64_PEAK_LANE_INSTR, 4)})
        kernels.sort(key=lambda k: -k["ms_per_step"])
        dom = kernels[0]
        dom_stat = next(s for s in stats if s["name"] == dom["name"])
        traffic, traffic_note = stored_traffic(dom["name"])
        bound = "hbm" if dom["hbm_frac"] >= dom["fp64_valu_frac"] else "alu"
        step_bytes = ws.compulsory_bytes(hoisted)
        if form.endswith("ext"):
            # the timed step read the cache's transformed copy: no lift and forward transform of the 2 H C
            # cache operands (2 polynomials each: k ciphertext-prime rows, k + 1 auxiliary rows), but
            # the same for the 2 H ciphertexts the step appended to
            saved = 2 * (2 * ws.heads * ws.n_cts - 2 * ws.heads)
            fp64_step -= saved * (ws.prm.k * FP64_LANE_INSTR_PER_ITEM["ntt_fwd<mul,q-rows>"]
                                  + (ws.prm.k + 1) * FP64_LANE_INSTR_PER_ITEM["ntt_fwd<mul,aux-rows>"])
        roofline = {
            "bound": bound, "kernel": dom["name"],
            "achieved": dom["algo_GBps"] if bound == "hbm" else round(dom["fp64_valu_frac"] * FP64_VALU_PEAK_TFLOPS, 2),
            "peak": HBM_PEAK_GBS if bound == "hbm" else FP64_VALU_PEAK_TFLOPS,
            "unit": "GB/s" if bound == "hbm" else "TFLOP/s",
            "frac": dom["hbm_frac"] if bound == "hbm" else dom["fp64_valu_frac"],
            "traffic": traffic,
            "hbm_frac": dom["hbm_frac"], "fp64_valu_frac": dom["fp64_valu_frac"],
            "algo_bytes_per_launch": dom_stat["algo_bytes"] / dom_stat["launches"],
            "avg_launch_us": dom["avg_us"],
            "note": "neither unit is near its peak: at the step's launch sizes (96 to 1008 rows on 256 compute "
                    "units) a kernel's time is the latency of one or two rows per unit, not a rate",
            "step": {"ms": round(ms, 4), "compulsory_bytes": step_bytes,
                     "hbm_frac": round(step_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "fp64_lane_instr": round(fp64_step),
                     "fp64_valu_frac": round(fp64_step / (ms * 1e-3) / FP64_PEAK_LANE_INSTR, 4)},
        }
        if traffic_note:
            roofline["traffic_note"] = traffic_note

    secondary = None
    if not args.no_secondary and not profiling_run:
        rates = mult_relin_rates(torch, ws.P, ws, args.steps)
        secondary = {"metric": "ct-ct mult+relin/sec at N=8192", "value": rates["n8192_batch_48"],
                     "unit": "1/s", "batch": 48, "all": rates,
                     "transform": transform_rate(torch, ws),
                     "ct_pt_projections": cpvm_layer_us(torch, ws),
                     "scaled_config": c5_curve(torch, ws.P)}

    rounds = (f"both folding sums in rounds of hoisted rotation sums ({ws.w_fold} / {ws.w_block} bits per round: "
              f"{len(ws.round_sizes(0))} + {len(ws.round_sizes(1))} dependent key switches after the relinearisations "
              f"instead of {len(ws.g_fold)} + {len(ws.g_block)})"
              + ("; the context's products over the cache ciphertexts summed before one scaling" if ws.sum_first else ""))
    launch = {"serial": "three calls in sequence",
              "serial_hoisted": "three calls in sequence, " + rounds,
              "ext": "cg_decode_step_ext: scores, context and append side by side on three streams; the products "
                     "read the cache's transformed copy and the step refreshes the copy of the 24 ciphertexts it "
                     "appends to",
              "plain": "cg_decode_step: scores, context and append side by side on three streams",
              "hoisted": "cg_decode_step_hoisted: three streams, " + rounds,
              "hoisted_ext": "cg_decode_step_hoisted with the cache's transformed copy: three streams, " + rounds}[form]
    config = {"workload": "C4: decode step, 12 heads x d=64, 512-token encrypted KV cache, N=8192, "
                          "3+1 primes < 2^50, t=65537", "ops_per_step": ws.op_counts(hoisted),
              "arithmetic": "exact integer residues < 2^50 carried in FP64 registers; uint64 at the ABI",
              "derived_12_layers_ms_per_token": round(12 * ms, 3), "form": form, "launch": launch}
    if per_form:
        config["ms_per_step_cg_decode_step_ext"] = round(per_form["ext"], 4)
        config["ms_per_step_cg_decode_step"] = round(per_form["plain"], 4)
        config["ms_per_step_cg_decode_step_hoisted_ext"] = round(per_form["hoisted_ext"], 4)
        config["ms_per_step_cg_decode_step_hoisted"] = round(per_form["hoisted"], 4)
    if ms_serial is not None:
        config["ms_per_step_three_calls_in_sequence"] = round(ms_serial, 4)
    result = {
        "metric": "encrypted decode-step ms/token at 512 ctx",
        "value": round(ms, 4), "unit": "ms/token (one layer: 12 heads, CT x CT path)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": config,
        "secondary": secondary,
        "roofline": roofline,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline and not profiling_run:
        result["cpu_baseline"] = cpu_baseline(ws, hoisted)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
