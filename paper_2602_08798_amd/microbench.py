"""Micro-benchmarks of the library's building blocks (run on a GPU machine).

    python -m paper_2602_08798_amd.microbench modmul   FP64-FMA vs 32-bit-integer Barrett modular multiply
    python -m paper_2602_08798_amd.microbench ntt      forward/inverse transform throughput vs number of rows
    python -m paper_2602_08798_amd.microbench copy     plain device copy of known size (counter calibration)

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


if __name__ == "__main__":
    what = sys.argv[1] if len(sys.argv) > 1 else "modmul"
    {"modmul": modmul, "ntt": ntt, "copy": copy}[what]()
