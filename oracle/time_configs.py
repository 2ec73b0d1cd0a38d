"""Wall-clock of the CPU oracle on the benchmark configurations (reported baseline, not a target).

    python -m oracle.time_configs            C1, C2 and C4 in full; one head of C3; one step of C5

Every configuration is timed with one thread and with all threads the machine gives the process
(the oracle parallelises inside each operation with OpenMP).  C3 and C5 figures are for the stated
subset and are scaled linearly to the whole configuration in a second column, labelled as such.
"""
import os
import sys
import time

from . import Oracle, run_configs
from workloads import configs


def _timed(fn):
    t0 = time.perf_counter()
    fn()
    return time.perf_counter() - t0


def cases():
    def c1():
        inp = configs.c1_inputs()
        return Oracle(inp["prm"]), lambda orc: run_configs.run_c1(orc, inp), 1.0, "16 mult+relin pairs, N = 4096"

    def c2():
        st = configs.c2_inputs()
        return Oracle(st["prm"]), lambda orc: run_configs.run_c2(orc, st), 1.0, "decode scores, 1 head x 1 ciphertext"

    def c4():
        st = configs.c4_inputs()
        return Oracle(st["prm"]), lambda orc: run_configs.run_c4(orc, st), 1.0, "decode step, 12 heads, 512 tokens (one layer)"

    def c3():
        st = configs.c3_inputs()
        return (Oracle(st["prm"]), lambda orc: run_configs.run_c3(orc, st, heads=[0]), float(st["heads"]),
                "prefill, 1 of 12 heads (appends, Q K^T, compaction, A V)")

    def c5():
        st = configs.c5_inputs()
        return (Oracle(st["prm"]), lambda orc: run_configs.run_c5(orc, st, 1), 64.0,
                "scaled decode, 1 of 64 steps, 16 heads, N = 16384")

    return [("C1", c1), ("C2", c2), ("C4", c4), ("C3", c3), ("C5", c5)]


def main(argv):
    names = set(argv) if argv else None
    print(f"{'config':6s} {'threads':>7s} {'seconds':>10s} {'whole config (scaled)':>22s}  what", flush=True)
    for name, make in cases():
        if names and name not in names:
            continue
        orc, run, scale, what = make()
        all_threads = orc.threads
        for nt in (all_threads, 1):
            if nt == 1 and name in ("C3", "C5") and "--single-all" not in argv:
                # one thread on the long subsets takes many minutes; timed on request only
                continue
            orc.set_threads(nt)
            dt = _timed(lambda: run(orc))
            print(f"{name:6s} {nt:7d} {dt:10.2f} {dt * scale:22.1f}  {what}", flush=True)
        orc.set_threads(all_threads)


if __name__ == "__main__":
    main([a for a in sys.argv[1:]])
