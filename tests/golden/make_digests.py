"""Writes tests/golden/digests_<config>.json: SHA-256 of every output ciphertext of the five
benchmark configurations as computed by the CPU oracle (and by nothing else).

    python -m tests.golden.make_digests C1 C2 C4 C4H C4HS    (about a minute)
    python -m tests.golden.make_digests C3              (all 12 heads: tens of minutes)
    python -m tests.golden.make_digests C5              (all 64 steps: about 40 minutes on 8 cores)
    python -m tests.golden.make_digests C5H             (16 steps in the hoisted form: about 13 minutes)
    python -m tests.golden.make_digests C3H             (all heads in the hoisted forms: about 7 minutes)

The GPU tests recompute the same units with the HIP library from the same seeded inputs
(workloads.configs) and compare digests, i.e. every residue of every output, bit for bit.
"""
import hashlib
import json
import os
import sys
import time

import numpy as np

from oracle import Oracle, run_configs
from workloads import configs

HERE = os.path.dirname(os.path.abspath(__file__))
C5_STEPS = 64
C5H_STEPS = 16         # the scaled configuration in its hoisted form: the first steps only
C3H_HEADS = tuple(range(12))   # the prompt configuration in its hoisted forms: all heads


def digest(arr) -> str:
    return hashlib.sha256(np.ascontiguousarray(arr, dtype="<u8").tobytes()).hexdigest()


def main(names):
    for name in names:
        t0 = time.time()
        if name == "C1":
            inp = configs.c1_inputs(); out = run_configs.run_c1(Oracle(inp["prm"]), inp); note = "16 mult+relin pairs"
        elif name == "C2":
            inp = configs.c2_inputs(); out = run_configs.run_c2(Oracle(inp["prm"]), inp); note = "decode scores, 1 head x 1 ciphertext"
        elif name == "C4":
            inp = configs.c4_inputs(); out = run_configs.run_c4(Oracle(inp["prm"]), inp); note = "full decode step, 12 heads, 512-token cache"
        elif name in ("C4H", "C4HS"):
            from oracle import attention
            inp = configs.c4_inputs()
            wf, wb = configs.C4_ROUND_BITS
            keys = configs.galois_keys("C4", attention.hoisted_fold_galois(inp["prm"].n, inp["d2"], wf, wb))
            out = run_configs.run_c4_hoisted(Oracle(inp["prm"]), inp, wf, wb, keys, sum_first=name == "C4HS")
            note = f"full decode step, 12 heads, 512-token cache, folding sums in rounds of {wf} / {wb} bits (hoisted rotation sums)"
            if name == "C4HS":
                note += ", the context's products over the cache ciphertexts summed before the one scaling"
        elif name == "C3":
            inp = configs.c3_inputs()
            out = run_configs.run_c3(Oracle(inp["prm"]), inp, progress=lambda m: print(m, f"{time.time() - t0:.0f}s", flush=True))
            note = "prefill: 3072 appends, 12 x 128 generalised diagonals of Q K^T, their compaction (12 x 2), A V (12)"
        elif name == "C5":
            inp = configs.c5_inputs(); out = run_configs.run_c5(Oracle(inp["prm"]), inp, C5_STEPS)
            note = f"{C5_STEPS} successive decode steps with cache growth, 16 heads, N = 16384"
        elif name == "C3H":
            from oracle import attention
            inp = configs.c3_inputs()
            n, d2 = inp["prm"].n, inp["d2"]
            wf = configs.C4_ROUND_BITS[0]
            gals = sorted(set(attention.copy_galois(n, d2)[1:]) | set(attention.hoisted_fold_galois(n, d2, wf, 1)))
            keys = configs.galois_keys("C3", gals)
            out = run_configs.run_c3_hoisted(Oracle(inp["prm"]), inp, C3H_HEADS, keys, wf, configs.C4_SUM_BEFORE_SCALING)
            note = (f"prefill of head(s) {list(C3H_HEADS)} in the hoisted forms: 128 generalised diagonals of Q K^T with hoisted "
                    f"copies of K and folding sums in rounds of {wf} bits, A V with hoisted copies of V and its products "
                    f"summed before one scaling")
        elif name == "C5H":
            from oracle import attention
            inp = configs.c5_inputs()
            wf, wb = configs.C4_ROUND_BITS
            keys = configs.galois_keys("C5", attention.hoisted_fold_galois(inp["prm"].n, inp["d2"], wf, wb))
            out = run_configs.run_c5(Oracle(inp["prm"]), inp, C5H_STEPS, rounds=(wf, wb, keys, configs.C4_SUM_BEFORE_SCALING))
            note = (f"{C5H_STEPS} successive decode steps with cache growth, 16 heads, N = 16384, folding sums in rounds of "
                    f"{wf} / {wb} bits, the context's products summed before one scaling")
        else:
            raise SystemExit(f"unknown configuration {name}")
        doc = {"config": name, "what": note, "source": "oracle/ only (tests/golden/make_digests.py)",
               "hash": "sha256 of the little-endian uint64 residues of each output ciphertext",
               "digests": {k: digest(v) for k, v in out.items()}}
        path = os.path.join(HERE, f"digests_{name}.json")
        with open(path, "w") as f:
            json.dump(doc, f, indent=0, sort_keys=True)
        print(f"{name}: {len(out)} outputs, {time.time() - t0:.1f} s -> {path}", flush=True)


if __name__ == "__main__":
    main(sys.argv[1:] or ["C1", "C2", "C4", "C4H", "C4HS"])
