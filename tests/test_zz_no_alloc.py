"""The allocation-free entry point (cg_mul_relin_static, for callers that cannot call hipMalloc)
against cg_mul_relin on the same inputs: bit-identical outputs on two calls in a row, the second
with a smaller batch, so that whatever the first call left in the library's static scratch array
is shown not to matter."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from workloads import PRESETS, Stream, pseudo_ciphertexts, pseudo_switch_key


def say(msg):
    print(f"[gpu-no-alloc] {msg}", flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("name,first,second", [("C2", 9, 4), ("C1", 28, 5)])
def test_static_scratch_entry_point_matches_the_workspace_one(name, first, second):
    import torch
    import paper_2602_08798_amd as P
    from paper_2602_08798_amd.binding import CgError
    prm = PRESETS[name]
    ctx = P.Context(prm)
    lib = ctx.lib.dll
    limit = int(lib.cg_static_scratch_bytes())
    assert limit == 64 << 20
    assert ctx.workspace_bytes(first) <= limit < ctx.workspace_bytes(first + 1)
    qp = list(prm.q) + list(prm.p)
    rlk = ctx.ksk_prepare(P.to_device(pseudo_switch_key(Stream(71, 2), qp, prm.n, prm.dnum)))
    for call, batch in enumerate((first, second)):
        say(f"{name} call {call}: batch {batch}")
        a = P.to_device(pseudo_ciphertexts(Stream(71, 10 + call), prm.q, prm.n, batch))
        b = P.to_device(pseudo_ciphertexts(Stream(71, 20 + call), prm.q, prm.n, batch))
        want = ctx.mul_relin(a, b, rlk, batch)
        out = ctx.empty_ct(batch)
        out.fill_(-1)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        ctx.mul_relin_static(a, b, rlk, batch, out=out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert np.array_equal(P.to_host(out), P.to_host(want)), f"{name} call {call}: outputs differ"
    # one product more than the array holds: refused before anything is launched
    big = first + 1
    a = P.to_device(pseudo_ciphertexts(Stream(71, 30), prm.q, prm.n, big))
    out = ctx.empty_ct(big)
    out.fill_(-1)
    with pytest.raises(CgError, match="static"):
        ctx.mul_relin_static(a, a, rlk, big, out=out)
    torch.cuda.synchronize()
    assert bool((out == -1).all())
    ctx.close()
