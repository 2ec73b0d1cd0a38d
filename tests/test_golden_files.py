"""The stored digests are reproducible from the oracle (checked on the two small configurations)
and complete for all five."""
import json
import os

from oracle import Oracle, run_configs
from workloads import configs

from .golden.make_digests import digest

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _load(name):
    return json.load(open(os.path.join(GOLDEN, f"digests_{name}.json")))


def test_digest_files_cover_every_output_unit():
    assert len(_load("C1")["digests"]) == 16
    assert len(_load("C2")["digests"]) == 1
    assert len(_load("C4")["digests"]) == 48 + 12 + 24
    assert len(_load("C4H")["digests"]) == 48 + 12 + 24
    assert _load("C4H")["digests"] != _load("C4")["digests"]          # other ciphertexts, same append
    assert all(_load("C4H")["digests"][f"cache{c}"] == _load("C4")["digests"][f"cache{c}"] for c in range(24))
    # summing the context's products before the scaling changes the contexts and nothing else
    h, hs = _load("C4H")["digests"], _load("C4HS")["digests"]
    assert set(h) == set(hs) and all((h[k] != hs[k]) == k.startswith("context") for k in h)
    assert len(_load("C3")["digests"]) == 24 + 12 * (128 + 2 + 1)
    assert len(_load("C5")["digests"]) == 64 * (32 + 16 * 3 + 16)     # all 64 steps
    assert len(_load("C5H")["digests"]) == 16 * (32 + 16 * 3 + 16)
    assert len(_load("C3H")["digests"]) == 12 * (128 + 1)
    for name in ("C1", "C2", "C3", "C3H", "C4", "C4H", "C4HS", "C5", "C5H"):
        assert _load(name)["source"].startswith("oracle/ only")


def test_small_configurations_reproduce_their_digests():
    inp = configs.c1_inputs()
    out = run_configs.run_c1(Oracle(inp["prm"]), inp)
    assert {k: digest(v) for k, v in out.items()} == _load("C1")["digests"]
    st = configs.c2_inputs()
    out = run_configs.run_c2(Oracle(st["prm"]), st)
    assert {k: digest(v) for k, v in out.items()} == _load("C2")["digests"]
