"""The C-ABI library loads on a machine without a GPU and exports every symbol the headers declare."""
import os
import re

from paper_2602_08798_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported_and_bound():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    declared = sorted(set(re.findall(r"\b(cg_[a-z0-9_]+)\s*\(", text)))
    assert declared, "no declarations found"
    lib = binding.load_library()
    for name in declared:
        assert hasattr(lib.dll, name), f"{name} declared in the header but not exported"
    assert sorted(binding.exported_symbols()) == declared
    assert lib.strerror(0) == "ok" and "invalid" in lib.strerror(-1)


def test_host_arithmetic_header_against_128_bit_integers(tmp_path):
    """The device arithmetic is IEEE double + explicit fma; the same header runs on the host."""
    import subprocess
    exe = tmp_path / "modarith_check"
    src = os.path.join(ROOT, "tests", "host", "modarith_check.cpp")
    subprocess.run(["g++", "-O2", "-ffp-contract=off", "-march=native", "-o", str(exe), src], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr
