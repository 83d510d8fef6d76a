"""CPU-only regression: the oracle and the input recipe still give the values
frozen in tests/golden/oracle_c1_samples.txt (written by make_golden.py from
the oracle alone; the paper itself prints no numbers to compare with)."""
import importlib.util
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_matches_frozen_samples():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = {(n, i): v for n, i, v in mod.compute()}
    seen = 0
    for line in open(os.path.join(HERE, "golden", "oracle_c1_samples.txt")):
        if line.startswith("#"):
            continue
        name, idx, val = line.split()
        ref = float(val)
        got = now[(name, int(idx))]
        assert abs(got - ref) <= 1e-12 * max(1.0, abs(ref)), (name, idx, got, ref)
        seen += 1
    assert seen >= 80
