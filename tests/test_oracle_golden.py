"""The oracles still produce the values stored in tests/golden/c1_oracle_values.txt (written by
tests/golden/make_golden.py from oracle/ alone): a change to an oracle's arithmetic has to show up as a diff of
that file, with its justification."""
import importlib.util
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def _load_maker():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_oracles_reproduce_the_stored_values():
    stored = {}
    with open(os.path.join(HERE, "golden", "c1_oracle_values.txt")) as f:
        for line in f:
            if line.startswith("#") or "=" not in line:
                continue
            name, val = line.split("=", 1)
            stored[name.strip()] = float(val)
    now = _load_maker().values()
    assert set(now) == set(stored)
    for name, val in now.items():
        assert abs(val - stored[name]) <= 1e-12 * max(1.0, abs(stored[name])), (name, val, stored[name])
