"""The oracle still computes what it computed when tests/golden/c1_oracle_digest.json was written
(by tests/golden/make_golden.py, which calls only the oracle)."""
import importlib.util
import json
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_digest_of_the_tiny_configuration():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    want = json.load(open(os.path.join(HERE, "golden", "c1_oracle_digest.json")))
    got = mod.digests()
    assert got == want
    # the histogram is that of a static 4-bit grid with absmax calibration: every code in range, zero the mode
    for name, d in got.items():
        h = d["q_histogram"]
        assert sum(h) == 128 * 512 and h[8] == max(h)
