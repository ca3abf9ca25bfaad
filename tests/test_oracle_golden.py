"""Regression pin of the oracle + input generators against digests written by
tests/golden/make_golden.py (oracle only; see tests/golden/README.md).

Index metadata (integer PRNG only) must match exactly.  Value digests depend on the
host's libm (Box-Muller uses log/cos), so values are compared through their sums."""
import importlib.util
import os
import re

HERE = os.path.dirname(os.path.abspath(__file__))


def _parse(line):
    return dict(re.findall(r"(\w+)=(\S+)", line)), line.split()[0:2]


def test_oracle_digests_unchanged():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = open(os.path.join(HERE, "golden", "oracle_digests.txt")).read().splitlines()
    fresh = mod.entries()
    assert len(fresh) == len(stored)
    for a, b in zip(fresh, stored):
        fa, ha = _parse(a)
        fb, hb = _parse(b)
        assert ha == hb
        if "kpos" in fa:      # packing metadata: bit-exact
            assert (fa["grp"], fa["kpos"], fa["K"]) == (fb["grp"], fb["kpos"], fb["K"]), a
        else:                 # outputs: sums within 1e-6 relative of the absolute sum
            scale = float(fb["abssum"])
            assert abs(float(fa["sum"]) - float(fb["sum"])) <= 1e-6 * scale, a
            assert abs(float(fa["abssum"]) - scale) <= 1e-6 * scale, a
