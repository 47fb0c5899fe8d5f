"""The oracle still produces the stored digests (written by tests/golden/make_golden.py, which
calls only the oracle and the seeded generators)."""
import importlib.util
import json
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_digests_unchanged():
    spec = importlib.util.spec_from_file_location("make_golden",
                                                  os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(HERE, "golden", "oracle_digests.json")) as f:
        stored = json.load(f)
    assert mod.digests() == stored
