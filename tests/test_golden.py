"""The stored tiny-config trajectory (written by tests/golden/make_golden.py from the oracle alone) still
matches what the oracle computes: guards the oracle and the input generators against silent drift."""
import importlib.util
import json
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_reproduces_stored_tiny_trajectory():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    got = mod.compute()
    with open(os.path.join(HERE, "golden", "tiny_fp32_seed0.json")) as f:
        want = json.load(f)
    for key in ("first_tokens", "tokens", "exit_layer", "batch_exit_layer"):
        assert got[key] == want[key], key
    # the trajectory exercises the method: early batch exits happen and deeper ones follow
    assert min(want["batch_exit_layer"]) < 4 and len(set(want["batch_exit_layer"])) > 1
