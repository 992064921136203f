"""The stored tiny-config trajectories (written by tests/golden/make_golden.py from the oracle alone) still
match what the oracle computes: guards the oracle and the input generators against silent drift."""
import importlib.util
import json
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def load_generator():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_oracle_reproduces_stored_tiny_trajectory():
    got = load_generator().compute()
    with open(os.path.join(HERE, "golden", "tiny_fp32_seed0.json")) as f:
        want = json.load(f)
    for key in ("first_tokens", "tokens", "exit_layer", "batch_exit_layer"):
        assert got[key] == want[key], key
    # the trajectory exercises the method: early batch exits happen and deeper ones follow
    assert min(want["batch_exit_layer"]) < 4 and len(set(want["batch_exit_layer"])) > 1


def test_oracle_reproduces_stored_untied_trajectory_with_varying_tokens():
    got = load_generator().compute("tiny_fp32_untied_seed4")
    with open(os.path.join(HERE, "golden", "tiny_fp32_untied_seed4.json")) as f:
        want = json.load(f)
    for key in ("first_tokens", "tokens", "exit_layer", "batch_exit_layer"):
        assert got[key] == want[key], key
    # this one exercises the token path: every sequence emits a different token at every step, the batch leaves
    # at layers 2, 3 and 4, and no decision is close
    steps = len(want["tokens"])
    for b in range(len(want["first_tokens"])):
        assert len({t[b] for t in want["tokens"]}) == steps
    assert set(want["batch_exit_layer"]) == {2, 3, 4}
    assert min(want["min_margin"]) > 1e-3
