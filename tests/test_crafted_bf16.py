"""Crafted decode iterations in which the PLACE of one bf16 rounding decides a discrete result (a cached bf16 value
or the token).  The cases and their expected results are stored in tests/golden/crafted_bf16_rounding.json, written
by tests/golden/make_crafted_bf16.py from the oracle alone.  On the CPU: the oracle reproduces every stored result,
every value it rounds on the way keeps the stated distance from a rounding boundary (so float32 arithmetic that
rounds at the same places must land on the same bf16 values), and the oracle with the named mistake planted ends in
the other stored result.  On the GPU (-m gpu): the HIP path reproduces the stored results bit for bit, so a kernel
that rounds anywhere else than the numerics contract says fails one of these."""
import json
import os
import sys

import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "golden"))

import make_crafted_bf16 as M   # noqa: E402
from oracle_mutants import planted   # noqa: E402

with open(M.OUT) as _f:
    DOC = json.load(_f)
CASES = {c["mistake"]: c for c in DOC["cases"]}


def test_the_stored_cases_cover_the_contract():
    assert DOC["shape"] == {"d_model": M.D, "n_heads": M.H, "head_dim": M.DH, "d_ffn": M.FF, "vocab": M.V,
                            "n_layers": M.NL, "context": M.CTX}
    for must in ("attention output not rounded", "SwiGLU product not rounded", "FFN-norm operand not rounded",
                 "residual stream rounded after the FFN", "residual stream rounded after attention",
                 "FFN-norm row factor applied after the rounding", "attention-norm row factor applied after the rounding",
                 "exit-head logits rounded", "filling operand not rounded", "q rounded"):
        assert must in CASES, must


@pytest.mark.parametrize("name", sorted(CASES))
def test_oracle_reproduces_the_stored_result_and_the_planted_mistake_changes_it(name):
    c = CASES[name]
    good, margin, gap = M.run(c["params"], c["mode"], log_margins=True)
    assert good == c["result"]
    assert margin >= DOC["margin"] and gap >= DOC["token_gap"], (margin, gap)
    with planted(name):
        bad, _, _ = M.run(c["params"], c["mode"])
    assert bad == c["result_with_mistake"] and bad != good


@pytest.mark.gpu
@pytest.mark.parametrize("name", sorted(CASES))
def test_hip_path_reproduces_the_stored_result_bit_for_bit(name):
    from gpu_harness import HipRun
    c = CASES[name]
    cfg = M.crafted_config(c["mode"])
    w, Ks, Vs = M.build(c["params"])
    lens = torch.tensor([M.CTX], dtype=torch.int32)
    run = HipRun(cfg, w, lens, 1, seed=0, pool_fill=7.0)
    run.load_dense(Ks, Vs)
    tok, e, L, _, _ = run.step(torch.zeros(1, dtype=torch.int32), lens.long(), cfg.threshold)
    want = c["result"]
    assert (int(tok[0]), int(e[0]), L) == (want["token"], want["exit_layer"], want["batch_exit_layer"])
    for i in range(M.NL):
        k, v = run.kv_at(i + 1, 0, M.CTX)                       # [H][dh] bf16 of the new position
        for h in range(M.H):
            assert bool((k[h].double() == want["K"][i][h]).all()), f"K of layer {i + 1}, head {h}: {float(k[h, 0])} vs {want['K'][i][h]}"
            assert bool((v[h].double() == want["V"][i][h]).all()), f"V of layer {i + 1}, head {h}: {float(v[h, 0])} vs {want['V'][i][h]}"
