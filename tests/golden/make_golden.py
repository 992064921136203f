"""Writes tests/golden/tiny_fp32_seed0.json: tokens, exit layers and batch exit layers of the tiny fp32
workload (benchmark config 0, seed 0) as the CPU oracle computes them.  Calls only oracle/ and the input
generators.  The paper prints no worked example for this path, so these are regression values of the
pinned oracle, not published ones.     usage: python tests/golden/make_golden.py"""
import json
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import ee_oracle as O                      # noqa: E402
from paper_2407_20272_amd import workloads as W        # noqa: E402


def compute():
    cfg = W.CONFIGS[0]
    w = W.make_weights(cfg, seed=0)
    m = O.model_from_config(cfg, w)
    prompts, lens = W.make_prompts(cfg, seed=0), W.make_context_lens(cfg, seed=0)
    cache = O.DenseKV(cfg.n_layers, cfg.batch, cfg.prompt_len + cfg.decode_steps, cfg.n_heads, cfg.head_dim, cfg.dtype)
    tok = O.prefill(m, cache, prompts, lens)
    pos = lens.clone().long()
    out = {"first_tokens": tok.tolist(), "tokens": [], "exit_layer": [], "batch_exit_layer": [], "min_margin": []}
    for _ in range(cfg.decode_steps):
        tr = {}
        tok, e, L = O.decode_iteration(m, cache, tok, pos, cfg.threshold, trace=tr)
        conf = tr["conf"]
        margin = (conf[~conf.isnan()] - cfg.threshold).abs().min().item() if (~conf.isnan()).any() else None
        out["tokens"].append(tok.tolist())
        out["exit_layer"].append(e.tolist())
        out["batch_exit_layer"].append(L)
        out["min_margin"].append(margin)        # distance of the closest confidence to the threshold
        pos += 1
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_fp32_seed0.json")
    with open(path, "w") as f:
        json.dump(compute(), f, indent=1)
    print("wrote", path)
