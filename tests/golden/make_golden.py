"""Writes tests/golden/tiny_fp32_seed0.json and tiny_fp32_untied_seed4.json: tokens, exit layers and batch exit
layers of the tiny fp32 workload as the CPU oracle computes them.  The first is benchmark config 0 as defined
(seed 0, tied head: with weights of N(0, 0.02) every sequence repeats one token, so its value lies in the exit
layers); the second unties the head and widens the weights so that every decode step emits a different token and
the batch exit layer moves between 2 and 4, with every confidence at least 1.9e-3 from the threshold and every
winning logit 2.5e-3 of the largest ahead of the runner-up.  Calls only oracle/ and the input generators.  The
paper prints no worked example for this path, so these are regression values of the pinned oracle, not published
ones.     usage: python tests/golden/make_golden.py"""
import json
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import ee_oracle as O                      # noqa: E402
from paper_2407_20272_amd import workloads as W        # noqa: E402


def case(name):
    """(config, seed) of a stored trajectory."""
    if name == "tiny_fp32_seed0":
        return W.CONFIGS[0], 0
    if name == "tiny_fp32_untied_seed4":
        return W.CONFIGS[0].with_(tied_head=False, weight_std=0.08, logit_scale=2.0, threshold=0.5), 4
    raise KeyError(name)


CASES = ("tiny_fp32_seed0", "tiny_fp32_untied_seed4")


def compute(name="tiny_fp32_seed0"):
    cfg, seed = case(name)
    w = W.make_weights(cfg, seed=seed)
    m = O.model_from_config(cfg, w)
    prompts, lens = W.make_prompts(cfg, seed=seed), W.make_context_lens(cfg, seed=seed)
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
    for name in CASES:
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), name + ".json")
        with open(path, "w") as f:
            json.dump(compute(name), f, indent=1)
        print("wrote", path)
