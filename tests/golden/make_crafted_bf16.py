"""Finds and stores crafted decode iterations in which the PLACE of one bf16 rounding decides a discrete result.

    python tests/golden/make_crafted_bf16.py          (rewrites tests/golden/crafted_bf16_rounding.json)
    python tests/golden/make_crafted_bf16.py "<mistake>" ...   (searches the named cases again, keeps the others)

Calls only the oracle (and the input generators' config record).  For every planted rounding mistake of
tests/oracle_mutants.py the script searches a family of small block-constant models for one decode iteration where

  * the oracle with the mistake planted ends in a different discrete result than the oracle as it stands: a
    different bf16 value cached for this position in some layer, or a different token; and
  * every value the oracle rounds to bf16 on the way sits at least MARGIN of a bf16 step away from a rounding
    boundary, and the token's logit leads the runner-up by TOKEN_GAP of the largest logit, so that an
    implementation which rounds at the SAME places in float32 arithmetic must reproduce the stored result bit
    for bit, while one that rounds elsewhere gets the other result.

A model of the family is block-constant: the channels of the hidden state fall into groups, every matrix is constant
on (output group x input group) blocks, every vector constant on groups, all values small multiples of 1/16 (exact
in bf16).  The whole iteration then runs on a handful of distinct numbers, few enough for all of them to keep their
distance from the rounding boundaries at once.  Rotary embedding is switched off (it would break the block
structure; the rotation has pins of its own).
"""
import json
import os
import sys

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(HERE))

from oracle import ee_oracle as O          # noqa: E402
from oracle_mutants import MUTANTS, planted   # noqa: E402
from paper_2407_20272_amd import workloads as W   # noqa: E402

F64 = torch.float64
BF = torch.bfloat16
MARGIN = 0.06          # of one bf16 step (2^-8 .. 2^-7 relative): float32 noise is about a thousand times smaller
TOKEN_GAP = 2e-3
OUT = os.path.join(HERE, "crafted_bf16_rounding.json")

D, H, DH, FF, V, NL, CTX = 128, 2, 64, 64, 64, 2, 3      # channels per group: 64 (= one head); FFN groups of 32
GD, GF = 2, 2


def crafted_config(mode):
    """mode "full": no sequence ever exits (threshold 2), the result is read from the K/V the layers cache and the
    token.  mode "exit": everybody exits after layer 1 (threshold 0), the result is the FILLED K/V of layer 2 and the
    token from the exit head's hidden state."""
    return W.reduced(W.CONFIGS[1], n_layers=NL, d_model=D, n_heads=H, head_dim=DH, d_ffn=FF, vocab=V, batch=1,
                     prompt_len=CTX, min_prompt_len=CTX, decode_steps=1, rope_theta=0.0, exit_every=1,
                     logit_scale=1.0, threshold=2.0 if mode == "full" else 0.0)


def draw_params(g):
    """Random block values, multiples of 1/16 (1/64 for the wide contractions, so sums stay moderate)."""
    def blk(rows, cols, lo, hi, unit):
        return (torch.randint(lo, hi + 1, (rows, cols), generator=g).to(F64) * unit).tolist()
    # LM head: the second half of the vocabulary repeats the first with one block moved by 1/256, so that close pairs
    # of logits exist (a rounding of the logits can then change which of two tokens wins)
    lm = torch.randint(-32, 33, (V // 2, GD), generator=g)
    nudge = torch.zeros(V // 2, GD, dtype=torch.long)
    nudge[torch.arange(V // 2), torch.randint(0, GD, (V // 2,), generator=g)] = torch.randint(0, 2, (V // 2,), generator=g) * 2 - 1
    p = {"embed": blk(1, GD, -24, 24, 1 / 8)[0], "g_final": blk(1, GD, 8, 24, 1 / 16)[0],
         "w_lm": (torch.cat([lm, lm + nudge]).to(F64) / 256).tolist(), "layers": [],
         "K": [blk(CTX, H, -16, 16, 1 / 8) for _ in range(NL)], "V": [blk(CTX, H, -16, 16, 1 / 8) for _ in range(NL)]}
    for _ in range(NL):
        p["layers"].append({"g_attn": blk(1, GD, 8, 24, 1 / 16)[0], "g_ffn": blk(1, GD, 8, 24, 1 / 16)[0],
                            "w_q": blk(GD, GD, -8, 8, 1 / 256), "w_k": blk(GD, GD, -8, 8, 1 / 256),
                            "w_v": blk(GD, GD, -16, 16, 1 / 256), "w_o": blk(GD, GD, -16, 16, 1 / 128),
                            "w_gate": blk(GF, GD, -16, 16, 1 / 256), "w_up": blk(GF, GD, -16, 16, 1 / 256),
                            "w_down": blk(GD, GF, -16, 16, 1 / 64)})
    return p


def expand(block, rows_per, cols_per):
    t = torch.tensor(block, dtype=F64)
    if t.dim() == 1:
        return t.repeat_interleave(cols_per).to(BF)
    return t.repeat_interleave(rows_per, 0).repeat_interleave(cols_per, 1).to(BF)


def build(p):
    """Weights (the dict layout of workloads.make_weights), dense cache contents [1][CTX][H][dh] per layer, token."""
    cd, cf = D // GD, FF // GF
    w = {"embed": expand([p["embed"]] * V, 1, cd), "g_final": expand(p["g_final"], 1, cd), "w_lm": expand(p["w_lm"], 1, cd),
         "layers": []}
    for lp in p["layers"]:
        w["layers"].append({"g_attn": expand(lp["g_attn"], 1, cd), "g_ffn": expand(lp["g_ffn"], 1, cd),
                            "w_q": expand(lp["w_q"], cd, cd), "w_k": expand(lp["w_k"], cd, cd), "w_v": expand(lp["w_v"], cd, cd),
                            "w_o": expand(lp["w_o"], cd, cd), "w_gate": expand(lp["w_gate"], cf, cd),
                            "w_up": expand(lp["w_up"], cf, cd), "w_down": expand(lp["w_down"], cd, cf)})
    Ks = [torch.tensor(k, dtype=F64)[None, :, :, None].expand(1, CTX, H, DH).to(BF).contiguous() for k in p["K"]]
    Vs = [torch.tensor(v, dtype=F64)[None, :, :, None].expand(1, CTX, H, DH).to(BF).contiguous() for v in p["V"]]
    return w, Ks, Vs


class MarginLog:
    """Replaces the oracle's store(): same result, and the smallest distance of a rounded value from a bf16
    rounding boundary (in bf16 steps; 0.5 = the value is a bf16 number already) is kept."""

    def __init__(self):
        self.min_margin = 0.5
        self.real = O.store

    def __call__(self, x, dtype):
        out = self.real(x, dtype)
        if dtype == "bf16" and x.numel():
            xf = x.to(torch.float32).to(F64)
            nz = xf.abs() > 1e-30
            if bool(nz.any()):
                step = torch.exp2(torch.floor(torch.log2(xf[nz].abs())) - 7)
                self.min_margin = min(self.min_margin, float((0.5 - (xf[nz] - out[nz]).abs() / step).min()))
        return out


def run(p, mode, log_margins=False):
    """One decode iteration of the oracle; returns (result, min margin, token gap).  The result holds, for the new
    position, the K and V bf16 values of every layer (one number per head: they are constant over a head's channels,
    the full rows are compared in the tests), the token, the exit layer and the batch exit layer."""
    cfg = crafted_config(mode)
    w, Ks, Vs = build(p)
    m = O.model_from_config(cfg, w)
    lens = torch.tensor([CTX], dtype=torch.int32)
    pad = [torch.zeros(1, 1, H, DH, dtype=BF)]
    cache = O.DenseKV.from_tensors([torch.cat([k] + pad, 1) for k in Ks], [torch.cat([v] + pad, 1) for v in Vs], lens, "bf16")
    log = MarginLog()
    if log_margins:
        O.store = log
    try:
        tr = {}
        tok, e, L = O.decode_iteration(m, cache, torch.zeros(1, dtype=torch.int32), lens.long(), cfg.threshold, trace=tr)
    finally:
        O.store = log.real
    z = O.head_logits(m, tr["h_exit"])[0]
    top = torch.topk(z, 2).values
    gap = float((top[0] - top[1]) / z.abs().max())
    for i in range(NL):          # block-constant model: one value per head
        assert bool((cache.K[i][0, CTX] == cache.K[i][0, CTX, :, :1]).all()) and bool((cache.V[i][0, CTX] == cache.V[i][0, CTX, :, :1]).all())
    res = {"K": [cache.K[i][0, CTX, :, 0].to(F64).tolist() for i in range(NL)],
           "V": [cache.V[i][0, CTX, :, 0].to(F64).tolist() for i in range(NL)],
           "token": int(tok[0]), "exit_layer": int(e[0]), "batch_exit_layer": int(L)}
    return res, log.min_margin, gap


def finite(res):
    return all(abs(x) < 1e4 for kv in (res["K"], res["V"]) for row in kv for x in row)


def search(name, mode, seed, budget=30000):
    g = torch.Generator().manual_seed(seed)
    for trial in range(budget):
        p = draw_params(g)
        good, margin, gap = run(p, mode, log_margins=True)
        if margin < MARGIN or gap < TOKEN_GAP or not finite(good):
            continue
        with planted(name):
            bad, _, _ = run(p, mode)
        if bad == good:
            continue
        return {"mistake": name, "mode": mode, "params": p, "result": good, "result_with_mistake": bad,
                "min_margin": margin, "token_gap": gap, "trials": trial + 1}
    return None


def mode_of(name):
    return "exit" if MUTANTS[name][0] in ("head_logits", "kv_fill") else "full"


def main():
    only = sys.argv[1:]
    doc = {"cases": []}
    if only and os.path.exists(OUT):
        with open(OUT) as f:
            doc = json.load(f)
    have = {c["mistake"]: c for c in doc["cases"]}
    for k, name in enumerate(sorted(MUTANTS)):
        if name == "filled K rounded before the rotation":
            continue          # needs the rotary embedding, which the block-constant family switches off
        if only and name not in only:
            continue
        c = search(name, mode_of(name), seed=1000 + k)
        if c is None:
            # not every misplaced rounding can decide a discrete result within this small family; such a mistake is
            # still caught on the CPU by the brute-force pin of the storage points
            print(f"{name}: no case within the search budget", flush=True)
            have.pop(name, None)
            continue
        print(f"{name}: found after {c['trials']} trials, margin {c['min_margin']:.3f}, token gap {c['token_gap']:.2e}",
              flush=True)
        have[name] = c
    head = {"what": "crafted decode iterations whose discrete result depends on where one bf16 rounding is placed; "
                    "written by tests/golden/make_crafted_bf16.py from the oracle alone",
            "shape": {"d_model": D, "n_heads": H, "head_dim": DH, "d_ffn": FF, "vocab": V, "n_layers": NL, "context": CTX},
            "margin": MARGIN, "token_gap": TOKEN_GAP}
    with open(OUT, "w") as f:          # one case per line
        f.write(json.dumps(head)[:-1] + ', "cases": [\n')
        f.write(",\n".join(json.dumps(have[k]) for k in sorted(have)))
        f.write("\n]}\n")
    print("wrote", OUT)


if __name__ == "__main__":
    main()
