"""Iteration-level scheduling around the decode step: a host-side harness, not part of the decode path.

The paper (Section 3, iteration-level scheduling as in Orca / vLLM) runs one iteration at a time over the
sequences that are currently active: finished sequences leave after an iteration and waiting requests take
their place.  This module does that around `ee_decode_iteration`:

  * prompts are pushed through the decode step WITHOUT exit checks, several positions per call: a prompt
    chunk is a set of batch rows that share one block table (`ee_batch.row_table`), which is causal because
    every row caches its K/V before any row attends;
  * decode iterations run over the active sequences with the chosen exit rule;
  * a finished request frees its blocks and a waiting one is admitted (evict / replenish);
  * every token gets a timestamp, from which the paper's inner-token latency (sum over sequences of finish time minus
    first-token time, over all generated tokens) and the time between consecutive tokens of one request follow.

Only orchestration and argument marshalling happen here; every step of the path runs in the HIP library.

    python -m paper_2407_20272_amd.serving --config 1 --requests 96 --max-batch 32
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import sys
import time
from typing import Dict, List, Optional

import torch

from . import binding as B
from . import workloads as W


class BlockAllocator:
    """Free list over the physical KV blocks."""

    def __init__(self, num_blocks: int):
        self.free = list(range(num_blocks - 1, -1, -1))

    def take(self, n: int) -> Optional[List[int]]:
        if n > len(self.free):
            return None
        out = [self.free.pop() for _ in range(n)]
        return out

    def give(self, blocks: List[int]):
        self.free.extend(reversed(blocks))


@dataclasses.dataclass
class Request:
    rid: int
    prompt: List[int]
    max_new_tokens: int
    blocks: List[int] = dataclasses.field(default_factory=list)
    consumed: int = 0                       # prompt positions already cached
    generated: List[int] = dataclasses.field(default_factory=list)
    exit_layers: List[int] = dataclasses.field(default_factory=list)
    token_times: List[float] = dataclasses.field(default_factory=list)
    arrived: float = 0.0

    @property
    def context_len(self) -> int:           # positions cached so far
        return self.consumed + max(len(self.generated) - 1, 0)

    @property
    def done(self) -> bool:
        return len(self.generated) >= self.max_new_tokens


class Engine:
    """One model, one paged cache, a queue of requests; `step()` runs one iteration."""

    def __init__(self, cfg, model: B.DeviceModel, num_blocks: int, max_batch: int, max_context: int,
                 chunk: int = 16, max_rows: int = 512, exit_rule: int = B.EE_EXIT_BATCH, thresholds=None):
        self.cfg, self.model = cfg, model
        self.cache = B.PagedKV(cfg, num_blocks)
        self.alloc = BlockAllocator(num_blocks)
        self.max_batch, self.max_context = max_batch, max_context
        self.chunk, self.max_rows = chunk, max(max_rows, max_batch)
        self.exit_rule = exit_rule
        self.thresholds = cfg.threshold if thresholds is None else thresholds
        self.max_blocks = (max_context + cfg.block_size - 1) // cfg.block_size
        self.ws = B.Workspace(model.desc, self.max_rows, max_context)
        self.waiting: List[Request] = []
        self.active: List[Request] = []
        self.finished: List[Request] = []
        self.iterations = {"prefill": 0, "decode": 0}
        self.L_hist: Dict[int, int] = {}
        rows = self.max_rows
        self._out_tok = torch.zeros(rows, dtype=torch.int32, device="cuda")
        self._out_exit = torch.zeros(rows, dtype=torch.int32, device="cuda")
        self._out_L = torch.zeros(1, dtype=torch.int32, device="cuda")

    # -- queue ---------------------------------------------------------------------------------------
    def add_request(self, prompt: List[int], max_new_tokens: int) -> Request:
        assert len(prompt) >= 1 and max_new_tokens >= 1
        assert len(prompt) + max_new_tokens <= self.max_context, "request longer than max_context"
        r = Request(len(self.waiting) + len(self.active) + len(self.finished), list(prompt), max_new_tokens,
                    arrived=time.perf_counter())
        self.waiting.append(r)
        return r

    def _admit(self):
        while self.waiting and len(self.active) < self.max_batch:
            r = self.waiting[0]
            need = (len(r.prompt) + r.max_new_tokens + self.cfg.block_size - 1) // self.cfg.block_size
            blocks = self.alloc.take(need)
            if blocks is None:
                break                       # no room in the cache: wait for an eviction
            r.blocks = blocks
            self.active.append(self.waiting.pop(0))

    def _evict(self):
        keep = []
        for r in self.active:
            if r.done:
                self.alloc.give(r.blocks)
                r.blocks = []
                self.finished.append(r)
            else:
                keep.append(r)
        self.active = keep

    # -- one iteration -------------------------------------------------------------------------------
    def _tables(self, reqs: List[Request]) -> torch.Tensor:
        t = torch.zeros(len(reqs), self.max_blocks, dtype=torch.int32)
        for i, r in enumerate(reqs):
            t[i, :len(r.blocks)] = torch.tensor(r.blocks, dtype=torch.int32)
        return t.cuda()

    def _call(self, tokens, pos, tables, row_table, rule):
        n = len(tokens)
        tok = torch.tensor(tokens, dtype=torch.int32).cuda()
        p = torch.tensor(pos, dtype=torch.int32).cuda()
        rt = None if row_table is None else torch.tensor(row_table, dtype=torch.int32).cuda()
        batch = B.make_batch(tok, p, tables, max(pos) + 1, rt)
        B.ee_decode_iteration(self.model, self.cache, batch, self.thresholds if rule else 2.0, None, rule,
                              self._out_tok[:n], self._out_exit[:n], self._out_L, None, None, self.ws)
        torch.cuda.synchronize()
        return self._out_tok[:n].cpu().tolist(), self._out_exit[:n].cpu().tolist(), int(self._out_L.item())

    def step(self) -> bool:
        """Runs one iteration (a prompt-chunk iteration if any active request still has prompt left, else a
        decode iteration).  Returns False when nothing is left to do."""
        self._admit()
        if not self.active:
            return False
        filling = [r for r in self.active if r.consumed < len(r.prompt)]
        if filling:
            tokens, pos, row_table, reqs, last_row = [], [], [], [], {}
            share = max(self.chunk, self.max_rows // len(filling))   # few prompts in flight: longer chunks each
            for r in filling:
                take = min(share, len(r.prompt) - r.consumed, self.max_rows - len(tokens))
                if take <= 0:
                    break
                reqs.append(r)
                for j in range(take):
                    tokens.append(r.prompt[r.consumed + j])
                    pos.append(r.consumed + j)
                    row_table.append(len(reqs) - 1)
                last_row[r.rid] = len(tokens) - 1
            out, _, _ = self._call(tokens, pos, self._tables(reqs), row_table, B.EE_EXIT_NONE)
            now = time.perf_counter()
            for r in reqs:
                r.consumed += sum(1 for x in row_table if reqs[x] is r)
                if r.consumed == len(r.prompt):          # the prediction after the last prompt token
                    r.generated.append(out[last_row[r.rid]])
                    r.exit_layers.append(self.cfg.n_layers)
                    r.token_times.append(now)
            self.iterations["prefill"] += 1
        else:
            reqs = self.active
            tokens = [r.generated[-1] for r in reqs]
            pos = [r.context_len for r in reqs]
            out, ex, L = self._call(tokens, pos, self._tables(reqs), None, self.exit_rule)
            now = time.perf_counter()
            for r, t, e in zip(reqs, out, ex):
                r.generated.append(t)
                r.exit_layers.append(e)
                r.token_times.append(now)
            self.L_hist[L] = self.L_hist.get(L, 0) + 1
            self.iterations["decode"] += 1
        self._evict()
        return True

    def run(self):
        while self.step():
            pass
        return self.finished


def summary(finished: List[Request], wall: float, iterations: Dict[str, int]) -> Dict:
    """Throughput and latency figures of a finished run.

    inner_token_latency_ms is the paper's definition (Evaluation, "Latency"): every sequence's decoding latency is its
    finish time minus its first-token time; the inner-token latency is the sum of those over all sequences divided by
    the total number of generated tokens.  token_gap_ms (mean and percentiles of the time between consecutive tokens
    of one request) is reported beside it."""
    gaps = sorted(b - a for r in finished for a, b in zip(r.token_times, r.token_times[1:]))
    n_tok = sum(len(r.generated) for r in finished)
    decoding = sum(r.token_times[-1] - r.token_times[0] for r in finished if r.token_times)

    def q(p):
        return gaps[min(len(gaps) - 1, int(p * len(gaps)))] * 1e3 if gaps else None

    return {"requests": len(finished), "generated_tokens": n_tok, "wall_s": wall, "tokens_per_s": n_tok / wall,
            "inner_token_latency_ms": decoding / n_tok * 1e3 if n_tok else None,
            "token_gap_ms": {"mean": sum(gaps) / len(gaps) * 1e3 if gaps else None, "p50": q(0.5), "p99": q(0.99)},
            "iterations": iterations}


def main():
    ap = argparse.ArgumentParser(description="iteration-level scheduling harness on synthetic requests")
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--requests", type=int, default=96)
    ap.add_argument("--max-batch", type=int, default=32)
    ap.add_argument("--prompt-min", type=int, default=64)
    ap.add_argument("--prompt-max", type=int, default=512)
    ap.add_argument("--new-min", type=int, default=16)
    ap.add_argument("--new-max", type=int, default=96)
    ap.add_argument("--chunk", type=int, default=16)
    ap.add_argument("--max-rows", type=int, default=512, help="rows of one prompt-chunk iteration (all prompts in flight together)")
    ap.add_argument("--exit-rule", choices=["none", "batch", "per_sequence"], default="batch")
    ap.add_argument("--conf-mode", type=int, default=-1, help="-1: the config's measure")
    ap.add_argument("--threshold", type=float, default=0.0)
    args = ap.parse_args()
    B.lib()
    cfg = W.CONFIGS[args.config]
    if args.conf_mode >= 0:
        cfg = cfg.with_(conf_mode=args.conf_mode)
    w = W.make_weights(cfg, seed=0, device="cuda")
    model = B.DeviceModel(cfg, w)
    del w
    g = torch.Generator().manual_seed(0)
    max_ctx = args.prompt_max + args.new_max
    blocks = args.max_batch * ((max_ctx + cfg.block_size - 1) // cfg.block_size)
    rule = {"none": B.EE_EXIT_NONE, "batch": B.EE_EXIT_BATCH, "per_sequence": B.EE_EXIT_PER_SEQUENCE}[args.exit_rule]
    eng = Engine(cfg, model, blocks, args.max_batch, max_ctx, chunk=args.chunk, max_rows=args.max_rows, exit_rule=rule,
                 thresholds=args.threshold or None)
    for _ in range(args.requests):
        pl = int(torch.randint(args.prompt_min, args.prompt_max + 1, (1,), generator=g))
        nn = int(torch.randint(args.new_min, args.new_max + 1, (1,), generator=g))
        eng.add_request(torch.randint(0, cfg.vocab, (pl,), generator=g).tolist(), nn)
    t0 = time.perf_counter()
    done = eng.run()
    out = summary(done, time.perf_counter() - t0, eng.iterations)
    out.update({"workload": cfg.name, "exit_rule": args.exit_rule, "conf_mode": cfg.conf_mode, "max_batch": args.max_batch,
                "chunk": args.chunk, "max_rows": args.max_rows, "batch_exit_layer_hist": dict(sorted(eng.L_hist.items())), "data": "synthetic"})
    print(json.dumps(out))


if __name__ == "__main__":
    sys.exit(main())
