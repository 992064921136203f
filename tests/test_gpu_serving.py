"""The scheduling harness around the decode step: prompt chunks (several rows per sequence in one call) against the
oracle's token-by-token prefill, and a whole evict / replenish run against the oracle run request by request."""
import pytest
import torch

from oracle import ee_oracle as O
from paper_2407_20272_amd import binding as B
from paper_2407_20272_amd import serving as S
from paper_2407_20272_amd import workloads as W
from gpu_harness import F64, assert_close_scaled, tol_of

pytestmark = pytest.mark.gpu
TINY, L7B = W.CONFIGS[0], W.CONFIGS[1]


def make_requests(cfg, n, seed, pmin, pmax, nmin, nmax):
    g = torch.Generator().manual_seed(seed)
    out = []
    for _ in range(n):
        pl = int(torch.randint(pmin, pmax + 1, (1,), generator=g))
        nn = int(torch.randint(nmin, nmax + 1, (1,), generator=g))
        out.append((torch.randint(0, cfg.vocab, (pl,), generator=g, dtype=torch.int32), nn))
    return out


def oracle_alone(cfg, w, prompt, n_new, rule, threshold):
    """One request on its own: prefill, then n_new - 1 decode iterations.  Returns (tokens, exit layers, cache)."""
    m = O.model_from_config(cfg, w)
    P = int(prompt.shape[0])
    cache = O.DenseKV(cfg.n_layers, 1, P + n_new, cfg.n_heads, cfg.head_dim, cfg.dtype)
    tok = O.prefill(m, cache, prompt[None], torch.tensor([P]))
    toks, exits = [int(tok[0])], [cfg.n_layers]
    pos = torch.tensor([P])
    for _ in range(n_new - 1):
        if rule == B.EE_EXIT_PER_SEQUENCE:
            tok, e, _ = O.decode_iteration_freeze(m, cache, tok, pos, threshold)
        else:
            tok, e, _ = O.decode_iteration(m, cache, tok, pos, threshold, heads=rule != B.EE_EXIT_NONE)
        toks.append(int(tok[0]))
        exits.append(int(e[0]))
        pos = pos + 1
    return toks, exits, cache


@pytest.mark.parametrize("name", ["tiny_fp32", "bf16_160_rows"])
def test_prompt_chunks_match_token_by_token_prefill(name):
    """Rows that share a block table at consecutive positions: cache contents and first tokens equal the oracle's
    token-by-token prefill.  The bf16 case pushes 160 rows per call (the tiled projection kernel's path)."""
    if name == "tiny_fp32":
        cfg, n_req, chunk, pmax = TINY, 5, 4, 19
    else:
        cfg = W.reduced(L7B, n_layers=3, d_model=256, n_heads=2, head_dim=128, d_ffn=352, vocab=1024, weight_std=0.05)
        n_req, chunk, pmax = 20, 8, 30
    w = W.make_weights(cfg, seed=51, gain_jitter=0.1)
    model = B.DeviceModel(cfg, w)
    reqs = make_requests(cfg, n_req, 51, 3, pmax, 1, 1)
    eng = S.Engine(cfg, model, num_blocks=n_req * 3, max_batch=n_req, max_context=pmax + 1, chunk=chunk,
                   max_rows=n_req * chunk, exit_rule=B.EE_EXIT_NONE)
    handles = [eng.add_request(p.tolist(), n) for p, n in reqs]
    eng._admit()
    blocks = {r.rid: list(r.blocks) for r in eng.active}
    eng.run()
    assert eng.iterations["prefill"] >= 2 and eng.iterations["decode"] == 0
    tol = tol_of(cfg)
    m = O.model_from_config(cfg, w)
    for r, (prompt, _) in zip(handles, reqs):
        P = int(prompt.shape[0])
        oc = O.DenseKV(cfg.n_layers, 1, P + 1, cfg.n_heads, cfg.head_dim, cfg.dtype)
        h_last = torch.zeros(1, cfg.d_model, dtype=F64)
        first = O.prefill(m, oc, prompt[None], torch.tensor([P]), last_hidden=h_last)
        if r.generated[0] != int(first[0]):
            z = O.head_logits(m, h_last)[0]
            top = torch.topk(z, 2).values
            assert float(top[0] - top[1]) <= tol * float(z.abs().max()), f"first token of request {r.rid}"
        for i in range(cfg.n_layers):
            for p in range(P):
                blk, off = blocks[r.rid][p // cfg.block_size], p % cfg.block_size
                assert_close_scaled(eng.cache.k[i, blk, :, off, :].cpu(), oc.K[i][0, p], tol, f"K layer {i + 1} req {r.rid} pos {p}")
                assert_close_scaled(eng.cache.v[i, blk, :, off, :].cpu(), oc.V[i][0, p], tol, f"V layer {i + 1} req {r.rid} pos {p}")


@pytest.mark.parametrize("rule,conf_mode,threshold", [(B.EE_EXIT_NONE, 0, 0.8), (B.EE_EXIT_PER_SEQUENCE, 0, 0.8),
                                                       (B.EE_EXIT_PER_SEQUENCE, 2, 0.6)])
def test_evict_and_replenish_run_matches_each_request_alone(rule, conf_mode, threshold):
    """Seven requests through three batch slots: requests finish and leave, waiting ones take their place, prompt
    chunks and decode iterations interleave.  With full layers or per-sequence exit a request does not depend on
    its batch mates, so every request must produce what the oracle produces for it alone (fp32: exactly)."""
    cfg = TINY.with_(conf_mode=conf_mode)
    w = W.make_weights(cfg, seed=52, gain_jitter=0.1)
    model = B.DeviceModel(cfg, w)
    reqs = make_requests(cfg, 7, 52, 3, 20, 2, 6)
    eng = S.Engine(cfg, model, num_blocks=8, max_batch=3, max_context=26, chunk=4, max_rows=12, exit_rule=rule,
                   thresholds=threshold)
    handles = [eng.add_request(p.tolist(), n) for p, n in reqs]
    done = eng.run()
    assert len(done) == 7 and not eng.active and not eng.waiting
    assert len(eng.alloc.free) == 8                                    # every block came back
    assert eng.iterations["prefill"] > 0 and eng.iterations["decode"] > 0
    early = 0
    for r, (prompt, n_new) in zip(handles, reqs):
        toks, exits, _ = oracle_alone(cfg, w, prompt, n_new, rule, threshold)
        assert r.generated == toks, (r.rid, r.generated, toks)
        assert r.exit_layers == exits, (r.rid, r.exit_layers, exits)
        assert len(r.token_times) == n_new and all(b >= a for a, b in zip(r.token_times, r.token_times[1:]))
        early += sum(e < cfg.n_layers for e in exits)
    if rule == B.EE_EXIT_PER_SEQUENCE:
        assert early > 0                                               # the rule did something
    s = S.summary(done, 1.0, eng.iterations)
    assert s["generated_tokens"] == sum(n for _, n in reqs)
