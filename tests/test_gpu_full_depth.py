"""Parity at FULL depth and full size for every benchmark configuration with 7B / 13B-shaped models: the real layer
count (32 / 40), batch, width, context mix, block-table structure, head spacing and exit rule.

The pools are filled on the device (seeded N(0, 0.3^2) contents, as bench.py does for ragged workloads) and only the
sampled sequences' K/V is read back through the block tables for the oracle.  The oracle runs the sampled sequences
with the GPU's batch exit layer imposed (sequences interact only through it; it is checked over the full GPU output).
Each test prints its wall time, the batch exit layer and the number of near-threshold decisions / near-tie tokens."""
import math
import time

import pytest
import torch

from oracle import ee_oracle as O
from paper_2407_20272_amd import binding as B
from paper_2407_20272_amd import workloads as W
from gpu_harness import F64, HipRun, assert_close_scaled, check_confidences, near_threshold, tol_of
from test_gpu_configs import oracle_with_imposed_L

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1200)]


class SharedModel:
    """One set of random weights on the device (packed once) and on the host, shared by the cases of a shape."""

    def __init__(self, cfg, seed):
        w = W.make_weights(cfg, seed=seed, device="cuda", gain_jitter=0.1)
        self.cfg, self.seed = cfg, seed
        self.dev = B.DeviceModel(cfg, w)
        self.w_cpu = W.weights_to(w, "cpu")
        del w
        torch.cuda.empty_cache()

    def oracle(self, cfg):
        return O.model_from_config(cfg, self.w_cpu)

    def device(self, cfg):
        """The same packed weights under another exit rule / batch (a second host-side record, nothing copied)."""
        import copy
        v = copy.copy(self.dev)
        v.cfg = cfg
        v.desc = B.make_desc(cfg)
        v.c = B.ee_model(v.desc, self.dev.c.embed, self.dev.c.g_final, self.dev.c.w_lm, self.dev.layers, self.dev.c.w_cls,
                         self.dev.c.b_cls)
        return v


@pytest.fixture(scope="module")
def model7b():
    m = SharedModel(W.CONFIGS[1], seed=7)
    yield m
    del m
    torch.cuda.empty_cache()


def report(capsys, what, t0, **kw):
    with capsys.disabled():
        print(f"\n[full depth] {what}: {time.time() - t0:.1f} s, " + ", ".join(f"{k} {v}" for k, v in kw.items()), flush=True)


def device_filled_run(shared, cfg, seed, extra_tokens, kv_scale=0.3):
    lens = W.make_context_lens(cfg, seed=seed)
    run = HipRun(cfg, None, lens, extra_tokens, seed=seed, spare_blocks=1, model=shared.device(cfg))
    g = torch.Generator(device="cuda").manual_seed(1000 + seed)
    for i in range(cfg.n_layers):
        run.cache.k[i].normal_(0.0, kv_scale, generator=g)
        run.cache.v[i].normal_(0.0, kv_scale, generator=g)
    return run, lens


def sampled_cache(run, cfg, sample, lens, extra_tokens):
    """The sampled sequences' K/V read back through the block tables: an oracle cache over them."""
    ctx = int(lens[sample].max()) + extra_tokens
    bt = run.block_tables[sample]
    Ks = [W.paged_to_dense(run.cache.k[i], bt, ctx).cpu() for i in range(cfg.n_layers)]
    Vs = [W.paged_to_dense(run.cache.v[i], bt, ctx).cpu() for i in range(cfg.n_layers)]
    return O.DenseKV.from_tensors(Ks, Vs, lens[sample], cfg.dtype)


def check_iteration(cfg, m, run, oc, sample, tokens, pos, lam, forced, g_out, what):
    """One GPU iteration (already run: g_out) against the oracle on the sampled sequences.  Returns the oracle's
    tokens for the sample and the counts of tolerated divergences."""
    tol = tol_of(cfg)
    n = cfg.n_layers
    g_tok, g_exit, g_L, g_conf, g_hid = g_out
    assert g_L == int(g_exit.max()), "batch exit layer must be the largest per-sequence exit layer"
    f_s = None if forced is None else forced[sample]
    tr = {}
    o_tok, o_exit, _ = oracle_with_imposed_L(m, oc, tokens[sample], pos[sample].long(), lam, f_s, g_L, tr)
    near = ties = 0
    replay = False
    for r, b in enumerate(sample):
        if int(o_exit[r]) != int(g_exit[b]):
            i = min(int(o_exit[r]), int(g_exit[b]))
            assert forced is None and near_threshold(cfg, m, tr, i, r, lam), \
                f"{what}: exit layer of sequence {b}: gpu {int(g_exit[b])}, oracle {int(o_exit[r])}, confidence " \
                f"{float(tr['conf'][i - 1, r])} is not near the threshold"
            near += 1
            replay = True
    assert_close_scaled(g_hid[sample], tr["h_exit"], tol, f"{what}: hidden state at the batch exit layer", dim=-1, depth=g_L)
    z = O.head_logits(m, tr["h_exit"])
    for r, b in enumerate(sample):
        if int(g_tok[b]) != int(o_tok[r]):
            top = torch.topk(z[r], 2).values
            assert float(top[0] - top[1]) <= tol * float(z[r].abs().max()), f"{what}: token of sequence {b}"
            ties += 1
    if forced is None and not replay:
        gc = g_conf[:, sample].to(F64)
        assert torch.equal(~tr["conf"].isnan(), ~gc.isnan()), f"{what}: different (layer, sequence) pairs were checked"
        check_confidences(cfg, m, tr, gc, what)
    for i in range(1, n + 1):                       # this position's K/V in every layer (forward or filled)
        for r, b in enumerate(sample):
            p = int(pos[b])
            k, v = run.kv_at(i, b, p)
            assert_close_scaled(k, oc.K[i - 1][r, p], tol, f"{what}: K layer {i} sequence {b}", depth=min(i, g_L + 1))
            assert_close_scaled(v, oc.V[i - 1][r, p], tol, f"{what}: V layer {i} sequence {b}", depth=min(i, g_L + 1))
    return o_tok, near, ties


def one_iteration(capsys, shared, cfg, seed, sample, forced=None, lam=None, what=""):
    t0 = time.time()
    lam = cfg.threshold if lam is None else lam
    run, lens = device_filled_run(shared, cfg, seed, 1)
    tokens = torch.randint(0, cfg.vocab, (cfg.batch,), generator=torch.Generator().manual_seed(seed), dtype=torch.int32)
    g_out = run.step(tokens, lens.long(), lam, forced=forced)
    oc = sampled_cache(run, cfg, sample, lens, 1)
    _, near, ties = check_iteration(cfg, shared.oracle(cfg), run, oc, sample, tokens, lens, lam, forced, g_out, what)
    report(capsys, what, t0, batch_exit_layer=g_out[2], near_threshold=near, near_tie=ties,
           exit_layers=sorted(set(g_out[1].tolist())))
    return g_out[2]


# ------------------------------------------------------------------------------------------------------
# config 1: prompt chunks on the GPU, then consecutive decode iterations in lock step
# ------------------------------------------------------------------------------------------------------
def test_config1_chunked_prefill_then_four_decode_iterations(capsys, model7b):
    """Batch 32, prompts of 512 tokens pushed through the decode step in chunks of 16 positions per sequence (no exit
    checks), then four decode iterations with the config's exit rule.  The oracle starts from the GPU's cache of the
    sampled sequences and stays in lock step: token feedback, position advance, the first decode position opening a
    new block (512 = 32 blocks of 16)."""
    t0 = time.time()
    cfg = W.CONFIGS[1]
    Bsz, n, P, steps, T = cfg.batch, cfg.n_layers, cfg.prompt_len, 4, 16
    sample = [0, 17, 31]
    lens = W.make_context_lens(cfg, seed=7)
    run = HipRun(cfg, None, lens, steps, seed=7, spare_blocks=1, model=model7b.device(cfg), pool_fill=7.0)
    prompts = W.make_prompts(cfg, seed=7)
    # prompt chunks: rows = (sequence, position) pairs that share the sequence's block table
    ws = B.Workspace(run.model.desc, Bsz * T, P + steps)
    out_tok = torch.zeros(Bsz * T, dtype=torch.int32, device="cuda")
    out_exit = torch.zeros(Bsz * T, dtype=torch.int32, device="cuda")
    out_L = torch.zeros(1, dtype=torch.int32, device="cuda")
    row_table = torch.arange(Bsz, dtype=torch.int32).repeat_interleave(T).cuda()
    for p0 in range(0, P, T):
        toks = prompts[:, p0:p0 + T].reshape(-1).contiguous().cuda()
        pos = (torch.arange(p0, p0 + T, dtype=torch.int32)[None, :].expand(Bsz, T)).reshape(-1).contiguous().cuda()
        batch = B.make_batch(toks, pos, run.bt_dev, P + steps, row_table=row_table)
        B.ee_decode_iteration(run.model, run.cache, batch, 2.0, None, B.EE_EXIT_NONE, out_tok, out_exit, out_L, None, None, ws)
    torch.cuda.synchronize()
    first = out_tok.view(Bsz, T)[:, -1].cpu().clone()           # prediction after the last prompt token
    m = model7b.oracle(cfg)
    oc = sampled_cache(run, cfg, sample, lens, steps)
    pos = lens.clone()
    tok = first.clone()
    Ls, near_all, ties_all = [], 0, 0
    for s in range(steps):
        g_out = run.step(tok, pos.long(), cfg.threshold)
        o_tok, near, ties = check_iteration(cfg, m, run, oc, sample, tok, pos, cfg.threshold, None, g_out, f"decode step {s}")
        near_all, ties_all = near_all + near, ties_all + ties
        Ls.append(g_out[2])
        nxt = g_out[0].clone()
        for r, b in enumerate(sample):                           # teacher forcing: the sample continues from the oracle's tokens
            nxt[b] = o_tok[r]
        tok = nxt
        pos = pos + 1
    report(capsys, "config 1, chunked prefill + 4 decode iterations", t0, batch_exit_layers=Ls, near_threshold=near_all,
           near_tie=ties_all)


def test_config1_full_depth_softmax_response_top1_minus_top2(capsys, model7b):
    """The paper's own softmax-response measure (Section 2.1: top-1 minus top-2 probability of the exit head) at the 7B
    shape, 32 layers, batch 32: same fused reduction with the runner-up logit carried along.  The threshold is set
    where the batch leaves inside the model."""
    cfg = W.CONFIGS[1].with_(conf_mode=1, threshold=0.6, name="llama7b_b32_ctx512_softmax_response")
    L = one_iteration(capsys, model7b, cfg, seed=11, sample=[0, 9, 31], what="config 1 shape, top-1 minus top-2")
    assert 1 <= L <= cfg.n_layers


# ------------------------------------------------------------------------------------------------------
# config 2: batch 256, ragged contexts 128..2048, shuffled blocks, 32 layers
# ------------------------------------------------------------------------------------------------------
def test_config2_full_depth_batch256_ragged_shuffled(capsys, model7b):
    cfg = W.CONFIGS[2]
    L = one_iteration(capsys, model7b, cfg, seed=2, sample=[0, 100, 255], what="config 2 (batch 256, ragged, shuffled)")
    assert 1 <= L <= cfg.n_layers


# ------------------------------------------------------------------------------------------------------
# config 3: forced exit layers from the truncated geometric distribution on [8, 32], batch 64 / 256 / 512
# ------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("batch,ctx,mean", [(64, 1024, 12.0), (256, 1024, 20.0), (512, 768, 12.0)])
def test_config3_full_depth_forced_exit_sweep(capsys, model7b, batch, ctx, mean):
    cfg = W.CONFIGS[3].with_(batch=batch, prompt_len=ctx, min_prompt_len=ctx, name=f"llama7b_exit_sweep_b{batch}")
    forced = W.make_forced_exit_layers(batch, 1, mean=mean, seed=3)[0]
    if batch == 64:
        forced = torch.clamp(forced, max=20)      # a batch that does leave early: KV filling over the top 12 layers
    L = one_iteration(capsys, model7b, cfg, seed=3, sample=[0, batch // 2, batch - 1], forced=forced,
                      what=f"config 3 (batch {batch}, context {ctx}, forced exits of mean {mean})")
    assert L == int(forced.max())
