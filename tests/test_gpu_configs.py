"""Parity at the shapes of every benchmark configuration, at REDUCED depth: each case keeps the configuration's real
width, batch, context mix, block-table structure and exit rule and reduces the number of layers, so that many variants
(widths, row counts, exit rules, confidence measures) run in seconds.  The same configurations at their full depth and
size are in test_gpu_full_depth.py / test_gpu_full_depth_13b.py.  The check itself runs on a seeded subset of sequences
(sequences interact only through the batch exit layer, which is checked over the full GPU output)."""
import math

import pytest
import torch

from oracle import ee_oracle as O
from paper_2407_20272_amd import binding as B
from paper_2407_20272_amd import workloads as W
from gpu_harness import F64, HipRun, assert_close_scaled, check_confidences, near_threshold, tol_of

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def setup_case(cfg, seed, sample, kv_scale=0.5):
    """Model, synthetic cache contents (generated per layer on the GPU, handed to both sides), one token per
    sequence.  Returns (run, w_cpu, lens, tokens, Ks_s, Vs_s): the last two are the sampled sequences' dense K/V."""
    n, Bsz = cfg.n_layers, cfg.batch
    w = W.make_weights(cfg, seed=seed, device="cuda", gain_jitter=0.1)
    lens = W.make_context_lens(cfg, seed=seed)
    run = HipRun(cfg, None, lens, 1, seed=seed, spare_blocks=1, weights_dev=w)
    w_cpu = W.weights_to(w, "cpu")
    del w
    max_ctx = int(lens.max()) + 1
    Ks_s, Vs_s = [], []
    for i in range(n):
        one = cfg.with_(n_layers=1)
        Kd, Vd = W.make_dense_kv(one, lens, max_ctx, seed=seed * 1000 + i, device="cuda", scale=kv_scale)
        run.cache.k[i] = W.dense_to_paged(Kd[0], run.block_tables, run.num_blocks, cfg.block_size)
        run.cache.v[i] = W.dense_to_paged(Vd[0], run.block_tables, run.num_blocks, cfg.block_size)
        Ks_s.append(Kd[0][sample].cpu())
        Vs_s.append(Vd[0][sample].cpu())
        del Kd, Vd
    tokens = torch.randint(0, cfg.vocab, (Bsz,), generator=torch.Generator().manual_seed(seed), dtype=torch.int32)
    return run, w_cpu, lens, tokens, Ks_s, Vs_s


def one_iteration_case(cfg, seed, sample, forced=None, kv_scale=0.5, threshold=None, expect_early=None):
    """Synthetic cache contents (no prefill), ONE decode iteration on the GPU over the whole batch; the oracle runs
    the sampled sequences with the GPU's batch exit layer imposed through forced exits of the remaining ones."""
    tol = tol_of(cfg)
    lam = cfg.threshold if threshold is None else threshold
    n, Bsz = cfg.n_layers, cfg.batch
    run, w_cpu, lens, tokens, Ks_s, Vs_s = setup_case(cfg, seed, sample, kv_scale)
    sub_lens = lens[sample]
    g_tok, g_exit, g_L, g_conf, g_hid = run.step(tokens, lens.long(), lam, forced=forced)
    assert g_L == int(g_exit.max()), "batch exit layer must be the largest per-sequence exit layer"
    if expect_early is not None:
        assert (g_L < n) == expect_early
    # oracle on the sample; sequences outside it only matter through L, so L is imposed: the sampled sequences get
    # their own rule (forced or threshold) and one extra pseudo-constraint: nobody may stop the loop before g_L.
    m = O.model_from_config(cfg, w_cpu)
    oc = O.DenseKV.from_tensors(Ks_s, Vs_s, sub_lens, cfg.dtype)
    f_s = None if forced is None else forced[sample]
    tr = {}
    o_tok, o_exit, o_L = oracle_with_imposed_L(m, oc, tokens[sample], sub_lens.long(), lam, f_s, g_L, tr)
    near = 0
    for r, b in enumerate(sample):
        if int(o_exit[r]) != int(g_exit[b]):
            i = min(int(o_exit[r]), int(g_exit[b]))
            assert forced is None and near_threshold(cfg, m, tr, i, r, lam), (b, int(o_exit[r]), int(g_exit[b]))
            near += 1
    assert_close_scaled(g_hid[sample], tr["h_exit"], tol, "hidden state at the batch exit layer", dim=-1, depth=g_L)
    z = O.head_logits(m, tr["h_exit"])
    for r, b in enumerate(sample):
        if int(g_tok[b]) != int(o_tok[r]):
            top = torch.topk(z[r], 2).values
            assert float(top[0] - top[1]) <= tol * float(z[r].abs().max()), f"token of sequence {b}"
    ev = ~tr["conf"].isnan()
    gc = g_conf[:, sample].to(F64)
    if forced is None and near == 0:
        assert torch.equal(ev, ~gc.isnan())
        check_confidences(cfg, m, tr, gc, "one iteration")
    for i in range(1, n + 1):                       # this position's K/V in every layer (forward or filled)
        for r, b in enumerate(sample):
            k, v = run.kv_at(i, b, int(lens[b]))
            assert_close_scaled(k, oc.K[i - 1][r, int(lens[b])], tol, f"K layer {i} sequence {b}", depth=min(i, g_L + 1))
            assert_close_scaled(v, oc.V[i - 1][r, int(lens[b])], tol, f"V layer {i} sequence {b}", depth=min(i, g_L + 1))
    return g_L, near


def oracle_with_imposed_L(m, cache, tokens, pos, lam, forced, L, trace):
    """Algorithm 1 on a subset of the batch whose exit layer L was decided by the whole batch: the subset's own
    statuses follow the normal rule; the loop leaves at L.  Implemented by appending no sequence but by running
    the oracle's own steps: decode_iteration with a per-sequence forced layer when forced, else a replay that stops
    at L.  Uses only oracle functions."""
    n = m.n_layers
    Bs = tokens.shape[0]
    h = O.store(m.weights["embed"][tokens.long()], m.dtype)
    status, exit_layer = [False] * Bs, [n] * Bs
    conf_log = torch.full((n, Bs), float("nan"), dtype=F64)
    trace["h"] = []
    for i in range(1, L + 1):
        h_prev = h
        h = O.layer_forward(m, i, h, cache, pos)
        trace["h"].append(h.clone())
        if O.has_exit_head(m, i):
            rows = [b for b in range(Bs) if not status[b]]
            if rows:
                c, _ = O.exit_check(m, i, h, rows, h_prev)
                conf = {b: float(c[r]) for r, b in enumerate(rows)}
                for b in rows:
                    conf_log[i - 1, b] = conf[b]
                if forced is not None:
                    conf = {b: (math.inf if i >= int(forced[b]) else -math.inf) for b in rows}
                O.update_status(status, exit_layer, i, conf, lam)
    O.kv_fill(m, cache, h, pos, L + 1)
    trace["conf"], trace["h_exit"] = conf_log, h.clone()
    return O.transform_to_tokens(m, h), torch.tensor(exit_layer, dtype=torch.int32), L


def per_sequence_case(cfg, seed, sample, forced, kv_scale=0.5):
    """Per-sequence exit at a configuration's shape: with this rule no sequence depends on its batch mates, so the
    oracle simply runs the sampled sequences as a batch of their own."""
    tol = tol_of(cfg)
    n = cfg.n_layers
    run, w_cpu, lens, tokens, Ks_s, Vs_s = setup_case(cfg, seed, sample, kv_scale)
    sub_lens = lens[sample]
    g_tok, g_exit, g_L, g_conf, g_hid = run.step(tokens, lens.long(), cfg.threshold, forced=forced, heads=2)
    if cfg.exit_every == 1:   # a check after every layer but the last: forced layers come back as given
        assert torch.equal(g_exit, torch.clamp(forced, max=n)), "forced exit layers must come back as given"
    assert g_L == int(g_exit.max())
    m = O.model_from_config(cfg, w_cpu)
    oc = O.DenseKV.from_tensors(Ks_s, Vs_s, sub_lens, cfg.dtype)
    tr = {}
    o_tok, o_exit, o_L = O.decode_iteration_freeze(m, oc, tokens[sample], sub_lens.long(), cfg.threshold,
                                                   forced_exit_layer=forced[sample], trace=tr)
    assert torch.equal(o_exit, g_exit[sample])
    assert_close_scaled(g_hid[sample], tr["h_exit"], tol, "each sequence's own exit hidden state", dim=-1, depth=g_L)
    z = O.head_logits(m, tr["h_exit"])
    for r, b in enumerate(sample):
        if int(g_tok[b]) != int(o_tok[r]):
            top = torch.topk(z[r], 2).values
            assert float(top[0] - top[1]) <= tol * float(z[r].abs().max()), f"token of sequence {b}"
    for i in range(1, n + 1):
        for r, b in enumerate(sample):
            k, v = run.kv_at(i, b, int(lens[b]))
            assert_close_scaled(k, oc.K[i - 1][r, int(lens[b])], tol, f"K layer {i} sequence {b}", depth=i)
            assert_close_scaled(v, oc.V[i - 1][r, int(lens[b])], tol, f"V layer {i} sequence {b}", depth=i)
    return g_L


def test_per_sequence_exit_at_7b_width_batch32_and_batch256():
    """Sequences leaving one by one at the 7B width: batch 32 (streaming projection kernel) and batch 256 with
    ragged contexts and shuffled blocks (tiled kernel); sampled sequences cover an early, a middle and a late exit."""
    cfg = W.reduced(W.CONFIGS[1], n_layers=5)
    forced = torch.tensor([1 + (b * 7) % 5 for b in range(cfg.batch)], dtype=torch.int32)
    forced[0], forced[13], forced[31] = 1, 3, 5
    assert per_sequence_case(cfg, seed=7, sample=[0, 13, 31], forced=forced) == 5
    cfg = W.reduced(W.CONFIGS[2], n_layers=4)
    forced = torch.tensor([1 + (b * 5) % 3 for b in range(cfg.batch)], dtype=torch.int32)      # everybody by layer 3
    forced[0], forced[100], forced[255] = 1, 2, 3
    assert per_sequence_case(cfg, seed=8, sample=[0, 100, 255], forced=forced) == 3


def test_config1_llama7b_width_batch32_depth4():
    cfg = W.reduced(W.CONFIGS[1], n_layers=4, logit_scale=4.0)       # logit scale raised so exits happen by layer 3
    one_iteration_case(cfg, seed=1, sample=[0, 13, 31])


@pytest.mark.parametrize("conf_mode,threshold", [(2, 0.85), (3, 0.6)])
def test_config1_width_headless_measures(conf_mode, threshold):
    """Hidden-state similarity and classifier checks at the 7B width (no LM head inside the loop)."""
    cfg = W.reduced(W.CONFIGS[1], n_layers=6, conf_mode=conf_mode, threshold=threshold)
    one_iteration_case(cfg, seed=9, sample=[0, 13, 31])


def test_config2_batch256_ragged_shuffled_depth3():
    cfg = W.reduced(W.CONFIGS[2], n_layers=3, logit_scale=5.0)
    L, near = one_iteration_case(cfg, seed=2, sample=[0, 100, 255])
    assert 1 <= L <= 3


@pytest.mark.parametrize("batch,ctx", [(64, 1024), (512, 768)])
def test_config3_exit_sweep_forced_exits(batch, ctx):
    cfg = W.reduced(W.CONFIGS[3], n_layers=4, batch=batch, prompt_len=ctx, min_prompt_len=ctx)
    forced = torch.clamp(W.make_forced_exit_layers(batch, 1, mean=12, seed=3)[0] - 8, 1, 4).to(torch.int32)  # 8..32 -> 1..4
    forced[::7] = 2
    L, _ = one_iteration_case(cfg, seed=3, sample=[0, batch // 2, batch - 1], forced=forced)
    assert L == int(forced.max())
    forced_early = torch.full((batch,), 2, dtype=torch.int32)
    L, _ = one_iteration_case(cfg, seed=4, sample=[1, batch - 2], forced=forced_early, expect_early=True)
    assert L == 2


def test_config4_llama13b_width_heads_every_4th_layer():
    cfg = W.reduced(W.CONFIGS[4], n_layers=9, batch=64, prompt_len=4096, min_prompt_len=4096, logit_scale=4.0,
                    d_ffn=1024)          # 13B attention/projection width, 40 heads, context 4096; FFN narrowed
    L, near = one_iteration_case(cfg, seed=5, sample=[0, 63], threshold=0.5)
    assert L in (4, 8, 9)


def test_config4_llama13b_ffn_width():
    cfg = W.reduced(W.CONFIGS[4], n_layers=2, batch=64, prompt_len=64, min_prompt_len=64, logit_scale=8.0)
    one_iteration_case(cfg, seed=6, sample=[0, 31, 63], threshold=0.3)


@pytest.mark.parametrize("batch", [96, 160])
def test_13b_width_row_counts_of_the_tiled_projection_kernel(batch):
    """13B widths (40, 120, 216 and 250 groups of output tiles: not multiples of 8, so the XCD-aware grid is
    padded) at row counts whose last 128-row chunk is short."""
    cfg = W.reduced(W.CONFIGS[4], n_layers=2, batch=batch, prompt_len=64, min_prompt_len=64, logit_scale=8.0)
    one_iteration_case(cfg, seed=7, sample=[0, batch // 2, batch - 1], threshold=0.3)


def test_config1_full_size_one_iteration_sampled():
    """The benchmark workload itself: 32 layers, batch 32, context 512, exit head after every layer, threshold 0.9
    (hidden state, exit layers, confidences, tokens and this position's K/V of all 32 layers for sampled sequences)."""
    L, near = one_iteration_case(W.CONFIGS[1], seed=7, sample=[0, 17, 31], kv_scale=0.3)
    assert 1 <= L <= 32


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "bf16_per_sequence_160"])
def test_hip_graph_replay_matches_eager(dtype):
    """The launch configuration bench.py times: one iteration captured into a HIP graph and replayed, with eager work and
    synchronisations between replays; every replay must reproduce the eager iteration's outputs bit for bit, in fp32 and
    in bf16 (no sum in either path depends on the order in which workgroups finish)."""
    if dtype == "fp32":
        cfg = W.CONFIGS[0].with_(n_layers=5, batch=8, prompt_len=40, min_prompt_len=40, weight_std=0.05, logit_scale=1.0,
                                 threshold=0.4)
    elif dtype == "bf16":
        cfg = W.reduced(W.CONFIGS[1], n_layers=5, d_model=512, n_heads=4, d_ffn=1408, vocab=2048, batch=32, prompt_len=40,
                        min_prompt_len=40, weight_std=0.05, logit_scale=1.0, threshold=0.4)
    else:   # per-sequence exit with the active rows compacted (device-side row map: nothing for the graph to bake in)
        cfg = W.reduced(W.CONFIGS[1], n_layers=5, d_model=512, n_heads=4, d_ffn=1408, vocab=2048, batch=160, prompt_len=40,
                        min_prompt_len=40, weight_std=0.05, logit_scale=1.0, threshold=0.4)
    exit_rule = B.EE_EXIT_PER_SEQUENCE if dtype == "bf16_per_sequence_160" else B.EE_EXIT_BATCH
    w = W.make_weights(cfg, seed=8, gain_jitter=0.1)
    lens = W.make_context_lens(cfg, seed=8)
    steps = 4
    run = HipRun(cfg, w, lens, steps + 2, seed=8)
    Ks, Vs = W.make_dense_kv(cfg, lens, int(lens.max()), seed=8, scale=0.5)
    run.load_dense(Ks, Vs)
    k0, v0 = run.cache.k.clone(), run.cache.v.clone()
    tok0 = W.make_prompts(cfg, seed=8)[:, 0].contiguous().cuda()
    tokens, ctx = tok0.clone(), lens.cuda().clone()
    batch = B.make_batch(tokens, ctx, run.bt_dev, int(lens.max()) + steps + 2)

    def iteration():
        B.ee_decode_iteration(run.model, run.cache, batch, cfg.threshold, None, exit_rule, run.out_tokens, run.out_exit,
                              run.out_L, None, run.out_hidden, run.ws)
        torch.add(run.out_tokens, 0, out=tokens)
        ctx.add_(1)

    def reset():
        run.cache.k.copy_(k0)
        run.cache.v.copy_(v0)
        tokens.copy_(tok0)
        ctx.copy_(lens.cuda())

    eager = []
    for s in range(steps):
        iteration()
        torch.cuda.synchronize()
        eager.append((run.out_tokens.cpu().clone(), run.out_exit.cpu().clone(), int(run.out_L.item()), run.out_hidden.cpu().clone()))
    k1, v1 = run.cache.k.clone(), run.cache.v.clone()
    side = torch.cuda.Stream()
    reset()
    with torch.cuda.stream(side):
        iteration()                                   # warm-up outside the capture
        torch.cuda.synchronize()
        reset()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            iteration()
    torch.cuda.synchronize()
    reset()
    scratch = torch.zeros(1 << 20, device="cuda")
    for s in range(steps):
        g.replay()
        scratch.add_(1.0)                             # the program's own eager work between replays
        torch.cuda.synchronize()
        t, e, L, h = eager[s]
        assert torch.equal(run.out_tokens.cpu(), t) and torch.equal(run.out_exit.cpu(), e) and int(run.out_L.item()) == L, s
        assert torch.equal(run.out_hidden.cpu(), h), s
    assert torch.equal(run.cache.k, k1) and torch.equal(run.cache.v, v1)
