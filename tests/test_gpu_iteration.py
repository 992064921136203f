"""Whole-iteration parity on the GPU: ee_decode_iteration against the CPU oracle in lock step (prefill + decode),
the oracle's invariants replayed on the HIP path, and the stored tiny-config trajectory."""
import json
import os

import pytest
import torch

from paper_2407_20272_amd import workloads as W
from gpu_harness import HipRun, lockstep

pytestmark = pytest.mark.gpu
TINY, L7B = W.CONFIGS[0], W.CONFIGS[1]
HERE = os.path.dirname(os.path.abspath(__file__))


def small_bf16(**kw):
    base = dict(n_layers=4, d_model=256, n_heads=2, head_dim=128, d_ffn=352, vocab=1024, batch=5, prompt_len=9,
                min_prompt_len=9, decode_steps=6, weight_std=0.05, logit_scale=1.0, threshold=0.5)
    base.update(kw)
    return W.reduced(L7B, **base)


def test_tiny_fp32_full_trajectory_matches_oracle_and_stored_values():
    """Benchmark config 0 exactly as defined (seed 0, gains 1): all 16 decode steps, zero tolerated divergences."""
    stats = lockstep(TINY, seed=0, steps=TINY.decode_steps, gain_jitter=0.0)
    assert stats["near_threshold"] == 0 and stats["near_tie"] == 0
    with open(os.path.join(HERE, "golden", "tiny_fp32_seed0.json")) as f:
        want = json.load(f)
    assert stats["L"] == want["batch_exit_layer"]


def test_tiny_fp32_untied_head_trajectory_with_varying_tokens():
    """The tiny shape with an untied head and wider weights (the stored second trajectory): every step emits a
    different token per sequence, the batch leaves at layers 2, 3 and 4; all 16 steps, zero tolerated divergences."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    cfg, seed = gen.case("tiny_fp32_untied_seed4")
    stats = lockstep(cfg, seed=seed, steps=cfg.decode_steps, gain_jitter=0.0)
    assert stats["near_threshold"] == 0 and stats["near_tie"] == 0
    with open(os.path.join(HERE, "golden", "tiny_fp32_untied_seed4.json")) as f:
        want = json.load(f)
    assert stats["L"] == want["batch_exit_layer"]


@pytest.mark.parametrize("seed", [1, 2])
def test_tiny_fp32_other_seeds_with_gain_jitter(seed):
    stats = lockstep(TINY.with_(decode_steps=6, weight_std=0.05, logit_scale=1.0, threshold=0.3), seed=seed, steps=6)
    assert stats["near_threshold"] == 0 and stats["near_tie"] == 0


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_two_sequences_long_prompts_attention_split_among_workgroups(dtype):
    """Two sequences with prompts of 140 to 300 tokens and two heads: the iteration's attention gives every
    (sequence, head) pair to two workgroups (a part of the context each) and merges them in a second launch."""
    if dtype == "fp32":
        cfg = TINY.with_(batch=2, n_heads=2, head_dim=128, prompt_len=300, min_prompt_len=140, decode_steps=3, weight_std=0.05,
                         logit_scale=1.0, threshold=0.3, shuffled_blocks=True)
    else:
        cfg = small_bf16(batch=2, prompt_len=300, min_prompt_len=140, shuffled_blocks=True)
    stats = lockstep(cfg, seed=47, steps=3)
    total = stats["decisions"] + stats["tokens"]
    assert stats["near_threshold"] + stats["near_tie"] <= max(2, total // 20), stats


def test_fp32_ragged_prompts_shuffled_blocks_conf_mode1():
    cfg = TINY.with_(batch=6, prompt_len=21, min_prompt_len=3, shuffled_blocks=True, conf_mode=1, weight_std=0.05,
                     logit_scale=2.0, threshold=0.2, n_layers=5, exit_every=2)
    stats = lockstep(cfg, seed=3, steps=5)
    assert stats["near_threshold"] == 0 and stats["near_tie"] == 0


@pytest.mark.parametrize("batch", [5, 32, 40, 70])
def test_small_bf16_lockstep(batch):
    """bf16 path (MFMA projections, tiled layouts): batch sizes below, at and above one and two 32-row tiles."""
    cfg = small_bf16(batch=batch, shuffled_blocks=True, prompt_len=12, min_prompt_len=4)
    stats = lockstep(cfg, seed=10 + batch, steps=5)
    total = stats["decisions"] + stats["tokens"]
    assert stats["near_threshold"] + stats["near_tie"] <= max(2, total // 20), stats
    assert len(set(stats["L"])) >= 1


def test_bf16_width_1280_partly_rearranged_tile_order():
    """d_model 1280 (10 heads x 128): the QKV projection has 80 whole and 40 halved tiles, so the XCD-aware tile
    order of the streaming kernel rearranges 64 of each and leaves the rest in place; KV filling runs too."""
    cfg = small_bf16(d_model=1280, n_heads=10, head_dim=128, n_layers=3, batch=7, threshold=0.35, shuffled_blocks=True)
    stats = lockstep(cfg, seed=61, steps=4)
    total = stats["decisions"] + stats["tokens"]
    assert stats["near_threshold"] + stats["near_tie"] <= max(2, total // 20), stats


@pytest.mark.parametrize("batch,n_layers,exit_every,conf_mode,threshold", [
    (1, 3, 1, 0, 0.4), (7, 6, 3, 0, 0.3), (33, 5, 2, 1, 0.2), (64, 4, 1, 0, 0.45), (12, 7, 1, 0, 0.9), (20, 5, 1, 0, 0.05)])
def test_bf16_exit_decision_carried_by_the_next_projection(batch, n_layers, exit_every, conf_mode, threshold):
    """Batches the streaming projection kernel serves (the exit decision of a layer is taken inside the next layer's
    QKV launch): one and two batch tiles, heads after every / every 2nd / 3rd layer, thresholds from "everybody
    leaves at the first head" (the projection after it runs speculatively) to "nobody ever leaves"."""
    cfg = small_bf16(batch=batch, n_layers=n_layers, exit_every=exit_every, conf_mode=conf_mode, threshold=threshold,
                     shuffled_blocks=True, prompt_len=10, min_prompt_len=3)
    stats = lockstep(cfg, seed=70 + batch, steps=4)
    total = stats["decisions"] + stats["tokens"]
    assert stats["near_threshold"] + stats["near_tie"] <= max(2, total // 20), stats


def test_small_bf16_head_dim_64_exit_every_2_mode1():
    cfg = small_bf16(n_heads=4, head_dim=64, n_layers=6, exit_every=2, conf_mode=1, batch=9, threshold=0.3)
    lockstep(cfg, seed=21, steps=4)


def test_threshold_above_one_equals_full_layer_path():
    """Invariant: a threshold no confidence can pass reproduces the head-less full-layer path bit for bit."""
    for cfg in (TINY.with_(decode_steps=4), small_bf16()):
        w = W.make_weights(cfg, seed=4, gain_jitter=0.1)
        prompts, lens = W.make_prompts(cfg, seed=4), W.make_context_lens(cfg, seed=4)
        outs = []
        for heads in (True, False):
            run = HipRun(cfg, w, lens, 4, seed=4)
            tok = run.prefill(prompts, lens)
            pos = lens.clone().long()
            toks = [tok]
            for s in range(4):
                tok, e, L, conf, hid = run.step(tok, pos, 1.0 + 1e-6, heads=heads)
                assert L == cfg.n_layers and bool((e == cfg.n_layers).all())
                toks.append(tok)
                pos += 1
            outs.append((torch.stack(toks), run.cache.k.clone(), run.cache.v.clone()))
        assert torch.equal(outs[0][0], outs[1][0])
        assert torch.equal(outs[0][1], outs[1][1]) and torch.equal(outs[0][2], outs[1][2])     # fp32 and bf16 alike


@pytest.mark.parametrize("cfg", [TINY.with_(n_layers=6, decode_steps=3), small_bf16(n_layers=6)], ids=["fp32", "bf16"])
def test_forced_exit_lockstep(cfg):
    """Synthetic confidence injection: per-sequence forced exit layers, the batch leaves at their maximum."""
    g = torch.Generator().manual_seed(9)
    forced = torch.randint(1, cfg.n_layers + 1, (4, cfg.batch), generator=g, dtype=torch.int32)
    forced[1] = 2                                  # static mode: everybody leaves at layer 2
    forced[2] = cfg.n_layers                       # nobody leaves early
    stats = lockstep(cfg, seed=5, steps=4, forced_seq=forced)
    assert stats["L"] == [int(forced[s].max()) for s in range(4)]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_saturated_model_forced_exit_cache_equals_full_pass(dtype):
    """Invariant: when the layers above L0 add nothing to the residual stream, a forced exit at L0 leaves the
    whole cache and the tokens identical to a full pass."""
    cfg = (TINY if dtype == "fp32" else small_bf16()).with_(n_layers=5)
    L0 = 3
    w = W.make_weights(cfg, seed=6, gain_jitter=0.1)
    for i in range(L0, cfg.n_layers):
        w["layers"][i]["w_o"].zero_()
        w["layers"][i]["w_down"].zero_()
    prompts, lens = W.make_prompts(cfg, seed=6), W.make_context_lens(cfg, seed=6)
    res = []
    for forced_mode in (True, False):
        run = HipRun(cfg, w, lens, 3, seed=6)
        tok = run.prefill(prompts, lens)
        pos = lens.clone().long()
        toks = []
        for s in range(3):
            f = torch.full((cfg.batch,), L0, dtype=torch.int32) if forced_mode else None
            tok, e, L, _, _ = run.step(tok, pos, 0.5, forced=f, heads=forced_mode)
            assert L == (L0 if forced_mode else cfg.n_layers)
            toks.append(tok)
            pos += 1
        res.append((torch.stack(toks), run.cache.k.clone(), run.cache.v.clone()))
    assert torch.equal(res[0][0], res[1][0])
    if dtype == "fp32":
        assert torch.equal(res[0][1], res[1][1]) and torch.equal(res[0][2], res[1][2])
    else:
        # Layers up to L0 ran the same kernels on the same values in both runs: identical bits.  Above L0 the filling
        # launch and the full pass's own QKV launch project the same normalised operand but sum the contraction in
        # different orders (different kernels; the V tiles of the forward launch are split between two workgroups), so
        # a value may land on the neighbouring bf16 number (or, where the terms cancel, within float noise of zero).
        for pool in (1, 2):
            assert torch.equal(res[0][pool][:L0], res[1][pool][:L0])
            a, b = res[0][pool][L0:].float(), res[1][pool][L0:].float()
            step = torch.exp2(torch.floor(torch.log2(torch.clamp(b.abs(), min=1e-30))) - 7)        # one bf16 step at b
            assert bool(((a - b).abs() <= torch.clamp(step * 1.001, min=1e-5 * float(b.abs().max()))).all()), \
                "a filled value is more than one bf16 step from the full pass's"
            assert float((a != b).float().mean()) < 0.02, "more than 2 % of the filled values differ in the last bit"


def test_empty_batch_is_a_noop():
    cfg = TINY
    w = W.make_weights(cfg, seed=0)
    run = HipRun(cfg, w, torch.tensor([3], dtype=torch.int32), 1)
    tok, e, L, conf, hid = run.step(torch.zeros(0, dtype=torch.int32), torch.zeros(0, dtype=torch.long), 0.5,
                                    rows=[])
    assert tok.numel() == 0 and e.numel() == 0


# ------------------------------------------------------------------------------------------------
# confidence measures without an exit head (Section 2.1): hidden states similarity (2), dedicated classifier (3)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("conf_mode,threshold", [(2, 0.65), (3, 0.62)])
def test_fp32_headless_measures_lockstep(conf_mode, threshold):
    cfg = TINY.with_(decode_steps=4, n_layers=6, conf_mode=conf_mode, threshold=threshold)
    stats = lockstep(cfg, seed=31, steps=4)
    assert stats["near_threshold"] == 0 and stats["near_tie"] == 0
    assert min(stats["L"]) < cfg.n_layers, stats["L"]          # the batch did leave early at least once


@pytest.mark.parametrize("batch", [7, 40])
@pytest.mark.parametrize("conf_mode,threshold", [(2, 0.78), (3, 0.55)])
def test_bf16_headless_measures_lockstep(conf_mode, threshold, batch):
    cfg = small_bf16(n_layers=6, batch=batch, prompt_len=12, min_prompt_len=4, shuffled_blocks=True,
                     conf_mode=conf_mode, threshold=threshold)
    stats = lockstep(cfg, seed=32, steps=5)
    total = stats["decisions"] + stats["tokens"]
    assert stats["near_threshold"] + stats["near_tie"] <= max(2, total // 20), stats
    assert stats["max_conf_err"] < 2e-2


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_similarity_with_checks_every_second_layer(dtype):
    """The previous hidden state is the one before layer i also where layer i-1 had no check."""
    base = TINY.with_(decode_steps=3) if dtype == "fp32" else small_bf16(batch=9)
    cfg = base.with_(n_layers=7, exit_every=2, conf_mode=2, threshold=0.7)
    lockstep(cfg, seed=33, steps=3)


@pytest.mark.parametrize("conf_mode", [2, 3])
def test_headless_measures_forced_exits(conf_mode):
    cfg = small_bf16(n_layers=6, conf_mode=conf_mode)
    g = torch.Generator().manual_seed(11)
    forced = torch.randint(1, cfg.n_layers + 1, (3, cfg.batch), generator=g, dtype=torch.int32)
    forced[1] = 1
    stats = lockstep(cfg, seed=34, steps=3, forced_seq=forced)
    assert stats["L"] == [int(forced[s].max()) for s in range(3)]


# ------------------------------------------------------------------------------------------------
# per-sequence exit (extension of Algorithm 1): every sequence leaves at its own layer
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("conf_mode,threshold", [(0, 0.8), (2, 0.65), (3, 0.62)])
def test_fp32_per_sequence_exit_lockstep(conf_mode, threshold):
    cfg = TINY.with_(decode_steps=4, n_layers=6, conf_mode=conf_mode, threshold=threshold)
    stats = lockstep(cfg, seed=31, steps=4, heads=2)
    assert stats["near_threshold"] == 0 and stats["near_tie"] == 0


@pytest.mark.parametrize("batch", [7, 40, 70])
@pytest.mark.parametrize("conf_mode,threshold", [(0, 0.5), (2, 0.78)])
def test_bf16_per_sequence_exit_lockstep(conf_mode, threshold, batch):
    cfg = small_bf16(n_layers=6, batch=batch, prompt_len=12, min_prompt_len=4, shuffled_blocks=True,
                     conf_mode=conf_mode, threshold=threshold)
    stats = lockstep(cfg, seed=41, steps=5, heads=2)
    total = stats["decisions"] + stats["tokens"]
    assert stats["near_threshold"] + stats["near_tie"] <= max(2, total // 20), stats


@pytest.mark.parametrize("cfg", [TINY.with_(n_layers=6, decode_steps=3), small_bf16(n_layers=6, batch=9)], ids=["fp32", "bf16"])
def test_per_sequence_forced_exits(cfg):
    """Mixed forced exit layers: sequences leave one by one; their K/V above their own exit layer is filled from
    their own hidden state (checked slot by slot against the oracle by the lock-step comparison)."""
    g = torch.Generator().manual_seed(19)
    forced = torch.randint(1, cfg.n_layers + 1, (4, cfg.batch), generator=g, dtype=torch.int32)
    forced[1] = 3                                  # everybody at layer 3: coincides with Algorithm 1
    forced[2] = cfg.n_layers                       # nobody leaves early
    forced[3, 0] = 1                               # one sequence leaves at once, the rest later
    stats = lockstep(cfg, seed=42, steps=4, forced_seq=forced, heads=2)
    assert stats["L"] == [int(forced[s].max()) for s in range(4)]


def compactable_bf16(**kw):
    """Widths at which every projection runs in the tiled kernel once the batch is a multiple of 128 rows: the
    per-sequence rule then compacts the rows that are still active."""
    return small_bf16(n_layers=6, d_ffn=384, prompt_len=10, min_prompt_len=3, shuffled_blocks=True, **kw)


@pytest.mark.parametrize("batch", [128, 256, 384])
@pytest.mark.parametrize("conf_mode,threshold", [(0, 0.5), (2, 0.78)])
def test_bf16_per_sequence_exit_compacted_rows_lockstep(conf_mode, threshold, batch):
    cfg = compactable_bf16(batch=batch, conf_mode=conf_mode, threshold=threshold)
    stats = lockstep(cfg, seed=43, steps=3, heads=2)
    total = stats["decisions"] + stats["tokens"]
    assert stats["near_threshold"] + stats["near_tie"] <= max(2, total // 20), stats


@pytest.mark.parametrize("batch", [385, 400, 481, 512])
@pytest.mark.parametrize("heads", [1, 2])
def test_bf16_385_to_512_rows_lockstep(batch, heads):
    """385 to 512 rows: LM head and gate/up run in the 256 x 256 ring kernel under Algorithm 1 (a second row block
    from one row to full), and stay in the tiled kernel with compacted rows under the per-sequence rule."""
    cfg = compactable_bf16(batch=batch)
    stats = lockstep(cfg, seed=46, steps=2, heads=heads)
    total = stats["decisions"] + stats["tokens"]
    assert stats["near_threshold"] + stats["near_tie"] <= max(2, total // 20), stats


@pytest.mark.parametrize("batch", [96, 150, 200])
@pytest.mark.parametrize("heads", [1, 2])
def test_bf16_row_counts_with_a_short_last_chunk(batch, heads):
    """Three, five and seven 32-row tiles: the tiled projection kernel pads its last 128-row chunk (and, under
    the per-sequence rule above 128 rows, compacts the active rows as well)."""
    cfg = compactable_bf16(batch=batch)
    stats = lockstep(cfg, seed=45, steps=3, heads=heads)
    total = stats["decisions"] + stats["tokens"]
    assert stats["near_threshold"] + stats["near_tie"] <= max(2, total // 20), stats


@pytest.mark.parametrize("exit_every", [1, 2])
def test_per_sequence_compaction_across_chunk_boundaries(exit_every):
    """Forced exits that take the number of active rows through 129, 128, 127, 1 and 0 (the projections work on
    128-row chunks), with the last sequence staying to the end or leaving one layer before it (KV filling of the
    last layer), and with checks after every second layer only (the row sums of sequences that have left move on
    through layers without a check)."""
    cfg = compactable_bf16(batch=256, exit_every=exit_every)
    n, Bsz = cfg.n_layers, cfg.batch
    forced = torch.full((3, Bsz), 4, dtype=torch.int32)
    forced[:, :127] = 1
    forced[:, 127] = 2
    forced[:, 128] = 3
    forced[0, 255] = n           # one sequence runs every layer
    forced[1, 255] = n - 1       # ... or leaves before the last layer, which is then filled
    forced[2] = torch.randint(1, n + 1, (Bsz,), generator=torch.Generator().manual_seed(5), dtype=torch.int32)
    stats = lockstep(cfg, seed=44, steps=3, forced_seq=forced, heads=2)
    want = [n, n - 1 if exit_every == 1 else n, int(forced[2].max())]
    if exit_every == 1:
        assert stats["L"] == want


@pytest.mark.parametrize("heads", [1, 2])
def test_batch_of_one_and_prompts_ending_on_block_boundaries(heads):
    """Degenerate sizes: a single sequence, and prompts whose next position opens a new 16-token block."""
    lockstep(small_bf16(batch=1, prompt_len=16, min_prompt_len=16, threshold=0.4), seed=61, steps=3, heads=heads)
    lockstep(small_bf16(batch=3, prompt_len=15, min_prompt_len=15, threshold=0.4), seed=62, steps=3, heads=heads)
    lockstep(TINY.with_(batch=1, prompt_len=31, min_prompt_len=31, decode_steps=3), seed=63, steps=3, heads=heads)


def test_sixty_four_layers_the_most_the_library_takes():
    """EE_MAX_LAYERS layers: the per-layer tables of the KV-filling launch are full; exits spread over the depth."""
    cfg = small_bf16(n_layers=64, d_model=128, n_heads=1, head_dim=128, d_ffn=128, vocab=256, batch=3, prompt_len=6,
                     min_prompt_len=6, weight_std=0.03, logit_scale=0.05, threshold=0.5)
    stats = lockstep(cfg, seed=71, steps=2, check_untouched=False)
    assert all(1 <= L <= 64 for L in stats["L"])
