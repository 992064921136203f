"""Seeded synthetic inputs for the early-exit decode step.

This module only *generates inputs*: model shapes, random weights, prompts,
context lengths, block tables, synthetic cache contents and forced exit layers.
It holds none of the method's arithmetic (no norm, projection, attention,
confidence or exit logic) and is imported by the tests, the benchmark and the
smoke check to hand identical bytes to the HIP path and to the CPU oracle.

The paper evaluates on news articles cut to 512 tokens with a fine-tuned
early-exit T5 (Evaluation, "Datasets"); neither is available here, so the
workloads below are synthetic stand-ins that keep the shapes: a ~512-token
context per sequence, a 32k-class vocabulary, exits possible after every layer.
"""
from __future__ import annotations

import dataclasses
import hashlib
import math
from typing import Dict, List

import torch


@dataclasses.dataclass(frozen=True)
class EEConfig:
    """Shape and exit rule of one synthetic early-exit decoder workload."""
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str                  # "fp32" or "bf16": storage type of weights, activations, KV
    exit_every: int             # exit head after layers i (1-based) with i % exit_every == 0, i < n_layers
    logit_scale: float          # exit-head logits at layer i are multiplied by logit_scale * i
    threshold: float            # lambda, same for every layer
    batch: int
    prompt_len: int             # context length before the first decode step (max over the batch)
    min_prompt_len: int         # ragged lower bound (== prompt_len when not ragged)
    decode_steps: int
    block_size: int = 16
    tied_head: bool = False     # LM head shares the embedding matrix
    shuffled_blocks: bool = False
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    # 0 = max softmax prob, 1 = top1 - top2 (softmax response as the paper writes it),
    # 2 = cosine similarity of consecutive hidden states, 3 = dedicated linear classifier (Section 2.1)
    conf_mode: int = 0
    weight_std: float = 0.02

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    def with_(self, **kw) -> "EEConfig":
        return dataclasses.replace(self, **kw)


def _llama7b(**kw) -> EEConfig:
    base = dict(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008, vocab=32000,
                dtype="bf16", exit_every=1, logit_scale=0.5, threshold=0.9)
    base.update(kw)
    return EEConfig(**base)


# The five workloads of the benchmark definition, in its order.  Index 3 is a family
# (batch x forced-exit mean); the entry here is its largest member that fits one GPU beside
# the others; `exit_sweep_configs()` lists the family.  Index 4 carries the one-GPU share
# (64 of the 128 sequences: the KV of all 128 at context 4160 is 436 GB and cannot fit 288 GB).
CONFIGS: List[EEConfig] = [
    EEConfig(name="tiny_fp32", n_layers=4, d_model=256, n_heads=4, head_dim=64, d_ffn=1024, vocab=2048,
             dtype="fp32", exit_every=1, logit_scale=4.0, threshold=0.8, batch=4, prompt_len=32,
             min_prompt_len=32, decode_steps=16, tied_head=True),
    _llama7b(name="llama7b_b32_ctx512", batch=32, prompt_len=512, min_prompt_len=512, decode_steps=128),
    _llama7b(name="llama7b_b256_ragged", batch=256, prompt_len=2048, min_prompt_len=128, decode_steps=64,
             shuffled_blocks=True),
    _llama7b(name="llama7b_exit_sweep", batch=256, prompt_len=1024, min_prompt_len=1024, decode_steps=32),
    EEConfig(name="llama13b_b64_ctx4096", n_layers=40, d_model=5120, n_heads=40, head_dim=128, d_ffn=13824,
             vocab=32000, dtype="bf16", exit_every=4, logit_scale=0.4, threshold=0.95, batch=64,
             prompt_len=4096, min_prompt_len=4096, decode_steps=64),
]


def exit_sweep_configs() -> List[EEConfig]:
    """Batch sizes of the exit-rate sweep.  Batch 512 at context 1024 needs 283 GB of KV, which
    does not fit beside 13.5 GB of weights, so that member runs at context 768."""
    out = []
    for b in (64, 256, 512):
        ctx = 1024 if b < 512 else 768
        out.append(CONFIGS[3].with_(name=f"llama7b_exit_sweep_b{b}", batch=b, prompt_len=ctx, min_prompt_len=ctx))
    return out


def reduced(cfg: EEConfig, **kw) -> EEConfig:
    """A smaller relative of `cfg` (fewer layers, narrower, shorter) for tests the oracle finishes in seconds."""
    return cfg.with_(name=cfg.name + "_reduced", **kw)


# ----------------------------------------------------------------------------------------------
# random streams: one independent torch generator per (seed, tensor name)
# ----------------------------------------------------------------------------------------------
def _gen(seed: int, name: str, device) -> torch.Generator:
    digest = hashlib.sha256(f"{seed}:{name}".encode()).digest()
    g = torch.Generator(device=device)
    g.manual_seed(int.from_bytes(digest[:8], "little") & 0x7FFFFFFFFFFFFFFF)
    return g


def _normal(shape, std, seed, name, device, dtype) -> torch.Tensor:
    x = torch.randn(shape, generator=_gen(seed, name, device), device=device, dtype=torch.float32)
    return x.mul_(std).to(dtype)


def make_weights(cfg: EEConfig, seed: int = 0, device="cpu", gain_jitter: float = 0.0) -> Dict:
    """Random-init weights in plain layouts.

    Every matrix is [out_features][in_features] row-major (y = x @ W^T), drawn N(0, weight_std^2) and
    stored in the config's dtype.  Norm gains are exactly 1 unless `gain_jitter` > 0 (tests use a
    jitter so that a dropped gain cannot pass).  Returns
      {"embed":[V,d], "g_final":[d], "w_lm":[V,d] (the same tensor as embed when tied),
       "layers":[{"g_attn":[d], "w_q","w_k","w_v","w_o":[d,d], "g_ffn":[d],
                  "w_gate","w_up":[f,d], "w_down":[d,f]} ...]}
    """
    dt = cfg.torch_dtype
    d, f, V = cfg.d_model, cfg.d_ffn, cfg.vocab
    std = cfg.weight_std

    def gain(name):
        g = torch.ones(d, device=device, dtype=torch.float32)
        if gain_jitter > 0:
            g += gain_jitter * torch.randn(d, generator=_gen(seed, name, device), device=device)
        return g.to(dt)

    w = {"embed": _normal((V, d), std, seed, "embed", device, dt), "g_final": gain("g_final")}
    w["w_lm"] = w["embed"] if cfg.tied_head else _normal((V, d), std, seed, "w_lm", device, dt)
    layers = []
    for i in range(1, cfg.n_layers + 1):
        layers.append({
            "g_attn": gain(f"l{i}.g_attn"),
            "w_q": _normal((d, d), std, seed, f"l{i}.w_q", device, dt),
            "w_k": _normal((d, d), std, seed, f"l{i}.w_k", device, dt),
            "w_v": _normal((d, d), std, seed, f"l{i}.w_v", device, dt),
            "w_o": _normal((d, d), std, seed, f"l{i}.w_o", device, dt),
            "g_ffn": gain(f"l{i}.g_ffn"),
            "w_gate": _normal((f, d), std, seed, f"l{i}.w_gate", device, dt),
            "w_up": _normal((f, d), std, seed, f"l{i}.w_up", device, dt),
            "w_down": _normal((d, f), std, seed, f"l{i}.w_down", device, dt),
        })
    w["layers"] = layers
    # Synthetic dedicated exit classifier (Section 2.1, third measure): one float32 weight row and one bias
    # per layer, applied to the hidden state at unit root mean square.  No trained classifier exists here:
    # rows are N(0, 1.5^2 / d), i.e. the unit's input has standard deviation 1.5 in every layer; the bias rises
    # linearly from -2 at layer 1 to +2 at layer n, so that deeper layers accept more often, as a trained one would.
    n = cfg.n_layers
    w["w_cls"] = _normal((n, d), 1.5 / d ** 0.5, seed, "w_cls", device, torch.float32)
    w["b_cls"] = torch.tensor([-2.0 + 4.0 * i / max(n - 1, 1) for i in range(n)], dtype=torch.float32, device=device)
    return w


def weights_to(w: Dict, device) -> Dict:
    """Copy a weight dict to another device, keeping the tied-head aliasing."""
    out = {"embed": w["embed"].to(device), "g_final": w["g_final"].to(device)}
    out["w_lm"] = out["embed"] if w["w_lm"] is w["embed"] else w["w_lm"].to(device)
    out["layers"] = [{k: v.to(device) for k, v in lw.items()} for lw in w["layers"]]
    for k in ("w_cls", "b_cls"):
        if k in w:
            out[k] = w[k].to(device)
    return out


def make_prompts(cfg: EEConfig, seed: int = 0, device="cpu") -> torch.Tensor:
    """Prompt token ids, uniform over the vocabulary: int32 [batch][prompt_len]."""
    return torch.randint(0, cfg.vocab, (cfg.batch, cfg.prompt_len), generator=_gen(seed, "prompt", "cpu"),
                         dtype=torch.int32).to(device)


def make_context_lens(cfg: EEConfig, seed: int = 0, device="cpu") -> torch.Tensor:
    """Per-sequence context length before the first decode step: uniform on [min_prompt_len, prompt_len]."""
    if cfg.min_prompt_len == cfg.prompt_len:
        return torch.full((cfg.batch,), cfg.prompt_len, dtype=torch.int32, device=device)
    return torch.randint(cfg.min_prompt_len, cfg.prompt_len + 1, (cfg.batch,),
                         generator=_gen(seed, "context_lens", "cpu"), dtype=torch.int32).to(device)


def blocks_needed(context_lens: torch.Tensor, extra_tokens: int, block_size: int) -> torch.Tensor:
    """Blocks each sequence needs to hold its context plus `extra_tokens` decoded positions."""
    return (context_lens.to(torch.int64) + extra_tokens + block_size - 1) // block_size


def make_block_tables(context_lens: torch.Tensor, extra_tokens: int, block_size: int, shuffled: bool,
                      seed: int = 0, spare_blocks: int = 0):
    """Caller-side block allocation.  Returns (block_tables int32 [B][max_blocks], num_blocks).

    Every sequence gets exactly the blocks it needs for context + extra_tokens positions; ids are
    consecutive, or a seeded random permutation of the pool when `shuffled`.  Unused table entries
    hold -1.  `spare_blocks` adds never-referenced blocks to the pool (tests check they stay untouched).
    """
    need = blocks_needed(context_lens.cpu(), extra_tokens, block_size)
    total = int(need.sum())
    num_blocks = total + spare_blocks
    ids = torch.randperm(num_blocks, generator=_gen(seed, "block_perm", "cpu")) if shuffled \
        else torch.arange(num_blocks)
    max_blocks = int(need.max()) if len(need) else 0
    table = torch.full((len(need), max_blocks), -1, dtype=torch.int32)
    at = 0
    for b, nb in enumerate(need.tolist()):
        table[b, :nb] = ids[at:at + nb].to(torch.int32)
        at += nb
    return table, num_blocks


def slot_of(block_tables: torch.Tensor, b: int, pos: int, block_size: int):
    """(physical block, offset in block) that holds position `pos` of sequence `b`."""
    return int(block_tables[b, pos // block_size]), pos % block_size


def make_dense_kv(cfg: EEConfig, context_lens: torch.Tensor, max_ctx: int, seed: int = 0, device="cpu",
                  scale: float = 1.0):
    """Synthetic cache contents for tests that skip the prefill: per layer a pair of dense tensors
    [B][max_ctx][H][dh] in the config dtype, N(0, scale^2) for positions < context_lens[b], zero elsewhere.
    Returns (K list, V list), one entry per layer."""
    B, H, dh = cfg.batch, cfg.n_heads, cfg.head_dim
    valid = (torch.arange(max_ctx, device=device)[None, :] < context_lens.to(device)[:, None])
    Ks, Vs = [], []
    for i in range(1, cfg.n_layers + 1):
        for name, dst in (("k", Ks), ("v", Vs)):
            t = _normal((B, max_ctx, H, dh), scale, seed, f"kv.l{i}.{name}", device, torch.float32)
            t = t * valid[:, :, None, None]
            dst.append(t.to(cfg.torch_dtype))
    return Ks, Vs


def dense_to_paged(dense: torch.Tensor, block_tables: torch.Tensor, num_blocks: int, block_size: int,
                   fill: float = 0.0) -> torch.Tensor:
    """Lay one layer's dense cache [B][ctx][H][dh] out as a pool [num_blocks][H][block_size][dh].
    Slots no sequence owns hold `fill`.  A pure re-layout: no arithmetic on the values."""
    B, ctx, H, dh = dense.shape
    pool = torch.full((num_blocks, H, block_size, dh), fill, dtype=dense.dtype, device=dense.device)
    nlog = (ctx + block_size - 1) // block_size
    pad = nlog * block_size - ctx
    x = torch.nn.functional.pad(dense, (0, 0, 0, 0, 0, pad)) if pad else dense
    x = x.reshape(B, nlog, block_size, H, dh).permute(0, 1, 3, 2, 4)       # [B][nlog][H][bs][dh]
    bt = block_tables[:, :nlog].to(dense.device).long()
    ok = bt >= 0
    pool[bt[ok]] = x[ok]
    return pool


def paged_to_dense(pool: torch.Tensor, block_tables: torch.Tensor, ctx: int) -> torch.Tensor:
    """Inverse of `dense_to_paged` for the table's blocks: [B][ctx][H][dh] (zeros where the table has -1)."""
    nb, H, bs, dh = pool.shape
    B, max_blocks = block_tables.shape
    nlog = min(max_blocks, (ctx + bs - 1) // bs)
    bt = block_tables[:, :nlog].to(pool.device).long()
    g = pool[bt.clamp(min=0)] * (bt >= 0)[:, :, None, None, None].to(pool.dtype)   # [B][nlog][H][bs][dh]
    g = g.permute(0, 1, 3, 2, 4).reshape(B, nlog * bs, H, dh)
    if g.shape[1] < ctx:
        g = torch.nn.functional.pad(g, (0, 0, 0, 0, 0, ctx - g.shape[1]))
    return g[:, :ctx].contiguous()


def truncated_geometric_ratio(mean: float, lo: int = 8, hi: int = 32) -> float:
    """Ratio r of P(e = k) ~ r^(k - lo), k = lo..hi, whose mean is `mean` (bisection on r)."""
    def m(r):
        ks = range(lo, hi + 1)
        ws = [r ** (k - lo) for k in ks]
        return sum(k * w for k, w in zip(ks, ws)) / sum(ws)
    a, b = 1e-3, 1e3
    for _ in range(200):
        c = math.sqrt(a * b)
        if m(c) < mean:
            a = c
        else:
            b = c
    return math.sqrt(a * b)


def make_forced_exit_layers(batch: int, steps: int, mean: float, lo: int = 8, hi: int = 32,
                            seed: int = 0) -> torch.Tensor:
    """Synthetic confidence injection: int32 [steps][batch] exit layers drawn independently from the
    truncated geometric distribution on [lo, hi] with the given mean."""
    r = truncated_geometric_ratio(mean, lo, hi)
    p = torch.tensor([r ** (k - lo) for k in range(lo, hi + 1)], dtype=torch.float64)
    idx = torch.multinomial(p / p.sum(), steps * batch, replacement=True,
                            generator=_gen(seed, f"forced_exit_{mean}", "cpu"))
    return (idx + lo).to(torch.int32).reshape(steps, batch)
