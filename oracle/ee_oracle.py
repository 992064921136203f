"""CPU oracle for one iteration-level batched decode step of an early-exit decoder-only LLM.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file: it is called by the
tests, by the smoke check and by the benchmark's cpu_baseline leg.  It shares no code with the HIP
path and imports nothing from it.

What it follows.  The control flow is the paper's Algorithm 1 ("Iteration-level Batch Inference for
Early-exit LLMs") with the status rule of Section 3.1 and the cache filling of Section 3.2, applied
to a Llama-shaped decoder (RMSNorm, rotary positions, SwiGLU, untied or tied LM head) as the
benchmark definition fixes it.  Every step is written the plain way: no blocking, no fusion, no
reordering.  All arithmetic is float64.  For a bf16 workload the values that the decode step keeps
in bf16 storage are rounded to bf16 (round to nearest even) where they are stored:
  weights, embedding rows and cache contents (they arrive as bf16), the normalised input of every
  projection, the attention output, the SwiGLU product, and K/V when they enter the cache.
The residual stream, q, the scores, the softmax, the exit-head logits and the confidence are never
rounded.  For an fp32 workload nothing is rounded.

Readings taken where the paper is silent or inconsistent (each also listed in the design notes):
  * Status has one entry per sequence of the batch and starts False (Algorithm 1 prints "length n"
    and Section 3.1 once says "initially ... eligible"; the update rule only makes sense this way).
  * output_layer = n when the loop never breaks; the filling loop is then empty.
  * All tokens come from the batch's hidden state at output_layer, also for sequences whose own
    status turned true earlier.
  * compute_KV_pair(i, h) = what layer i's attention would cache for its input h:
    RMSNorm with layer i's attention gain, the K and V projections, rotary embedding on K.
  * confidence mode 0 = largest softmax probability (the benchmark definition); mode 1 = top-1 minus
    top-2 softmax probability (Section 2.1, softmax response).  Strict '>' against the threshold.
  * confidence mode 2 = cos(h_{i-1}, h_i) (Section 2.1, hidden states similarity): the hidden states
    after layers i-1 and i, h_0 being the embedding; taken on the float residual stream.
  * confidence mode 3 = M(h_i) (Section 2.1, dedicated classifier; the paper leaves M open), read as
    one linear unit per layer on the hidden state scaled to unit root mean square (no gain), followed
    by the logistic function: 1 / (1 + exp(-(w_i . h_i / sqrt(mean(h_i^2) + eps) + b_i))).  The scaling
    is what every other consumer of the residual stream in this model family applies; without it the
    unit's input grows with the norm of the residual stream, by orders of magnitude over the layers.
    Modes 2 and 3 never touch the LM head inside the loop; tokens still come from the hidden state at
    output_layer through transform_to_tokens, as Algorithm 1 says.
  * exit head = final RMSNorm gain + the LM head, logits multiplied by logit_scale * i (1-based i);
    no check after the last layer; ties in argmax go to the lowest index.

decode_iteration_freeze is an extension that the paper does not define (per-sequence exit instead of
the batch leaving together); its docstring states its rule.

Pins (tests/test_oracle_*.py): brute-force uncached causal forward, threshold > 1 equals the
head-less full-layer pass, forced exit on a saturated model leaves the cache identical to a full
pass, control logic against its three-line definition, closed forms of the confidence, rotary and
attention special cases against library routines.  The bf16 storage points listed above are pinned
by a second brute-force forward, from library routines, that rounds at exactly those points
(tests/test_oracle_bf16_contract.py): removing or adding any single rounding here fails it.  The 7B/13B-shaped token values themselves are
"parity unpinned" by anything external: no published value exists for them.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import torch

F64 = torch.float64


@dataclasses.dataclass
class OracleModel:
    """Model description + plain-layout weights ([out][in] matrices), any float dtype."""
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str            # "fp32" | "bf16": which storage rounding applies
    rms_eps: float
    rope_theta: float     # <= 0 disables the rotary embedding
    exit_every: int
    logit_scale: float
    conf_mode: int
    weights: Dict         # see paper_2407_20272_amd.workloads.make_weights for the keys


def store(x: torch.Tensor, dtype: str) -> torch.Tensor:
    """Value of x after it has been written to the workload's storage type and read back (float64)."""
    if dtype == "bf16":
        return x.to(torch.float32).to(torch.bfloat16).to(F64)
    return x.to(F64)


def rmsnorm(h: torch.Tensor, gain: torch.Tensor, eps: float) -> torch.Tensor:
    """Root-mean-square normalisation over the last axis, then the per-channel gain."""
    ms = (h * h).mean(dim=-1, keepdim=True)
    return h / torch.sqrt(ms + eps) * gain.to(F64)


def rope(x: torch.Tensor, pos: torch.Tensor, theta: float) -> torch.Tensor:
    """Rotary position embedding, split-half pairing: channel j is paired with j + dh/2 and the pair
    is rotated by the angle pos * theta^(-2j/dh).   x: [B][H][dh], pos: [B]."""
    if theta <= 0:
        return x
    dh = x.shape[-1]
    half = dh // 2
    j = torch.arange(half, dtype=F64)
    ang = pos.to(F64)[:, None] * theta ** (-2.0 * j / dh)[None, :]        # [B][half]
    c, s = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return torch.cat([a * c - b * s, b * c + a * s], dim=-1)


class DenseKV:
    """Per-layer dense caches K[i], V[i] of shape [B][max_ctx][H][dh] (layer index 1-based via k(i), v(i)).
    Contents are kept in the workload's storage dtype (torch.bfloat16 or torch.float64)."""

    def __init__(self, n_layers, batch, max_ctx, n_heads, head_dim, dtype: str):
        self.dtype = dtype
        t = torch.bfloat16 if dtype == "bf16" else F64
        self.K = [torch.zeros(batch, max_ctx, n_heads, head_dim, dtype=t) for _ in range(n_layers)]
        self.V = [torch.zeros(batch, max_ctx, n_heads, head_dim, dtype=t) for _ in range(n_layers)]
        self.written = [torch.zeros(batch, max_ctx, dtype=torch.bool) for _ in range(n_layers)]

    @classmethod
    def from_tensors(cls, Ks: List[torch.Tensor], Vs: List[torch.Tensor], context_lens, dtype: str):
        B, ctx, H, dh = Ks[0].shape
        c = cls(0, B, ctx, H, dh, dtype)
        t = torch.bfloat16 if dtype == "bf16" else F64
        c.K = [k.detach().cpu().to(t).clone() for k in Ks]
        c.V = [v.detach().cpu().to(t).clone() for v in Vs]
        valid = torch.arange(ctx)[None, :] < torch.as_tensor(context_lens).cpu()[:, None]
        c.written = [valid.clone() for _ in Ks]
        return c

    def put(self, i: int, b: int, pos: int, k: torch.Tensor, v: torch.Tensor):
        """KVCache.cache(i, K, V) of Algorithm 1 for one sequence and position."""
        self.K[i - 1][b, pos] = k.to(self.K[i - 1].dtype)
        self.V[i - 1][b, pos] = v.to(self.V[i - 1].dtype)
        self.written[i - 1][b, pos] = True


def _w(m: OracleModel, i: int, name: str) -> torch.Tensor:
    return m.weights["layers"][i - 1][name].to(F64)


def attention_decode(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor) -> torch.Tensor:
    """Single-query attention of one sequence: q [H][dh], K,V [T][H][dh] (all cached positions 0..p,
    the new token's own K/V included).  softmax(q.K^T / sqrt(dh)) . V per head -> [H][dh]."""
    dh = q.shape[-1]
    s = torch.einsum("hd,thd->ht", q, K.to(F64)) / math.sqrt(dh)
    p = torch.softmax(s, dim=-1)
    return torch.einsum("ht,thd->hd", p, V.to(F64))


def layer_forward(m: OracleModel, i: int, h: torch.Tensor, cache: DenseKV, pos: torch.Tensor) -> torch.Tensor:
    """M(i, hidden_states, KVCache) of Algorithm 1 without the exit check: one pre-norm decoder layer
    for one new token per sequence.  Caches this position's K/V of layer i on the way (Section 3.2:
    K/V are calculated and cached "in the process").   h: [B][d] -> [B][d]."""
    B = h.shape[0]
    H, dh, dt = m.n_heads, m.head_dim, m.dtype
    x = store(rmsnorm(h, m.weights["layers"][i - 1]["g_attn"], m.rms_eps), dt)
    q = (x @ _w(m, i, "w_q").T).reshape(B, H, dh)
    k = (x @ _w(m, i, "w_k").T).reshape(B, H, dh)
    v = (x @ _w(m, i, "w_v").T).reshape(B, H, dh)
    q = rope(q, pos, m.rope_theta)
    k = rope(k, pos, m.rope_theta)
    a = torch.empty(B, H, dh, dtype=F64)
    for b in range(B):
        p = int(pos[b])
        cache.put(i, b, p, store(k[b], dt), store(v[b], dt))
        a[b] = attention_decode(q[b], cache.K[i - 1][b, :p + 1], cache.V[i - 1][b, :p + 1])
    a = store(a.reshape(B, H * dh), dt)
    h = h + a @ _w(m, i, "w_o").T
    x = store(rmsnorm(h, m.weights["layers"][i - 1]["g_ffn"], m.rms_eps), dt)
    g = x @ _w(m, i, "w_gate").T
    u = x @ _w(m, i, "w_up").T
    act = store(g / (1.0 + torch.exp(-g)) * u, dt)
    return h + act @ _w(m, i, "w_down").T


def head_logits(m: OracleModel, h: torch.Tensor) -> torch.Tensor:
    """Unscaled LM-head logits of hidden rows h [R][d] -> [R][V]: final RMSNorm, then W_lm."""
    x = store(rmsnorm(h, m.weights["g_final"], m.rms_eps), m.dtype)
    return x @ m.weights["w_lm"].to(F64).T


def confidence(z: torch.Tensor, mode: int) -> torch.Tensor:
    """Confidence of each row of (already scaled) logits z [R][V].
    mode 0: largest softmax probability.  mode 1: top-1 minus top-2 softmax probability
    (the softmax-response measure of Section 2.1)."""
    p = torch.softmax(z, dim=-1)
    top = torch.topk(p, k=min(2, p.shape[-1]), dim=-1).values
    if mode == 0:
        return top[:, 0]
    second = top[:, 1] if top.shape[1] > 1 else torch.zeros_like(top[:, 0])
    return top[:, 0] - second


def similarity_confidence(h_prev: torch.Tensor, h: torch.Tensor) -> torch.Tensor:
    """Section 2.1, hidden states similarity: cos(h_{i-1}, h_i) per row of [R][d]."""
    a, b = h_prev.to(F64), h.to(F64)
    return (a * b).sum(dim=-1) / (a.pow(2).sum(dim=-1).sqrt() * b.pow(2).sum(dim=-1).sqrt())


def classifier_confidence(m: OracleModel, i: int, h: torch.Tensor) -> torch.Tensor:
    """Section 2.1, dedicated early-exit classifier M(h_i): logistic function of one linear unit per layer on
    the hidden state scaled to unit root mean square."""
    h = h.to(F64)
    x = h / torch.sqrt(h.pow(2).mean(dim=-1, keepdim=True) + m.rms_eps)
    t = x @ m.weights["w_cls"][i - 1].to(F64) + float(m.weights["b_cls"][i - 1])
    return 1.0 / (1.0 + torch.exp(-t))


def has_exit_head(m: OracleModel, i: int) -> bool:
    """Layers that carry an exit head: every exit_every-th layer, never the last one."""
    return i < m.n_layers and i % m.exit_every == 0


def exit_check(m: OracleModel, i: int, h: torch.Tensor, rows: List[int], h_prev: Optional[torch.Tensor] = None):
    """Confidence at layer i for the listed rows of h (and the exit head's arg max, where there is one).
    h_prev: the hidden state before layer i (only read by the similarity measure)."""
    if m.conf_mode == 2:
        return similarity_confidence(h_prev[rows], h[rows]), None
    if m.conf_mode == 3:
        return classifier_confidence(m, i, h[rows]), None
    z = head_logits(m, h[rows])
    return confidence((m.logit_scale * i) * z, m.conf_mode), torch.argmax(z, dim=-1)


def update_status(status: List[bool], exit_layer: List[int], i: int, conf: Dict[int, float], lam_i: float):
    """Section 3.1 status rule for layer i: a sequence whose status is False and whose confidence
    exceeds the threshold (strictly) becomes True and records i; a True status never reverts."""
    for b, c in conf.items():
        if not status[b] and c > lam_i:
            status[b] = True
            exit_layer[b] = i


def kv_fill(m: OracleModel, cache: DenseKV, h: torch.Tensor, pos: torch.Tensor, first_layer: int):
    """KV-cache filling loop of Algorithm 1 (Section 3.2): for every layer i >= first_layer compute
    this position's K and V from the exit hidden state h and cache them."""
    B, H, dh, dt = h.shape[0], m.n_heads, m.head_dim, m.dtype
    for i in range(first_layer, m.n_layers + 1):
        x = store(rmsnorm(h, m.weights["layers"][i - 1]["g_attn"], m.rms_eps), dt)
        k = rope((x @ _w(m, i, "w_k").T).reshape(B, H, dh), pos, m.rope_theta)
        v = (x @ _w(m, i, "w_v").T).reshape(B, H, dh)
        for b in range(B):
            cache.put(i, b, int(pos[b]), store(k[b], dt), store(v[b], dt))


def transform_to_tokens(m: OracleModel, h: torch.Tensor) -> torch.Tensor:
    """Greedy token per row: arg max of the LM-head logits, lowest index on ties."""
    z = head_logits(m, h)
    zmax = z.max(dim=-1, keepdim=True).values
    first = (z == zmax).to(torch.int64).argmax(dim=-1)          # first index attaining the max
    return first.to(torch.int32)


def decode_iteration(m: OracleModel, cache: DenseKV, tokens: torch.Tensor, pos: torch.Tensor,
                     thresholds, forced_exit_layer: Optional[torch.Tensor] = None, heads: bool = True,
                     trace: Optional[dict] = None):
    """One decode iteration (Algorithm 1).

    tokens [B] int: token each sequence consumes; pos [B] int: its position (= context length so far).
    thresholds: lambda_i for i = 1..n (sequence of n floats, or one float for all layers).
    forced_exit_layer [B] or None: synthetic confidence injection; the confidence of sequence b at
      layer i is replaced by +inf when i >= forced_exit_layer[b], -inf otherwise.
    heads=False: the full-layer baseline without any exit head.
    trace: optional dict that receives "h" (list of hidden states after each executed layer),
      "conf" ([n][B], NaN where not evaluated) and "h_exit".
    Returns (tokens [B] int32, exit_layer [B] int32, output_layer int).
    """
    n = m.n_layers
    B = int(tokens.shape[0])
    lam = [float(thresholds)] * n if isinstance(thresholds, (int, float)) else [float(t) for t in thresholds]
    h = store(m.weights["embed"][tokens.long()], m.dtype)                     # Embed(input_tokens)
    status = [False] * B
    exit_layer = [n] * B
    output_layer = n
    conf_log = torch.full((n, B), float("nan"), dtype=F64)
    if trace is not None:
        trace["h"] = []
    for i in range(1, n + 1):
        h_prev = h
        h = layer_forward(m, i, h, cache, pos)
        if trace is not None:
            trace["h"].append(h.clone())
        if heads and B > 0 and has_exit_head(m, i):
            rows = [b for b in range(B) if not status[b]]
            c, _ = exit_check(m, i, h, rows, h_prev)
            conf = {b: float(c[r]) for r, b in enumerate(rows)}
            for b in rows:
                conf_log[i - 1, b] = conf[b]
            if forced_exit_layer is not None:
                conf = {b: (math.inf if i >= int(forced_exit_layer[b]) else -math.inf) for b in rows}
            update_status(status, exit_layer, i, conf, lam[i - 1])
        if B > 0 and all(status):
            output_layer = i
            break
    kv_fill(m, cache, h, pos, output_layer + 1)
    out = transform_to_tokens(m, h) if B > 0 else torch.zeros(0, dtype=torch.int32)
    if trace is not None:
        trace["conf"] = conf_log
        trace["h_exit"] = h.clone()
    return out, torch.tensor(exit_layer, dtype=torch.int32), output_layer


def decode_iteration_freeze(m: OracleModel, cache: DenseKV, tokens: torch.Tensor, pos: torch.Tensor,
                            thresholds, forced_exit_layer: Optional[torch.Tensor] = None,
                            trace: Optional[dict] = None):
    """One decode iteration with PER-SEQUENCE early exit: an extension beyond Algorithm 1, which makes the
    whole batch leave together.  Same status rule (Section 3.1) and the same cache filling (Section 3.2), but
    applied to each sequence on its own:
      * a sequence whose status turns true at layer e_b stops there: layers e_b+1.. neither run for it nor
        cache K/V for it; it leaves the active set;
      * the loop ends after the first layer that leaves the active set empty (output_layer = max_b e_b),
        or after layer n;
      * K/V of this position for layers e_b+1..n are filled from the sequence's own hidden state at e_b;
      * its token comes from that same hidden state.
    A sequence never accepted has e_b = n and behaves as in a full-layer pass.  Every sequence's result is
    therefore what it would be in a batch of one.  Arguments and return value as decode_iteration
    (trace["h_exit"] holds each sequence's own exit hidden state; trace["h"][i-1] the batch's hidden states
    after layer i, a sequence that has left keeping its exit hidden state).
    """
    n = m.n_layers
    B = int(tokens.shape[0])
    lam = [float(thresholds)] * n if isinstance(thresholds, (int, float)) else [float(t) for t in thresholds]
    h = store(m.weights["embed"][tokens.long()], m.dtype).clone()
    status = [False] * B
    exit_layer = [n] * B
    output_layer = n
    conf_log = torch.full((n, B), float("nan"), dtype=F64)
    if trace is not None:
        trace["h"] = []
    for i in range(1, n + 1):
        active = [b for b in range(B) if not status[b]]
        if not active:
            break
        h_prev = h[active]
        h_new = layer_forward(m, i, h_prev, _RowView(cache, active), pos[active])
        if B > 0 and has_exit_head(m, i):
            full_prev, full_new = h.clone(), h.clone()
            full_new[active] = h_new
            c, _ = exit_check(m, i, full_new, active, full_prev)
            conf = {b: float(c[r]) for r, b in enumerate(active)}
            for b in active:
                conf_log[i - 1, b] = conf[b]
            if forced_exit_layer is not None:
                conf = {b: (math.inf if i >= int(forced_exit_layer[b]) else -math.inf) for b in active}
            update_status(status, exit_layer, i, conf, lam[i - 1])
        h[active] = h_new
        if trace is not None:
            trace["h"].append(h.clone())
        if B > 0 and all(status):
            output_layer = i
            break
    for e in sorted(set(exit_layer)):
        rows = [b for b in range(B) if exit_layer[b] == e]
        kv_fill(m, _RowView(cache, rows), h[rows], pos[rows], e + 1)
    out = transform_to_tokens(m, h) if B > 0 else torch.zeros(0, dtype=torch.int32)
    if trace is not None:
        trace["conf"] = conf_log
        trace["h_exit"] = h.clone()
    return out, torch.tensor(exit_layer, dtype=torch.int32), output_layer


def prefill(m: OracleModel, cache: DenseKV, prompts: torch.Tensor, lens: torch.Tensor,
            last_hidden: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Teacher-forced prompt pass through the decode step with no exit heads (full layers): position t
    of every sequence that is at least t+1 long.  Returns the first generated token of each sequence
    (the prediction after its last prompt token).  Sequences shorter than the longest simply stop early.
    last_hidden [B][d] float64, if given, receives the final hidden state each first token came from."""
    B, P = prompts.shape
    first = torch.zeros(B, dtype=torch.int32)
    for t in range(int(lens.max()) if B else 0):
        rows = [b for b in range(B) if int(lens[b]) > t]
        sub = _RowView(cache, rows)
        tr = {}
        tok, _, _ = decode_iteration(m, sub, prompts[rows, t], torch.full((len(rows),), t), 2.0, heads=False, trace=tr)
        for r, b in enumerate(rows):
            if int(lens[b]) == t + 1:
                first[b] = tok[r]
                if last_hidden is not None:
                    last_hidden[b] = tr["h_exit"][r]
    return first


class _RowView:
    """A DenseKV restricted to some sequences (used by the ragged prefill)."""

    def __init__(self, cache: DenseKV, rows: List[int]):
        self.cache, self.rows, self.dtype = cache, rows, cache.dtype
        self.K = [_Rows(k, rows) for k in cache.K]
        self.V = [_Rows(v, rows) for v in cache.V]

    def put(self, i, b, pos, k, v):
        self.cache.put(i, self.rows[b], pos, k, v)


class _Rows:
    def __init__(self, t, rows):
        self.t, self.rows = t, rows

    def __getitem__(self, idx):
        b, sl = idx
        return self.t[self.rows[b], sl]


def model_from_config(cfg, weights: Dict, **override) -> OracleModel:
    """Build the oracle's model record from a workload config (duck-typed: any object with the fields)."""
    kw = dict(n_layers=cfg.n_layers, d_model=cfg.d_model, n_heads=cfg.n_heads, head_dim=cfg.head_dim,
              d_ffn=cfg.d_ffn, vocab=cfg.vocab, dtype=cfg.dtype, rms_eps=cfg.rms_eps, rope_theta=cfg.rope_theta,
              exit_every=cfg.exit_every, logit_scale=cfg.logit_scale, conf_mode=cfg.conf_mode, weights=weights)
    kw.update(override)
    return OracleModel(**kw)
