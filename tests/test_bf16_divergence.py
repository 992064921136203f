"""How far two CORRECT bf16 computations of the decode step drift apart with depth (CPU only, no GPU involved).

The float64 oracle and the same oracle with every projection accumulated in float32 round to bf16 at the same storage
points, so both satisfy the numerics contract.  They still disagree on which way individual values round, and a deep
random-weight model amplifies the disagreement.  What this measures is the floor under any tolerance between the
oracle and an implementation that accumulates in float32 (the GPU path does): the tolerances of the GPU parity tests
(tests/gpu_harness.py) cite these figures."""
import pytest
import torch

from oracle import ee_oracle as O
from paper_2407_20272_amd import workloads as W

F64 = torch.float64


class _F32Weight:
    """Stands in for a float64 weight matrix: `x @ w.T` is computed in float32 and handed back as float64."""

    def __init__(self, t):
        self.t = t.to(torch.float32)

    @property
    def T(self):
        return self

    def __rmatmul__(self, x):
        return (x.to(torch.float32) @ self.t.T).to(F64)


def drift(d, n_layers, batch, seed=3, ctx=64):
    """Per layer: (relative RMS, largest error scaled by the row maximum) of the hidden state and of this position's
    K/V, between the float64 oracle and its float32-accumulating copy.  One full-layer decode iteration."""
    cfg = W.reduced(W.CONFIGS[1], n_layers=n_layers, d_model=d, n_heads=d // 128, d_ffn=int(d * 2.6875) // 16 * 16,
                    vocab=512, batch=batch, prompt_len=ctx, min_prompt_len=ctx)
    w = W.make_weights(cfg, seed=seed)
    m = O.model_from_config(cfg, w)
    lens = W.make_context_lens(cfg)
    Ks, Vs = W.make_dense_kv(cfg, lens, ctx + 1, seed=seed, scale=0.3)
    tok = torch.randint(0, cfg.vocab, (batch,), generator=torch.Generator().manual_seed(1))

    def run(f32):
        cache = O.DenseKV.from_tensors(Ks, Vs, lens, "bf16")
        saved = O._w
        if f32:
            O._w = lambda m_, i, name: _F32Weight(m_.weights["layers"][i - 1][name])
        try:
            tr = {}
            O.decode_iteration(m, cache, tok, lens.long(), 2.0, heads=False, trace=tr)
        finally:
            O._w = saved
        return tr, cache

    (a, ca), (b, cb) = run(False), run(True)
    out = []
    for i in range(n_layers):
        ha, hb = a["h"][i], b["h"][i]
        h_max = float(((ha - hb).abs() / ha.abs().amax(-1, keepdim=True)).max())
        h_rms = float((ha - hb).pow(2).mean().sqrt() / ha.pow(2).mean().sqrt())
        kv_max = kv_rms = 0.0
        for ta, tb in ((ca.K[i], cb.K[i]), (ca.V[i], cb.V[i])):
            xa, xb = ta[:, ctx].to(F64).flatten(1), tb[:, ctx].to(F64).flatten(1)
            kv_max = max(kv_max, float(((xa - xb).abs() / xa.abs().amax(-1, keepdim=True)).max()))
            kv_rms = max(kv_rms, float((xa - xb).pow(2).mean().sqrt() / xa.pow(2).mean().sqrt()))
        out.append((h_rms, h_max, kv_rms, kv_max))
    return out


def test_two_correct_bf16_computations_drift_apart_with_depth():
    """Width 1024, 32 layers: the drift grows with depth, is far above float32 noise, and at 32 layers the element-wise
    figure is already of the order of the stated 2e-2 while the norm-wise one stays below it."""
    r = drift(1024, 32, 8)
    h_rms = [x[0] for x in r]
    assert h_rms[3] < h_rms[15] < h_rms[31]
    assert h_rms[0] > 1e-5                       # bf16 rounding disagreements, not float32 rounding
    assert 3e-3 < h_rms[31] < 2e-2 and 3e-3 < r[31][2] < 2e-2
    assert max(x[1] for x in r) < 4e-2 and max(x[3] for x in r) < 4e-2
    assert max(x[1] for x in r[:8]) < 2e-2 and max(x[3] for x in r[:8]) < 2e-2


@pytest.mark.timeout(600)
def test_drift_at_the_7b_width_bounds_what_a_parity_test_can_ask():
    """Width 4096 (the 7B shape), 32 layers, 4 sequences: after 16 layers the two computations are still within 2e-2
    element by element; after 32 the largest element-wise difference reaches the stated 2e-2 while the relative RMS
    difference is about 1.5e-2.  Hence: element-wise 2e-2 up to 16 layers, norm-wise (RMS <= 2e-2, no element beyond
    4e-2) above."""
    r = drift(4096, 32, 4)
    for i, (h_rms, h_max, kv_rms, kv_max) in enumerate(r):
        if i % 4 == 3:
            print(f"layer {i + 1:2d}: hidden rms {h_rms:.2e} max {h_max:.2e} | K/V rms {kv_rms:.2e} max {kv_max:.2e}")
    assert max(max(x[1], x[3]) for x in r[:16]) < 2e-2           # element-wise bound holds up to 16 layers
    assert max(max(x[0], x[2]) for x in r) < 2e-2                # norm-wise bound holds at every depth
    assert max(max(x[1], x[3]) for x in r) < 4e-2
    assert max(max(x[1], x[3]) for x in r[24:]) > 1.5e-2         # and the element-wise bound is about exhausted at 32
    assert r[31][0] > 1e-2
