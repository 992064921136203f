"""The C-ABI library loads without a GPU, exports every symbol the header declares, and rejects bad
arguments on the host before anything is launched (no compute calls here)."""
import ctypes as C
import os
import re

import pytest

from paper_2407_20272_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "ee_decode.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ee_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = header_functions()
    assert set(names) == set(B.EXPORTS)
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n


def desc(**kw):
    d = dict(n_layers=4, d_model=256, n_heads=4, head_dim=64, d_ffn=1024, vocab=2048, dtype=B.EE_FP32, rms_eps=1e-5,
             rope_theta=1e4, exit_every=1, logit_scale=4.0, conf_mode=0)
    d.update(kw)
    return B.ee_model_desc(**d)


def test_workspace_sizes():
    L = B.lib()
    a = L.ee_workspace_bytes(C.byref(desc()), 4, 64)
    b = L.ee_workspace_bytes(C.byref(desc()), 8, 64)
    assert 0 < a < b and a % 256 == 0
    big = desc(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008, vocab=32000, dtype=B.EE_BF16)
    assert L.ee_workspace_bytes(C.byref(big), 32, 640) > 32 * 4096 * 4
    assert L.ee_workspace_bytes(C.byref(desc(head_dim=32, n_heads=8)), 4, 64) == 0      # unsupported head_dim
    assert "head_dim" in B.ee_last_error()
    assert L.ee_workspace_bytes(C.byref(desc(d_model=255)), 4, 64) == 0
    assert L.ee_workspace_bytes(None, 4, 64) == 0
    assert B.ee_packed_weight_bytes(64, 32) == 64 * 32 * 2
    # a workspace sized for B rows must serve every call with fewer rows (the serving harness sizes it once):
    # the size never shrinks as the batch grows, whichever kernels and layouts a batch size selects
    small_bf16 = desc(n_layers=3, d_model=256, n_heads=2, head_dim=128, d_ffn=384, vocab=1024, dtype=B.EE_BF16)
    for dsc in (desc(), small_bf16, big):
        sizes = [L.ee_workspace_bytes(C.byref(dsc), b, 64) for b in range(1, 600)]
        assert all(x > 0 for x in sizes)
        assert all(x <= y for x, y in zip(sizes, sizes[1:])), [i + 1 for i, (x, y) in enumerate(zip(sizes, sizes[1:])) if x > y]
    # bf16 path: the normalisation kernel holds a row of at most 8192 channels
    wide = desc(n_layers=2, d_model=16384, n_heads=128, head_dim=128, d_ffn=1024, vocab=512, dtype=B.EE_BF16)
    assert L.ee_workspace_bytes(C.byref(wide), 4, 64) == 0 and "8192" in B.ee_last_error()
    # the allocation-free exit check says what it needs, and refuses what its static array cannot hold
    small = L.ee_exit_check_noalloc_bytes(C.byref(big), 32)
    assert 0 < small <= B.EE_NOALLOC_SCRATCH_BYTES < L.ee_exit_check_noalloc_bytes(C.byref(big), 512)
    assert L.ee_exit_check_noalloc_bytes(None, 4) == 0


@pytest.mark.parametrize("bad,code", [
    (dict(n_layers=0), B.EE_ERR_INVALID_ARG),
    (dict(n_layers=65), B.EE_ERR_UNSUPPORTED),
    (dict(dtype=7), B.EE_ERR_INVALID_ARG),
    (dict(d_model=260), B.EE_ERR_SHAPE),
    (dict(exit_every=0), B.EE_ERR_INVALID_ARG),
    (dict(conf_mode=4), B.EE_ERR_INVALID_ARG),
    (dict(conf_mode=-1), B.EE_ERR_INVALID_ARG),
    (dict(logit_scale=-1.0), B.EE_ERR_INVALID_ARG),
])
def test_bad_descriptions_are_rejected(bad, code):
    L = B.lib()
    cache = B.ee_kv_cache(1, 1, 4, 16)
    batch = B.ee_batch(1, 1, 1, 1, 1, 1)
    rc = L.ee_paged_attention_decode(C.byref(desc(**bad)), C.byref(cache), 1, 1, C.byref(batch), 1, None, 0, None)
    assert rc == code, B.ee_last_error()


def test_bad_arguments_are_rejected_before_any_launch():
    L = B.lib()
    d = desc()
    layers = (B.ee_layer_weights * 4)(*[B.ee_layer_weights(1, 1, 1, 1, 1, 1) for _ in range(4)])
    model = B.ee_model(d, 1, 1, 1, layers)
    cache = B.ee_kv_cache(1, 1, 4, 16)
    batch = B.ee_batch(2, 1, 1, 1, 2, 17)
    th = (C.c_float * 4)(0.5, 0.5, 0.5, 0.5)

    def call(model=model, cache=cache, batch=batch, th=th, out=1, ws=256, ws_bytes=1 << 30):
        return L.ee_decode_iteration(C.byref(model) if model else None, C.byref(cache) if cache else None,
                                     C.byref(batch) if batch else None, th, None, 1, out, out, out, None, None, ws,
                                     ws_bytes, None)

    assert call(model=None) == B.EE_ERR_INVALID_ARG
    assert call(cache=None) == B.EE_ERR_INVALID_ARG
    assert call(batch=None) == B.EE_ERR_INVALID_ARG
    assert call(th=None) == B.EE_ERR_INVALID_ARG
    assert call(out=None) == B.EE_ERR_INVALID_ARG
    assert call(ws=None) == B.EE_ERR_WORKSPACE
    assert call(ws=264) == B.EE_ERR_WORKSPACE and "aligned" in B.ee_last_error()
    assert call(ws_bytes=16) == B.EE_ERR_WORKSPACE and "needed" in B.ee_last_error()
    assert call(cache=B.ee_kv_cache(1, 1, 4, 32)) == B.EE_ERR_UNSUPPORTED          # block size
    assert call(cache=B.ee_kv_cache(1, None, 4, 16)) == B.EE_ERR_INVALID_ARG
    assert call(batch=B.ee_batch(-1, 1, 1, 1, 2, 17)) == B.EE_ERR_INVALID_ARG
    assert call(batch=B.ee_batch(2, None, 1, 1, 2, 17)) == B.EE_ERR_INVALID_ARG
    assert call(batch=B.ee_batch(2, 1, 1, 1, 2, 40)) == B.EE_ERR_SHAPE               # max_context > max_blocks*16
    assert call(batch=B.ee_batch(0, None, None, None, 0, 0)) == B.EE_OK              # empty batch: a no-op
    bad_layers = (B.ee_layer_weights * 4)(*[B.ee_layer_weights(1, 1, None, 1, 1, 1) for _ in range(4)])
    assert call(model=B.ee_model(d, 1, 1, 1, bad_layers)) == B.EE_ERR_INVALID_ARG
    assert "layer 1" in B.ee_last_error()
    # measures without an exit head: the classifier needs its weights; the stand-alone check has no head to run
    assert call(model=B.ee_model(desc(conf_mode=3), 1, 1, 1, layers, None, None)) == B.EE_ERR_INVALID_ARG
    assert "w_cls" in B.ee_last_error()
    m2 = B.ee_model(desc(conf_mode=2), 1, 1, 1, layers)
    assert L.ee_exit_check(C.byref(m2), 1, 1, 2, 0.5, None, 1, 1, 1, 1, 1, None, None, 256, 1 << 30, None) == B.EE_ERR_UNSUPPORTED
    # several rows per sequence (prompt chunks) only without exit checks
    assert call(batch=B.ee_batch(2, 1, 1, 1, 2, 17, 1)) == B.EE_ERR_INVALID_ARG and "row_table" in B.ee_last_error()
    # the other entry points validate the same way
    assert L.ee_exit_check(C.byref(model), 9, 1, 2, 0.5, None, 1, 1, 1, 1, 1, None, None, 256, 1 << 30, None) == B.EE_ERR_INVALID_ARG
    assert L.ee_exit_check(C.byref(model), 1, None, 2, 0.5, None, 1, 1, 1, 1, 1, None, None, 256, 1 << 30, None) == B.EE_ERR_INVALID_ARG
    assert L.ee_exit_check(C.byref(model), 1, 1, 0, 0.5, None, 1, 1, 1, 1, 1, None, None, 256, 1 << 30, None) == B.EE_OK
    assert L.ee_kv_fill(C.byref(model), C.byref(cache), C.byref(batch), None, 1, 256, 1 << 30, None) == B.EE_ERR_INVALID_ARG
    assert L.ee_kv_fill(C.byref(model), C.byref(cache), C.byref(batch), 1, 1, 256, 8, None) == B.EE_ERR_WORKSPACE
    assert L.ee_paged_attention_decode(C.byref(d), C.byref(cache), 0, 1, C.byref(batch), 1, None, 0, None) == B.EE_ERR_INVALID_ARG
    assert L.ee_paged_attention_decode(C.byref(d), C.byref(cache), 1, None, C.byref(batch), 1, None, 0, None) == B.EE_ERR_INVALID_ARG
    wide = B.ee_batch(2, 1, 1, 1, 20000, 17)                                          # block table wider than the LDS copy
    assert L.ee_paged_attention_decode(C.byref(d), C.byref(cache), 1, 1, C.byref(wide), 1, None, 0, None) == B.EE_ERR_UNSUPPORTED
    assert "max_blocks" in B.ee_last_error()
    # the allocation-free variant validates like the one it mirrors, and checks the size limit on the host
    assert L.ee_exit_check_noalloc(C.byref(model), 9, 1, 2, 0.5, None, 1, 1, 1, 1, 1, None, None, None) == B.EE_ERR_INVALID_ARG
    assert L.ee_exit_check_noalloc(C.byref(m2), 1, 1, 2, 0.5, None, 1, 1, 1, 1, 1, None, None, None) == B.EE_ERR_UNSUPPORTED
    assert L.ee_exit_check_noalloc(C.byref(model), 1, 1, 0, 0.5, None, 1, 1, 1, 1, 1, None, None, None) == B.EE_OK
    big_model = B.ee_model(desc(vocab=1 << 20), 1, 1, 1, layers)
    assert L.ee_exit_check_noalloc(C.byref(big_model), 1, 1, 64, 0.5, None, 1, 1, 1, 1, 1, None, None, None) == B.EE_ERR_WORKSPACE
    assert "static array" in B.ee_last_error()
    # measurement helpers
    assert L.ee_calibration_read(None, 1 << 20, 1, 4, None) == B.EE_ERR_INVALID_ARG
    assert L.ee_calibration_read(16, 1024, 1, 4, None) == B.EE_ERR_INVALID_ARG          # too few bytes per workgroup
    assert L.ee_calibration_mfma(0, 10, 1, None) == B.EE_ERR_INVALID_ARG
    assert L.ee_calibration_intake(16, 1 << 30, 16, 1 << 20, 4, 7, 0, 1, None) == B.EE_ERR_INVALID_ARG    # 8, 16, 32 or 48 loads
    assert L.ee_calibration_intake(16, 1 << 30, 16, 3 << 20, 4, 8, 0, 1, None) == B.EE_ERR_INVALID_ARG    # common: a power of two
    assert L.ee_calibration_intake(16, 1 << 20, 16, 1 << 20, 256, 8, 0, 1, None) == B.EE_ERR_INVALID_ARG  # too little per wavefront
    assert L.ee_calibration_intake(16, 1 << 30, 16, 1 << 20, 24, 8, 1, 1, None) == B.EE_ERR_INVALID_ARG     # pairs: 16 | workgroups
    assert L.ee_calibration_mfma_tile(4, 3, 8, 1, None) == B.EE_ERR_INVALID_ARG       # odd step count
    assert L.ee_calibration_mfma_tile(4, 4, 5, 1, None) == B.EE_ERR_INVALID_ARG       # 0 or 8 fragment reads only
    assert L.ee_calibration_mfma_tile(4, 4, 8, None, None) == B.EE_ERR_INVALID_ARG
    assert L.ee_calibration_copy(None, 1, 4, None) == B.EE_ERR_INVALID_ARG
    assert L.ee_pack_weight(1, 33, 16, 0, 0, 1, None) == B.EE_ERR_SHAPE
    assert L.ee_pack_weight(1, 64, 16, 1, 24, 1, None) == B.EE_ERR_SHAPE
    assert L.ee_pack_weight(1, 64, 16, 9, 0, 1, None) == B.EE_ERR_INVALID_ARG
    assert L.ee_pack_weight(None, 64, 16, 0, 0, 1, None) == B.EE_ERR_INVALID_ARG


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(AssertionError):
        B._ptr(torch.zeros(4))
