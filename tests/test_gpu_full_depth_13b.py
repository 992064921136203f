"""Parity at full depth and full size for the 13B-shaped configuration (40 layers, exit heads after layers 4, 8, .., 36,
batch 64 = one GPU's share of the 128 sequences, context 4096).  A file of its own so that the 7B-shaped weights of the
other full-depth cases are released before these 26 GB of weights and 210 GB of cache are allocated."""
import pytest
import torch

from paper_2407_20272_amd import workloads as W
from test_gpu_full_depth import SharedModel, one_iteration

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1200)]


@pytest.fixture(scope="module")
def model13b():
    m = SharedModel(W.CONFIGS[4], seed=5)
    yield m
    del m
    torch.cuda.empty_cache()



# ------------------------------------------------------------------------------------------------------
# config 4: 13B shape, 40 layers, exit heads after layers 4, 8, .., 36, batch 64 (one GPU's share), context 4096
# ------------------------------------------------------------------------------------------------------
def test_config4_full_depth_13b_heads_every_4th_layer(capsys, model13b):
    cfg = W.CONFIGS[4]
    L = one_iteration(capsys, model13b, cfg, seed=5, sample=[0, 63], what="config 4 (13B shape, threshold 0.95)")
    assert L in (4, 8, 12, 16, 20, 24, 28, 32, 36, 40)


def test_config4_full_depth_13b_forced_exit_between_heads(capsys, model13b):
    """Forced exit layers that fall between heads: a sequence leaves at the first head at or above its layer, the batch
    at the largest of those (28 here), and K/V of layers 29..40 is filled at the 13B width."""
    cfg = W.CONFIGS[4]
    forced = torch.tensor([5 + (b * 7) % 22 for b in range(cfg.batch)], dtype=torch.int32)     # 5..26 -> heads 8..28
    L = one_iteration(capsys, model13b, cfg, seed=6, sample=[1, 40], forced=forced, what="config 4 (13B shape, forced exits)")
    assert L == 28
