"""Host logic of the scheduling harness that needs no GPU: the latency figures of a finished run."""
import pytest

from paper_2407_20272_amd import serving as S


def test_inner_token_latency_follows_the_papers_definition():
    """Evaluation, "Latency": decoding latency of a sequence = finish time - first-token time; inner-token latency =
    sum of the decoding latencies / total number of generated tokens (not the mean gap between tokens)."""
    a = S.Request(0, [1, 2, 3], 4, generated=[5, 6, 7, 8], token_times=[10.0, 10.5, 11.5, 12.0])      # 2.0 s over 4 tokens
    b = S.Request(1, [1], 2, generated=[9, 9], token_times=[20.0, 23.0])                               # 3.0 s over 2 tokens
    c = S.Request(2, [1], 1, generated=[4], token_times=[30.0])                                        # one token: no decoding time
    out = S.summary([a, b, c], wall=10.0, iterations={"prefill": 1, "decode": 4})
    assert out["generated_tokens"] == 7 and out["tokens_per_s"] == pytest.approx(0.7)
    assert out["inner_token_latency_ms"] == pytest.approx((2.0 + 3.0 + 0.0) / 7 * 1e3)
    gaps = sorted([0.5, 1.0, 0.5, 3.0])
    assert out["token_gap_ms"]["mean"] == pytest.approx(sum(gaps) / 4 * 1e3)
    assert out["token_gap_ms"]["p50"] == pytest.approx(gaps[2] * 1e3)
    assert S.summary([], wall=1.0, iterations={})["inner_token_latency_ms"] is None
