"""The decode entry point that allocates nothing (its workspace is a static device array inside the library),
checked against wq_decode_attention on the same cache: two calls in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

from paper_2605_02262_amd import binding as W
from paper_2605_02262_amd import synth
from tests import wq_harness as H

pytestmark = pytest.mark.gpu


def _pair(cfg: int, splits: int):
    """(context-based output, static-scratch output, oracle output) of one configuration"""
    bt = synth.batch(synth.workload(cfg))
    w = bt.w
    g = H.run_gpu(bt, splits=splits)
    o = H.run_oracle(bt, scores_override=g.scores.cpu().numpy())
    q = H.to_dev(bt.q, w.dtype)
    max_tok = int(np.diff(bt.t.kv_off).max())
    sm = 1.0 / float(np.sqrt(w.hd))
    lse = torch.empty(w.B, w.Hq, dtype=torch.float32, device="cuda")
    got = W.wq_decode_attention_static(q, g.pk, sm, splits, max_tok, W.DECODE_AUTO, lse=lse)
    # the same summation order on both sides: every bit must agree
    fixed_ctx = W.wq_decode_attention(g.ctx, q, g.pk, sm, splits, max_tok, W.DECODE_AUTO | W.DECODE_FIXED_SHARES)
    fixed_static = W.wq_decode_attention_static(q, g.pk, sm, splits, max_tok, W.DECODE_AUTO | W.DECODE_FIXED_SHARES)
    torch.cuda.synchronize()
    return g, o, got, lse, fixed_ctx, fixed_static


def test_static_scratch_decode_matches_the_context_call_twice_in_a_row():
    # first call: the 0.5B-shaped layer (6400 tokens, 8 splits); second call: the tiny configuration (144 tokens, 2 splits),
    # which finds the scratch as the first call left it
    for cfg, splits in ((1, 8), (0, 2)):
        g, o, got, lse, fixed_ctx, fixed_static = _pair(cfg, splits)
        ref = g.out.cpu().numpy()
        err_ctx = H.attention_error(got.cpu().numpy(), ref.astype(np.float64))
        err_orc = H.attention_error(got.cpu().numpy(), o.out)
        assert err_ctx <= H.ATTN_TOL and err_orc <= H.ATTN_TOL, (cfg, err_ctx, err_orc)
        assert np.allclose(lse.cpu().numpy(), o.lse, rtol=0, atol=2e-3), cfg
        assert torch.equal(fixed_ctx, fixed_static), cfg


def test_static_scratch_rejects_what_does_not_fit():
    bt = synth.batch(synth.workload(0))
    g = H.run_gpu(bt, splits=2)
    q = H.to_dev(bt.q, bt.w.dtype)
    with pytest.raises(W.WQError) as e:      # 1024 splits of 14 heads x 66 floats fit; a faked batch of 60000 sequences does not
        g.pk.desc.B = 60000
        try:
            W.wq_decode_attention_static(q.expand(60000, -1, -1), g.pk, 0.125, 1024, 144, W.DECODE_AUTO)
        finally:
            g.pk.desc.B = bt.w.B
    assert e.value.code == -4 and "static array" in str(e.value)
