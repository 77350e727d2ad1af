"""Parity at the full sizes of the measured configurations, in the launch configuration bench.py times
(automatic split count, matrix-core decode kernel).  Needs an MI355X and about a minute of host time."""
import dataclasses

import numpy as np
import pytest

from paper_2605_02262_amd import synth

pytestmark = pytest.mark.gpu


def _full(bt, **kw):
    from tests import wq_harness as H
    g = H.run_gpu(bt, **kw)
    ov = kw.get("scores_override")
    o = H.run_oracle(bt, scores_override=ov if ov is not None else g.scores.cpu().numpy(),
                     with_scores=kw.get("with_scores", True), cap=kw.get("cap"), off16=kw.get("off16"))
    if g.scores is not None:
        H.assert_scores_close(g.scores, o.scores)
    assert np.array_equal(g.bits.cpu().numpy(), o.bits)
    assert np.array_equal(g.perm.cpu().numpy(), o.perm)
    assert np.array_equal(g.seg.cpu().numpy(), o.seg)
    H.assert_packed_equal(g, o)
    err = H.attention_error(g.out.cpu().numpy(), o.out)
    assert err <= H.ATTN_TOL, f"attention error {err:.3e}"
    assert g.ctx.device_status() == 0
    return g, o


def test_long_video_7b_layer_full():
    """4 x (256 frames x 196 + 512 text) tokens, 28/4 heads, head_dim 128, mix 26/102/128 windows at 8/4/2 bits."""
    bt = synth.batch(synth.workload(3))
    g, o = _full(bt)
    # the window counts the mix rule gives, and end-to-end agreement of bits derived from GPU and oracle scores
    assert o.seg[0].tolist() == [128, 102, 26, 0]
    from oracle import wq_oracle as O
    # end to end: the bits that follow from the oracle's own scores are the bits that follow from the GPU's scores.  That
    # is a theorem when every score gap across a tier boundary exceeds twice the tolerance the scores are held to, so the
    # seeded inputs must satisfy that, for every sequence (window 0 is pinned and leaves the ranking)
    bits2, _, _ = O.assign_bits(o.scores.astype(np.float32), bt.t.win_off, 0, quota=bt.t.quota, top_bits=8, pin_first=1)
    from tests import wq_harness as H
    gaps, tols = [], []
    for b in range(bt.w.B):
        sb = o.scores[bt.t.win_off[b]:bt.t.win_off[b + 1]]
        n_top, n4, _ = bt.t.quota[b]
        rest = np.sort(sb[1:])[::-1]
        gaps += [rest[n_top - 2] - rest[n_top - 1], rest[n_top + n4 - 2] - rest[n_top + n4 - 1]]
        tols.append(H.SCORE_ATOL + H.SCORE_RTOL * np.abs(sb).max())
    dev = float(np.abs(g.scores.cpu().numpy().astype(np.float64) - o.scores).max())
    print(f"smallest score gap across a tier boundary {min(gaps):.3e}, twice the score tolerance {2 * max(tols):.3e}, "
          f"largest GPU-oracle score difference {dev:.3e}")
    assert min(gaps) > 2 * max(tols), (min(gaps), 2 * max(tols))
    assert np.array_equal(bits2, o.bits)

    # the literal pairwise form on the matrix cores at this size (workgroups of 128 rows x 512 text columns)
    import torch
    from tests import wq_harness as H
    from paper_2605_02262_amd import binding as W
    w, t = bt.w, bt.t
    tv, tt, tw = int(t.vis_off[-1]), int(t.txt_off[-1]), int(t.win_off[-1])
    s_pair = W.wq_window_scores(g.ctx, H.to_dev(bt.E_v, w.dtype), H.to_dev(bt.E_t, w.dtype), H.i32(t.vis_off), H.i32(t.txt_off),
                                H.i32(t.win_size), H.i32(t.win_off), tv, tt, tw, algo=W.SCORE_PAIRWISE_MFMA)
    torch.cuda.synchronize()
    H.assert_scores_close(s_pair, o.scores)

    # the unfused variant of the operator-fusion ablation at this size: sequence 0 of the dequantized copy against the
    # textbook attention (fp64) over exactly those rows
    tot = [int(sum(o.pk.cls_len[c][b] for c in range(3)) + o.pk.len16[b]) for b in range(w.B)]
    off = np.concatenate([[0], np.cumsum(tot)]).astype(np.int32)
    dense = W.PackedKV(w.B, w.Hkv, w.hd, w.group, g.pk.dtype16, [0, 0, 0], off)
    W.wq_dequantize(g.ctx, g.pk, dense)
    out = W.wq_decode_attention(g.ctx, H.to_dev(bt.q, w.dtype), dense, 1.0 / float(np.sqrt(w.hd)), 0, max(tot))
    torch.cuda.synchronize()
    assert g.ctx.device_status() == 0 and dense.len16.cpu().numpy().tolist() == tot
    k0 = dense.k16[:tot[0]].float().cpu().numpy()
    v0 = dense.v16[:tot[0]].float().cpu().numpy()
    want = O.attention_dense(bt.q[0], k0, v0, 1.0 / np.sqrt(w.hd))
    assert H.attention_error(out[0].cpu().numpy()[None], want[None]) <= H.ATTN_TOL
    # the copy is rounded into bf16 (2^-8 relative per value): near, not equal to, the attention over the exact values
    dev = H.attention_error(out.cpu().numpy(), o.out)
    print(f"unfused (bf16 copy) vs exact dequantized values: {dev:.3e}")
    assert dev <= 0.1


@pytest.mark.parametrize("layer", [0, 27])
def test_7b_batch8_sampled_layers(layer):
    """8 x (64 frames x 196 + 256 text) tokens; layers 0 and 27 of 28 (each layer has its own seeded K, V, q)."""
    w = synth.workload(2)
    bt = synth.batch(w, layer=layer, with_embeddings=(layer == 0))
    _full(bt, with_scores=(layer == 0), scores_override=None if layer == 0 else
          np.random.default_rng(layer).standard_normal(int(bt.t.win_off[-1])).astype(np.float32))


def test_7b_batch8_decode_steps_in_one_call():
    """The decode loop's step at full size, as bench.py --decode-loop launches it (automatic split count, one launch that
    appends the generated token and attends): two steps on layer 13's cache, each against the oracle over the grown cache."""
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    from tests import wq_harness as H
    w = synth.workload(2)
    bt = synth.batch(w, layer=13, with_embeddings=False)
    cap, off16 = H.capacities(w, slack=2)
    g, o = _full(bt, with_scores=False, cap=cap, off16=off16,
                 scores_override=np.random.default_rng(13).standard_normal(int(bt.t.win_off[-1])).astype(np.float32))
    rng = np.random.default_rng(14)
    sm = 1.0 / float(np.sqrt(w.hd))
    max_tok = int(np.diff(bt.t.kv_off).max()) + 2
    for step in range(2):
        kn = synth.round_bf16(rng.standard_normal((w.B, w.Hkv, w.hd)).astype(np.float32))
        vn = synth.round_bf16(rng.standard_normal((w.B, w.Hkv, w.hd)).astype(np.float32))
        qn = synth.round_bf16(bt.q * (1.0 + 0.1 * rng.standard_normal(bt.q.shape).astype(np.float32)))
        out = W.wq_decode_append_attention(g.ctx, H.to_dev(qn, w.dtype), g.pk, H.to_dev(kn, w.dtype), H.to_dev(vn, w.dtype), sm, 0, max_tok)
        for b in range(w.B):
            r = int(o.pk.off16[b] + o.pk.len16[b])
            o.pk.k16[r], o.pk.v16[r] = kn[b], vn[b]
            o.pk.len16[b] += 1
        assert np.array_equal(g.pk.len16.cpu().numpy(), o.pk.len16)
        err = H.attention_error(out.cpu().numpy(), O.decode_attention(qn, o.pk, sm))
        assert err <= H.ATTN_TOL, f"step {step}: attention error {err:.3e}"
    assert g.ctx.device_status() == 0


def test_ragged_batch32():
    """32 sequences, 8..128 frames, windows of 98 or 196, Dirichlet bit mixes incl. all-2-bit and all-8-bit, at the
    configuration's own embedding width (3584)."""
    bt = synth.batch(synth.workload(4))
    assert bt.E_v.shape[1] == 3584
    g, o = _full(bt)
    assert o.seg[0, 0] == bt.t.win_off[1] and o.seg[1, 2] == bt.t.win_off[2] - bt.t.win_off[1]
    from tests import wq_harness as H
    dev = float(np.abs(g.scores.cpu().numpy().astype(np.float64) - o.scores).max())
    print(f"ragged batch at D = 3584: largest GPU-oracle score difference {dev:.3e} over scores up to {np.abs(o.scores).max():.3e}")


def test_paper_operating_point_16bit_top_tier():
    """The paper's own setting (Sec. 4.1 defaults, Sec. 4.3 token counts): batch 1, 100 frames, windows of 32 tokens,
    top tier (first window and the best-scoring one) kept 16-bit, 217 / 393 windows at 4 / 2 bits, 135 text tokens."""
    bt = synth.batch(synth.workload(5))
    g, o = _full(bt)
    assert o.seg[0].tolist() == [393, 217, 0, 2]
    assert int(o.pk.len16[0]) == 2 * 32 + 16 + 135            # 215 16-bit rows, the paper's count
    assert int(o.bits[0]) == 16                               # first window pinned (Sec. 3.2.2)
