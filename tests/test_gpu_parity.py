"""GPU-vs-oracle parity through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

from paper_2605_02262_amd import synth

pytestmark = pytest.mark.gpu


def _h():
    from tests import wq_harness as H
    return H


def _check(bt, H, **kw):
    g = H.run_gpu(bt, **kw)
    o = H.run_oracle(bt, scores_override=None if g.scores is None else g.scores.cpu().numpy(),
                     **{k: v for k, v in kw.items() if k in ("mode", "thresholds", "cap", "off16", "with_scores")})
    if g.scores is not None:
        H.assert_scores_close(g.scores, o.scores)
    assert np.array_equal(g.bits.cpu().numpy(), o.bits)
    assert np.array_equal(g.perm.cpu().numpy(), o.perm)
    assert np.array_equal(g.seg.cpu().numpy(), o.seg)
    H.assert_packed_equal(g, o)
    err = H.attention_error(g.out.cpu().numpy(), o.out)
    assert err <= H.ATTN_TOL, f"attention error {err:.3e}"
    lse_g, lse_o = g.lse.cpu().numpy().astype(np.float64), o.lse
    fin = np.isfinite(lse_o)
    assert np.abs(lse_g[fin] - lse_o[fin]).max(initial=0.0) <= 2e-3
    assert g.ctx.device_status() == 0
    return g, o, err


@pytest.mark.parametrize("algo", [1, 2], ids=["generic", "mfma"])
@pytest.mark.parametrize("cfg", [0, 1])
def test_configs_small(cfg, algo):
    H = _h()
    bt = synth.batch(synth.workload(cfg))
    for splits in (1, 3, 0):
        _check(bt, H, splits=splits, algo=algo)


def _custom(seed, hd, g, Hkv, rep, dtype, specs, top_bits=8, pin=1, D=64, sigma=1.0):
    w = synth.Workload(f"custom-{seed}", dtype, synth.BF16 if dtype == synth.BF16 else synth.F16, Hkv * rep, Hkv, hd, g,
                       D, sigma, specs, seed, top_bits=top_bits, pin_first=pin)
    return synth.batch(w)


@pytest.mark.parametrize("hd,g", [(64, 32), (64, 64), (128, 32), (128, 64), (128, 128)])
@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16, synth.F32])
def test_shapes_and_dtypes_ragged(hd, g, dtype):
    H = _h()
    specs = [synth.SeqSpec(5, 21, 15, 9, (2, 3, 2)),              # 105 tokens, S=15 -> 7 windows, no tail
             synth.SeqSpec(3, 10, 7, 0, (1, 1, 2), tail=3),       # tail of 5 (33 = 4*7+5), no text
             synth.SeqSpec(0, 10, 4, 5, (0, 0, 0)),               # no visual tokens at all
             synth.SeqSpec(9, 16, 16, 40, (3, 3, 3))]
    bt = _custom(100 + hd + g + dtype, hd, g, 2, 7, dtype, specs)
    _check(bt, H, splits=2)


def test_paper_tiers_threshold_mode_and_16bit_top():
    """The paper's own rule: thresholds, top tier kept 16-bit, first window pinned (Sec. 3.2.1-3.2.2)."""
    H = _h()
    specs = [synth.SeqSpec(12, 32, 32, 24, (0, 0, 0)), synth.SeqSpec(7, 32, 32, 8, (0, 0, 0))]
    bt = _custom(7, 128, 64, 4, 7, synth.BF16, specs, top_bits=16, pin=1, D=128)
    # thresholds straddling the score range so that all three tiers appear
    th = np.array([[0.004, 0.03], [0.0, 0.02]], dtype=np.float32)
    cap = [12 * 32 + 7 * 32] * 3
    off16 = np.array([0, 12 * 32 + 24, 12 * 32 + 24 + 7 * 32 + 8], dtype=np.int32)
    g, o, _ = _check(bt, H, mode=1, thresholds=th, cap=cap, off16=off16, splits=4)
    assert o.bits[0] == 16 and o.bits[12] == 16
    assert len(set(o.bits.tolist())) >= 2


def test_rep_variants_and_single_head():
    H = _h()
    for rep, Hkv in ((1, 3), (4, 2), (8, 1)):
        specs = [synth.SeqSpec(6, 20, 20, 11, (2, 2, 2))]
        bt = _custom(40 + rep, 128, 64, Hkv, rep, synth.BF16, specs)
        _check(bt, H, splits=2)


def test_all_one_class_and_capacity_overflow_flag():
    H = _h()
    from paper_2605_02262_amd import binding as W
    for quota in ((6, 0, 0), (0, 6, 0), (0, 0, 6)):
        specs = [synth.SeqSpec(6, 33, 33, 5, quota)]
        bt = _custom(50 + quota[0], 128, 64, 4, 7, synth.BF16, specs, pin=0)
        _check(bt, H, splits=2)
    # a class buffer that is too small: flagged on the device, nothing written out of bounds
    specs = [synth.SeqSpec(6, 33, 33, 5, (2, 2, 2))]
    bt = _custom(60, 128, 64, 4, 7, synth.BF16, specs, pin=0)
    g = H.run_gpu(bt, cap=[32, 96, 96], splits=1)
    assert g.ctx.device_status() & W.DEV_CLASS_OVERFLOW
    assert int(g.pk.cls_len[0][0]) == 0


def test_scores_only_larger_D():
    """Scores at the 7B embedding width on a ragged batch, against the fp64 oracle."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    specs = [synth.SeqSpec(3, 196, 196, 256, (1, 1, 1)), synth.SeqSpec(5, 196, 98, 100, (3, 3, 4))]
    w = synth.Workload("scores", synth.BF16, synth.BF16, 28, 4, 128, 64, 3584, 1.5, specs, 5)
    t = synth.tables(w)
    ets, evs = zip(*[synth.embeddings(w, b) for b in range(w.B)])
    Et, Ev = np.concatenate(ets), np.concatenate(evs)
    ctx = W.Context(W.workspace_bytes(w.B, 0, 0, 0, Ev.shape[0], Et.shape[0], w.D))
    s = W.wq_window_scores(ctx, H.to_dev(Ev, w.dtype), H.to_dev(Et, w.dtype), H.i32(t.vis_off), H.i32(t.txt_off),
                           H.i32(t.win_size), H.i32(t.win_off), Ev.shape[0], Et.shape[0], int(t.win_off[-1]))
    torch.cuda.synchronize()
    want = O.window_scores(Ev, Et, t.vis_off, t.txt_off, t.win_size, t.win_off, form="pooled")
    H.assert_scores_close(s, want)
    pair = O.window_scores(Ev[:196], Et[:256], [0, 196], [0, 256], [196], [0, 1], form="pairwise")
    assert abs(pair[0] - want[0]) < 1e-12


@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16])
def test_scores_pairwise_on_matrix_cores(dtype):
    """The literal pairwise form on the matrix cores against the fp64 oracle (pairwise form where it is affordable)."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    specs = [synth.SeqSpec(3, 70, 35, 150, (1, 1, 1)),             # 210 rows: tiles of 128 with a ragged tail, 150 text tokens
             synth.SeqSpec(0, 10, 4, 5, (0, 0, 0)),                # no visual rows
             synth.SeqSpec(2, 196, 98, 300, (1, 1, 2), tail=5),    # 397 rows, 300 text tokens: three column tiles
             synth.SeqSpec(2, 64, 64, 0, (1, 1, 0))]               # no text at all -> scores 0
    w = synth.Workload("pair", dtype, dtype, 28, 4, 128, 64, 896, 1.5, specs, 9)
    t = synth.tables(w)
    ets, evs = zip(*[synth.embeddings(w, b) for b in range(w.B)])
    Et, Ev = np.concatenate(ets), np.concatenate(evs)
    ctx = W.Context(W.workspace_bytes(w.B, 0, 0, 0, Ev.shape[0], Et.shape[0], w.D))
    args = (H.to_dev(Ev, dtype), H.to_dev(Et, dtype), H.i32(t.vis_off), H.i32(t.txt_off), H.i32(t.win_size), H.i32(t.win_off),
            Ev.shape[0], Et.shape[0], int(t.win_off[-1]))
    s_mfma = W.wq_window_scores(ctx, *args, algo=W.SCORE_PAIRWISE_MFMA)
    s_pool = W.wq_window_scores(ctx, *args, algo=W.SCORE_POOLED)
    torch.cuda.synchronize()
    want = O.window_scores(Ev, Et, t.vis_off, t.txt_off, t.win_size, t.win_off, form="pairwise")
    H.assert_scores_close(s_mfma, want)
    H.assert_scores_close(s_pool, want)


def test_scores_random_shapes_both_forms():
    """Seeded random batches through both scoring forms against the oracle's literal pairwise form: text lengths on both
    sides of the matrix-core kernel's tile and pass edges (16, 64, 128, 256, 512 columns; more than one pass), ragged rows."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    rng = np.random.default_rng(5)
    for it in range(16):
        dtype = [synth.BF16, synth.F16][rng.integers(2)]
        D = int(rng.choice([128, 256, 384, 640]))
        specs = []
        for _ in range(int(rng.integers(1, 5))):
            S, nw, tail = int(rng.integers(1, 50)), int(rng.integers(0, 20)), int(rng.integers(0, 5))
            nt = int(rng.choice([0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 511, 512, 513, 700, 1100]))
            specs.append(synth.SeqSpec(nw, S, S, nt, (0, 0, nw), tail=tail) if nw > 0 else synth.SeqSpec(0, 10, 4, max(nt, 1), (0, 0, 0)))
        w = synth.Workload(f"scores-random-{it}", dtype, dtype, 14, 2, 64, 32, D, 1.0, specs, 500 + it)
        t = synth.tables(w)
        if int(t.win_off[-1]) == 0:
            continue
        ets, evs = zip(*[synth.embeddings(w, b) for b in range(w.B)])
        Et, Ev = np.concatenate(ets), np.concatenate(evs)
        ctx = W.Context(W.workspace_bytes(w.B, 0, 0, 0, Ev.shape[0], Et.shape[0], w.D))
        args = (H.to_dev(Ev, dtype), H.to_dev(Et, dtype), H.i32(t.vis_off), H.i32(t.txt_off), H.i32(t.win_size), H.i32(t.win_off),
                Ev.shape[0], Et.shape[0], int(t.win_off[-1]))
        s_mfma = W.wq_window_scores(ctx, *args, algo=W.SCORE_PAIRWISE_MFMA)
        s_pool = W.wq_window_scores(ctx, *args, algo=W.SCORE_POOLED)
        torch.cuda.synchronize()
        want = O.window_scores(Ev, Et, t.vis_off, t.txt_off, t.win_size, t.win_off, form="pairwise")
        H.assert_scores_close(s_mfma, want)
        H.assert_scores_close(s_pool, want)


@pytest.mark.parametrize("case", ["112-row tiles", "128-row tiles", "96-row tiles"])
def test_scores_pairwise_runs_of_tiles_per_workgroup(case):
    """More row tiles than the chip has compute units: a workgroup of the matrix-core kernel then walks a contiguous run
    of tiles, handing the loads of a tile's first step over from the last step of the tile (or pass) before it, and a
    run ends where a sequence ends.  First case: four sequences whose text lengths take the kernel through its 128-,
    256- and 512-column tilings, one, two and three passes (three: the weights do not fit LDS at once), 112-row tiles,
    ragged ends.  Second case: a row count for which the host picks 128-row tiles, two passes.  Third case: 96-row tiles and
    an odd number of steps over D (the two LDS buffers change roles from one unit to the next).  Against the fp64 oracle's
    literal pairwise form."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    if case == "112-row tiles":
        specs = [synth.SeqSpec(600, 49, 49, 20, (1, 1, 1)),              # 29 400 rows, 20 text tokens
                 synth.SeqSpec(640, 64, 64, 700, (1, 1, 1), tail=7),     # 40 967 rows, two passes of 512 columns
                 synth.SeqSpec(100, 49, 49, 1100, (1, 1, 1)),            # 4 900 rows, three passes
                 synth.SeqSpec(60, 49, 49, 200, (1, 1, 1))]              # 2 940 rows, 256-column tiling
    elif case == "128-row tiles":
        specs = [synth.SeqSpec(625, 64, 64, 600, (1, 1, 1)),             # 40 000 rows
                 synth.SeqSpec(399, 64, 64, 530, (1, 1, 1))]             # 25 536 rows: 65 536 in all = 2 x 256 tiles of 128
    else:
        specs = [synth.SeqSpec(400, 50, 50, 600, (1, 1, 1)),             # 20 000 rows
                 synth.SeqSpec(260, 50, 50, 530, (1, 1, 1), tail=3)]     # 13 003 rows: 345 tiles of 96
    D = 384 if case == "96-row tiles" else 128
    w = synth.Workload("pair-runs", synth.BF16, synth.BF16, 28, 4, 128, 64, D, 1.5, specs, 21)
    t = synth.tables(w)
    ets, evs = zip(*[synth.embeddings(w, b) for b in range(w.B)])
    Et, Ev = np.concatenate(ets), np.concatenate(evs)
    ctx = W.Context(W.workspace_bytes(w.B, 0, 0, 0, Ev.shape[0], Et.shape[0], w.D))
    args = (H.to_dev(Ev, w.dtype), H.to_dev(Et, w.dtype), H.i32(t.vis_off), H.i32(t.txt_off), H.i32(t.win_size), H.i32(t.win_off),
            Ev.shape[0], Et.shape[0], int(t.win_off[-1]))
    s_mfma = W.wq_window_scores(ctx, *args, algo=W.SCORE_PAIRWISE_MFMA)
    torch.cuda.synchronize()
    want = O.window_scores(Ev, Et, t.vis_off, t.txt_off, t.win_size, t.win_off, form="pairwise")
    H.assert_scores_close(s_mfma, want)


def test_decode_fixed_shares_is_reproducible_and_agrees_with_block_pool():
    """WQ_DECODE_FIXED_SHARES: the same bits on every run; the default (blocks handed out as wavefronts get free)
    sums in a run-dependent order and agrees to rounding.  Both are checked against the oracle."""
    H = _h()
    from paper_2605_02262_amd import binding as W
    bt = synth.batch(synth.workload(1))
    fixed = W.DECODE_MFMA | W.DECODE_FIXED_SHARES
    g, o, _ = _check(bt, H, splits=3, algo=fixed)
    first = g.out.clone()
    for _ in range(3):
        g2 = H.run_gpu(bt, splits=3, algo=fixed)
        assert torch.equal(g2.out, first)
    g3, _, _ = _check(bt, H, splits=3, algo=W.DECODE_MFMA)
    assert H.attention_error(g3.out.cpu().numpy(), first.cpu().numpy().astype(np.float64)) <= H.ATTN_TOL


def test_batch_shared_configuration_by_vote_then_threshold_mode_end_to_end():
    """Sec. 3.2.3: thresholds from f1/f2 for a few layer similarities, widths by the threshold rule (16-bit top
    tier), one configuration per batch by majority vote, then the cache and decode attention on it."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    specs = [synth.SeqSpec(6, 32, 16, 9, (0, 0, 0)), synth.SeqSpec(6, 32, 16, 5, (0, 0, 0)),
             synth.SeqSpec(4, 32, 16, 7, (0, 0, 0)), synth.SeqSpec(6, 32, 16, 0, (0, 0, 0), tail=5),
             synth.SeqSpec(5, 32, 16, 3, (0, 0, 0))]
    bt = _custom(77, 128, 64, 2, 7, synth.BF16, specs, top_bits=16, pin=1)
    w, t = bt.w, bt.t
    sc = O.window_scores(bt.E_v, bt.E_t, t.vis_off, t.txt_off, t.win_size, t.win_off).astype(np.float32)
    # layer similarities -> thresholds; rescale them to the range of these synthetic scores so all three tiers occur
    lo, hi = W.wq_layer_thresholds([0.35, 0.6, 0.9], 2.0)
    qs = np.quantile(sc, [0.0, 1.0])
    for tl, th in zip(lo, hi):
        thr = np.tile(np.array([[qs[0] + tl * (qs[1] - qs[0]), qs[0] + th * (qs[1] - qs[0])]], np.float32), (w.B, 1))
        ctx = W.Context(W.workspace_bytes(w.B, w.Hq, w.hd, 4))
        win_off = H.i32(t.win_off)
        max_w = int(np.diff(t.win_off).max())
        bits, perm, seg = W.wq_assign_bits(ctx, torch.from_numpy(sc).cuda(), win_off, max_w, W.MODE_THRESHOLD, None,
                                           torch.from_numpy(thr).cuda(), 16, 1)
        vb, vp, vs = W.wq_vote_bits(ctx, bits, win_off, max_w)
        ob, op_, os_ = O.assign_bits(sc, t.win_off, 1, thresholds=thr, top_bits=16, pin_first=1)
        assert np.array_equal(bits.cpu().numpy(), ob)
        wb, wp, wseg = O.vote_bits(ob, t.win_off)
        assert np.array_equal(vb.cpu().numpy(), wb) and np.array_equal(vp.cpu().numpy(), wp)
        assert np.array_equal(vs.cpu().numpy(), wseg)
        # in place (bits_out aliasing bits_in) gives the same
        rc = W.lib().wq_vote_bits(ctx.handle, bits.data_ptr(), w.B, win_off.data_ptr(), max_w, bits.data_ptr(),
                                  perm.data_ptr(), seg.data_ptr())
        assert rc == 0
        torch.cuda.synchronize()
        assert np.array_equal(bits.cpu().numpy(), wb) and np.array_equal(perm.cpu().numpy(), wp)
        # the shared configuration through the rest of the path
        cap, off16 = [0, 0, 0], []
        for b, s in enumerate(w.seqs):
            for c in range(3):
                cap[c] += (int(wseg[b, c]) * s.win_size + 31) // 32 * 32
            off16.append(int(wseg[b, 3]) * s.win_size + (s.n_vis - s.n_win * s.win_size) + s.n_text + 8)
        off16 = np.concatenate([[0], np.cumsum(off16)]).astype(np.int32)
        cap = [max(c, 32) for c in cap]
        pk = W.PackedKV(w.B, w.Hkv, w.hd, w.group, torch.bfloat16, cap, off16, fill=0xA5)
        K, V = H.to_dev(bt.K, w.dtype), H.to_dev(bt.V, w.dtype)
        W.wq_reorder_quantize(ctx, K, V, H.i32(t.kv_off), H.i32(t.win_size), win_off, vp, vs, int(t.kv_off[-1]), pk)
        out = W.wq_decode_attention(ctx, H.to_dev(bt.q, w.dtype), pk, 1.0 / float(np.sqrt(w.hd)), 2, 300)
        torch.cuda.synchronize()
        opk = O.reorder_quantize(bt.K, bt.V, t.kv_off, t.win_size, t.win_off, wp, wseg, w.group, off16=off16[:-1], cap=cap,
                                 cap16=int(off16[-1]))
        ref = O.decode_attention(bt.q, opk, 1.0 / np.sqrt(w.hd))
        assert H.attention_error(out.cpu().numpy(), ref) <= H.ATTN_TOL
        assert ctx.device_status() == 0


def test_append_generated_tokens_then_decode():
    """Sec. 2.2 / Sec. 3.1: generated tokens are appended 16-bit at the end of the cache; every decode step attends
    over the quantized segments plus the grown 16-bit segment.  Three steps, then a full segment raises the flag."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    specs = [synth.SeqSpec(6, 21, 21, 9, (1, 3, 2)), synth.SeqSpec(4, 16, 16, 30, (1, 2, 1))]
    bt = _custom(31, 128, 64, 2, 7, synth.BF16, specs)
    w = bt.w
    cap, off16 = H.capacities(w, slack=3)
    g = H.run_gpu(bt, cap=cap, off16=off16, splits=2)
    o = H.run_oracle(bt, scores_override=g.scores.cpu().numpy(), cap=cap, off16=off16)
    H.assert_packed_equal(g, o)
    rng = np.random.default_rng(9)
    sm = 1.0 / float(np.sqrt(w.hd))
    for step in range(3):
        kn = synth.round_bf16(rng.standard_normal((w.B, w.Hkv, w.hd)).astype(np.float32))
        vn = synth.round_bf16(rng.standard_normal((w.B, w.Hkv, w.hd)).astype(np.float32))
        qn = synth.round_bf16(rng.standard_normal((w.B, w.Hq, w.hd)).astype(np.float32))
        W.wq_append_kv(g.ctx, H.to_dev(kn, w.dtype), H.to_dev(vn, w.dtype), g.pk)
        for b in range(w.B):                                   # the same append on the oracle's arrays
            r = int(o.pk.off16[b] + o.pk.len16[b])
            o.pk.k16[r], o.pk.v16[r] = kn[b], vn[b]
            o.pk.len16[b] += 1
        out = W.wq_decode_attention(g.ctx, H.to_dev(qn, w.dtype), g.pk, sm, 2, 400)
        torch.cuda.synchronize()
        assert np.array_equal(g.pk.len16.cpu().numpy(), o.pk.len16)
        ref = O.decode_attention(qn, o.pk, sm)
        assert H.attention_error(out.cpu().numpy(), ref) <= H.ATTN_TOL
    assert g.ctx.device_status() == 0
    kn = H.to_dev(np.zeros((w.B, w.Hkv, w.hd), np.float32), w.dtype)
    W.wq_append_kv(g.ctx, kn, kn, g.pk)                        # every segment had room for exactly three rows
    assert g.ctx.device_status() == 2
    assert np.array_equal(g.pk.len16.cpu().numpy(), o.pk.len16)


@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16])
def test_decode_step_in_one_call_equals_append_then_decode(dtype):
    """Sec. 2.2: a decode step appends the generated token and attends over the grown cache.  The one-call form must
    leave the same rows and row counts in the cache and give, with fixed shares, bit for bit the same attention as
    wq_append_kv followed by wq_decode_attention; both are also held to the oracle.  The last step finds one segment
    full: that sequence is attended without the new token and the flag is raised."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    specs = [synth.SeqSpec(6, 21, 21, 9, (1, 3, 2)), synth.SeqSpec(4, 16, 16, 30, (1, 2, 1)), synth.SeqSpec(5, 32, 20, 3, (1, 1, 3))]
    bt = _custom(33, 128, 64, 2, 7, dtype, specs)
    w = bt.w
    cap, off16 = H.capacities(w, slack=4)
    off16 = np.array(off16).copy()
    off16[2:] += 1                                              # one more row for sequence 1: sequence 0 and 2 fill up first
    g = H.run_gpu(bt, cap=cap, off16=off16, splits=3)
    o = H.run_oracle(bt, scores_override=g.scores.cpu().numpy(), cap=cap, off16=off16)
    H.assert_packed_equal(g, o)
    rnd = synth.round_bf16 if dtype == synth.BF16 else synth.round_f16
    rng = np.random.default_rng(10)
    sm = 1.0 / float(np.sqrt(w.hd))
    algo = W.DECODE_AUTO | W.DECODE_FIXED_SHARES
    for step in range(4):
        kn = rnd(rng.standard_normal((w.B, w.Hkv, w.hd)).astype(np.float32))
        vn = rnd(rng.standard_normal((w.B, w.Hkv, w.hd)).astype(np.float32))
        qn = rnd(rng.standard_normal((w.B, w.Hq, w.hd)).astype(np.float32))
        kd, vd, qd = H.to_dev(kn, w.dtype), H.to_dev(vn, w.dtype), H.to_dev(qn, w.dtype)
        saved = g.pk.k16.clone(), g.pk.v16.clone(), g.pk.len16.clone()
        W.wq_append_kv(g.ctx, kd, vd, g.pk)
        two = W.wq_decode_attention(g.ctx, qd, g.pk, sm, 3, 400, algo).clone()
        torch.cuda.synchronize()
        want = g.pk.k16.clone(), g.pk.v16.clone(), g.pk.len16.clone()
        st_two = g.ctx.device_status()
        for dst, src in zip((g.pk.k16, g.pk.v16, g.pk.len16), saved):
            dst.copy_(src)
        lse = torch.empty(w.B, w.Hq, dtype=torch.float32, device="cuda")
        one = W.wq_decode_append_attention(g.ctx, qd, g.pk, kd, vd, sm, 3, 400, algo, lse=lse)
        torch.cuda.synchronize()
        assert g.ctx.device_status() == st_two == (2 if step == 3 else 0)
        for got, exp in zip((g.pk.k16, g.pk.v16, g.pk.len16), want):
            assert torch.equal(got, exp)
        assert torch.equal(one, two)
        for b in range(w.B):                                   # the same append on the oracle's arrays
            r = int(o.pk.off16[b] + o.pk.len16[b])
            if r < off16[b + 1]:
                o.pk.k16[r], o.pk.v16[r] = kn[b], vn[b]
                o.pk.len16[b] += 1
        assert np.array_equal(g.pk.len16.cpu().numpy(), o.pk.len16)
        ref, ref_lse = O.decode_attention(qn, o.pk, sm, want_lse=True)
        assert H.attention_error(one.cpu().numpy(), ref) <= H.ATTN_TOL
        assert np.abs(lse.cpu().numpy() - ref_lse).max() <= 1e-3
        free = W.wq_decode_append_attention(g.ctx, qd, g.pk, kd, vd, sm, 2, 400) if step == 0 else None    # free shares, other split count
        if free is not None:
            torch.cuda.synchronize()
            for b in range(w.B):
                r = int(o.pk.off16[b] + o.pk.len16[b])
                o.pk.k16[r], o.pk.v16[r] = kn[b], vn[b]
                o.pk.len16[b] += 1
            assert np.array_equal(g.pk.len16.cpu().numpy(), o.pk.len16)
            assert H.attention_error(free.cpu().numpy(), O.decode_attention(qn, o.pk, sm)) <= H.ATTN_TOL


def test_decode_step_in_one_call_falls_back_to_two_launches():
    """The generic kernel and a query or new rows of another element type cannot append in the launch: the call then
    makes the two launches itself, with the same result."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    specs = [synth.SeqSpec(3, 16, 16, 5, (1, 1, 1)), synth.SeqSpec(4, 8, 8, 12, (1, 2, 1))]
    bt = _custom(34, 128, 64, 2, 4, synth.F16, specs)
    w = bt.w
    cap, off16 = H.capacities(w, slack=4)
    g = H.run_gpu(bt, cap=cap, off16=off16, splits=2)
    o = H.run_oracle(bt, scores_override=g.scores.cpu().numpy(), cap=cap, off16=off16)
    rng = np.random.default_rng(11)
    sm = 1.0 / float(np.sqrt(w.hd))
    for step, (algo, new_dt, q_dt) in enumerate([(W.DECODE_GENERIC, synth.F16, synth.F16), (W.DECODE_AUTO, synth.F32, synth.F16),
                                                 (W.DECODE_AUTO, synth.F16, synth.F32)]):
        kn = synth.round_f16(rng.standard_normal((w.B, w.Hkv, w.hd)).astype(np.float32))
        vn = synth.round_f16(rng.standard_normal((w.B, w.Hkv, w.hd)).astype(np.float32))
        qn = synth.round_f16(rng.standard_normal((w.B, w.Hq, w.hd)).astype(np.float32))
        out = W.wq_decode_append_attention(g.ctx, H.to_dev(qn, q_dt), g.pk, H.to_dev(kn, new_dt), H.to_dev(vn, new_dt), sm, 2, 400, algo)
        torch.cuda.synchronize()
        for b in range(w.B):
            r = int(o.pk.off16[b] + o.pk.len16[b])
            o.pk.k16[r], o.pk.v16[r] = kn[b], vn[b]
            o.pk.len16[b] += 1
        assert np.array_equal(g.pk.len16.cpu().numpy(), o.pk.len16)
        assert H.attention_error(out.cpu().numpy(), O.decode_attention(qn, o.pk, sm)) <= H.ATTN_TOL
    assert g.ctx.device_status() == 0


def test_decode_step_in_a_hip_graph_replays_like_eager():
    """A decode step of two layers (the one-call form: one launch per layer, which also resets its arrival counters for
    the next replay) captured in one HIP graph: every replay (with eager work and synchronisation in between) gives
    what append and decode give when launched one by one on an identical second cache."""
    H = _h()
    from paper_2605_02262_amd import binding as W
    specs = [synth.SeqSpec(6, 21, 21, 9, (1, 3, 2)), synth.SeqSpec(4, 16, 16, 30, (1, 2, 1))]
    bt = _custom(41, 128, 64, 2, 7, synth.BF16, specs)
    w = bt.w
    cap, off16 = H.capacities(w, slack=6)
    algo = W.DECODE_MFMA | W.DECODE_FIXED_SHARES
    runs = [[H.run_gpu(bt, cap=cap, off16=off16, splits=2, algo=algo) for _ in range(2)] for _ in range(2)]   # [eager|graph][layer]
    rng = np.random.default_rng(3)
    mk = lambda *s: H.to_dev(synth.round_bf16(rng.standard_normal(s).astype(np.float32)), w.dtype)
    kn, vn, qn = [mk(w.B, w.Hkv, w.hd) for _ in range(2)], [mk(w.B, w.Hkv, w.hd) for _ in range(2)], [mk(w.B, w.Hq, w.hd) for _ in range(2)]
    sm = 1.0 / float(np.sqrt(w.hd))
    outs = [[torch.zeros(w.B, w.Hq, w.hd, device="cuda") for _ in range(2)] for _ in range(2)]

    def step(which):
        for layer in range(2):
            g = runs[which][layer]
            if which == 1:
                W.wq_decode_append_attention(g.ctx, qn[layer], g.pk, kn[layer], vn[layer], sm, 2, 400, algo, out=outs[which][layer])
                continue
            W.wq_append_kv(g.ctx, kn[layer], vn[layer], g.pk)
            W.wq_decode_attention(g.ctx, qn[layer], g.pk, sm, 2, 400, algo, out=outs[which][layer])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    for g in runs[1]:
        g.ctx.set_stream(side)
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(1)
    for rep in range(4):
        step(0)                                   # eager, on the default stream
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph.replay()
        torch.cuda.synchronize()
        for layer in range(2):
            assert torch.equal(outs[0][layer], outs[1][layer]), f"replay {rep}, layer {layer}"
            assert torch.equal(runs[0][layer].pk.len16, runs[1][layer].pk.len16)
            assert torch.equal(runs[0][layer].pk.k16, runs[1][layer].pk.k16) and torch.equal(runs[0][layer].pk.v16, runs[1][layer].pk.v16)
        assert float(outs[1][0].abs().max()) > 0
    assert runs[1][0].ctx.device_status() == 0


def _dense_expected(o, dtype16):
    """Per sequence: the values m + s*code of the oracle's logical codes (fp64, the format's definition written out) in
    cache order [2-bit | 4-bit | 8-bit], then the oracle's 16-bit rows.  Returns (K, V) lists of [rows, Hkv, hd]."""
    pk = o.pk
    G = pk.hd // pk.group
    Ks, Vs = [], []
    for b in range(pk.B):
        parts = [[], []]
        for c in range(3):
            a, n = int(pk.cls_off[c][b]), int(pk.cls_len[c][b])
            for pl in range(2):
                code = pk.codes[c][pl, :, a:a + n, :].astype(np.float64)                       # [Hkv, n, hd]
                s = pk.sbits[c][pl, :, a:a + n, :].astype(np.uint16).view(np.float16).astype(np.float64)
                m = pk.mbits[c][pl, :, a:a + n, :].astype(np.uint16).view(np.float16).astype(np.float64)
                val = np.repeat(m, pk.group, axis=-1) + np.repeat(s, pk.group, axis=-1) * code
                parts[pl].append(np.transpose(val, (1, 0, 2)))                                   # [n, Hkv, hd]
        a, n = int(pk.off16[b]), int(pk.len16[b])
        parts[0].append(pk.k16[a:a + n].astype(np.float64))
        parts[1].append(pk.v16[a:a + n].astype(np.float64))
        Ks.append(np.concatenate(parts[0]))
        Vs.append(np.concatenate(parts[1]))
    return Ks, Vs


def _check_dense(g_run, o, bt, H, splits=2):
    """wq_dequantize of a finished GPU run into a dense 16-bit copy: tables, every value against m + s*code, attention
    over the copy against the textbook attention (fp64) over exactly the rows that were written."""
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    w = bt.w
    pk = g_run.pk
    totals = [int(sum(o.pk.cls_len[c][b] for c in range(3)) + o.pk.len16[b]) for b in range(w.B)]
    off = np.concatenate([[0], np.cumsum([n + 3 for n in totals])]).astype(np.int32)      # a little slack per sequence
    dense = W.PackedKV(w.B, w.Hkv, w.hd, w.group, pk.dtype16, [0, 0, 0], off, fill=0xA5)
    W.wq_dequantize(g_run.ctx, pk, dense)
    q = H.to_dev(bt.q, w.dtype)
    out = W.wq_decode_attention(g_run.ctx, q, dense, 1.0 / float(np.sqrt(w.hd)), splits, max(totals + [1]))
    torch.cuda.synchronize()
    assert g_run.ctx.device_status() == 0
    assert np.array_equal(dense.len16.cpu().numpy(), np.asarray(totals, np.int32))
    for c in range(3):
        assert int(dense.cls_len[c].abs().sum().item()) == 0 and int(dense.cls_off[c].abs().sum().item()) == 0
    Ks, Vs = _dense_expected(o, w.dtype16)
    half_ulp = 2.0 ** -8 if w.dtype16 == synth.BF16 else 2.0 ** -11
    k16, v16 = dense.k16.float().cpu().numpy().astype(np.float64), dense.v16.float().cpu().numpy().astype(np.float64)
    for b in range(w.B):
        a, n = int(off[b]), totals[b]
        for got, want in ((k16[a:a + n], Ks[b]), (v16[a:a + n], Vs[b])):
            assert got.shape == want.shape
            assert np.all(np.abs(got - want) <= half_ulp * np.abs(want) * 1.0001 + 2.0 ** -25), "dequantized value off by more than one rounding"
    # The dense copy holds the values rounded into the 16-bit type (2^-8 relative for bf16), so its attention differs
    # from the attention over the exact values m + s*code by more than the fused kernel's error: a sanity bound only.
    assert H.attention_error(out.cpu().numpy(), o.out) <= 5e-2
    # The bar proper: the textbook attention (fp64) over exactly the rows that were written.
    for b in range(w.B):
        a, n = int(off[b]), totals[b]
        if n == 0:
            continue
        want = O.attention_dense(bt.q[b], k16[a:a + n].astype(np.float32), v16[a:a + n].astype(np.float32), 1.0 / np.sqrt(w.hd))
        assert H.attention_error(out[b].cpu().numpy()[None], want[None]) <= H.ATTN_TOL


@pytest.mark.parametrize("dtype,hd,g", [(synth.BF16, 128, 64), (synth.F16, 64, 32)])
def test_unfused_ablation_dequantize_to_memory_then_16bit_attention(dtype, hd, g):
    """wq_dequantize (the unfused variant of the operator-fusion ablation, Sec. 3.3.3 and Sec. 4.4): every dequantized value is the
    format's m + s*code rounded once into the 16-bit type; decode attention over the dense copy agrees with the fp64
    textbook attention over those rows."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    specs = [synth.SeqSpec(9, 21, 21, 13, (2, 3, 4)),             # 189 tokens: blocks of 32 with ragged ends in every class
             synth.SeqSpec(4, 16, 16, 40, (1, 1, 2)),
             synth.SeqSpec(0, 10, 4, 5, (0, 0, 0)),               # text only
             synth.SeqSpec(6, 32, 32, 0, (2, 2, 2), tail=7)]      # video tail, no text
    bt = _custom(321 + hd, hd, g, 2, 7, dtype, specs)
    w, t = bt.w, bt.t
    g_run, o, _ = _check(bt, H, splits=2)
    _check_dense(g_run, o, bt, H)


def test_dequantize_reports_a_destination_that_is_too_small():
    H = _h()
    from paper_2605_02262_amd import binding as W
    bt = synth.batch(synth.workload(0))
    g_run = H.run_gpu(bt)
    w = bt.w
    small = W.PackedKV(w.B, w.Hkv, w.hd, w.group, g_run.pk.dtype16, [0, 0, 0], np.array([0, 40], np.int32), fill=0x11)
    W.wq_dequantize(g_run.ctx, g_run.pk, small)
    torch.cuda.synchronize()
    assert g_run.ctx.device_status() == W.DEV_SEG16_OVERFLOW
    assert int(small.len16.sum().item()) == 0
    assert int((small.k16.view(torch.int16) != 0).sum().item()) == 0 and int((small.v16.view(torch.int16) != 0).sum().item()) == 0   # nothing was written


@pytest.mark.parametrize("seed", [7, 2024])
def test_random_ragged_workloads(seed):
    """Seeded random batches: 1-5 sequences, windows of 3-69 tokens, 0-13 windows, tails, text of 0-59 tokens, any shape,
    dtype, quota split (also quotas that leave windows over, and pins with a zero top quota), split count and kernel."""
    H = _h()
    from paper_2605_02262_amd import binding as W
    rng = np.random.default_rng(seed)
    worst = 0.0
    for it in range(25):
        hd, g = [(64, 32), (64, 64), (128, 32), (128, 64), (128, 128)][rng.integers(5)]
        dtype = [synth.BF16, synth.F16, synth.F32][rng.integers(3)]
        specs = []
        for _ in range(int(rng.integers(1, 6))):
            S, nw, nt, tail = int(rng.integers(3, 70)), int(rng.integers(0, 14)), int(rng.integers(0, 60)), int(rng.integers(0, 5))
            a = int(rng.integers(0, nw + 1))
            c = int(rng.integers(0, nw - a + 1))
            specs.append(synth.SeqSpec(nw, S, S, nt, (a, c, nw - a - c), tail=tail) if nw > 0 else
                         synth.SeqSpec(0, 10, 4, max(nt, 1), (0, 0, 0)))
        top = 16 if rng.integers(4) == 0 else 8
        w = synth.Workload(f"random-{seed}-{it}", dtype, synth.BF16 if dtype == synth.BF16 else synth.F16, 2 * int(rng.integers(1, 8)), 2,
                           hd, g, 64, 1.0, specs, 1000 * seed + it, top_bits=top, pin_first=int(rng.integers(2)))
        bt = synth.batch(w)
        kw = dict(splits=int(rng.integers(0, 5)),
                  algo=[W.DECODE_AUTO, W.DECODE_GENERIC, W.DECODE_MFMA][rng.integers(3)] if hd // g == 2 else W.DECODE_AUTO)
        if top == 16:       # any window may end up in any class or in the 16-bit segment
            kw["cap"] = [sum((s.n_win * s.win_size + 31) // 32 * 32 for s in w.seqs)] * 3
            kw["off16"] = np.concatenate([[0], np.cumsum([s.n_vis + s.n_text + 4 for s in w.seqs])]).astype(np.int32)
        g_run, o, err = _check(bt, H, **kw)
        worst = max(worst, err)
        if it % 3 == 0:
            _check_dense(g_run, o, bt, H, splits=kw["splits"])
    assert worst <= H.ATTN_TOL


@pytest.mark.parametrize("hd,g", [(128, 64), (64, 32)])
def test_extreme_split_counts(hd, g):
    """Split counts from 1 to the largest allowed (1024: most workgroups get no block at all; beyond 64 splits the
    separate merge kernel takes over from the in-kernel merge), with and without fixed shares."""
    H = _h()
    from paper_2605_02262_amd import binding as W
    specs = [synth.SeqSpec(40, 50, 50, 70, (6, 14, 20)), synth.SeqSpec(3, 64, 64, 5, (1, 1, 1))]
    bt = _custom(55, hd, g, 2, 7, synth.BF16, specs)
    w = bt.w
    g_run, o, err = _check(bt, H, splits=1)
    q = H.to_dev(bt.q, w.dtype)
    sm = 1.0 / float(np.sqrt(w.hd))
    big = W.Context(W.workspace_bytes(w.B, w.Hq, w.hd, 1024))
    for splits in (2, 37, 64, 65, 300, 585, 586, 1024):     # (up to 64 the kernel merges its splits itself)
        for algo in (W.DECODE_AUTO, W.DECODE_AUTO | W.DECODE_FIXED_SHARES):
            lse = torch.empty(w.B, w.Hq, dtype=torch.float32, device="cuda")
            out = W.wq_decode_attention(big, q, g_run.pk, sm, splits, 2100, algo, lse=lse)
            torch.cuda.synchronize()
            assert H.attention_error(out.cpu().numpy(), o.out) <= H.ATTN_TOL, (splits, algo)
            assert np.abs(lse.cpu().numpy() - o.lse).max() <= 2e-3, (splits, algo)
    assert big.device_status() == 0


def test_random_decode_steps_in_one_call():
    """Seeded random caches of a few thousand tokens (1-8 sequences, 1-4 KV heads, 1-8 query heads each, both 16-bit types,
    any split count, with and without splits by length and fixed shares): decode steps in one call until every 16-bit
    segment is full, each against the oracle over the grown cache; the last step raises the flag and appends nothing."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    rng = np.random.default_rng(21)
    for it in range(10):
        hd, g = [(64, 32), (128, 64)][rng.integers(2)]
        dtype = [synth.BF16, synth.F16][rng.integers(2)]
        specs = []
        for _ in range(int(rng.integers(1, 9))):
            S, nw, nt, tail = int(rng.integers(16, 200)), int(rng.integers(1, 60)), int(rng.integers(0, 300)), int(rng.integers(0, 9))
            a = int(rng.integers(0, nw + 1))
            c = int(rng.integers(0, nw - a + 1))
            specs.append(synth.SeqSpec(nw, S, S, nt, (a, c, nw - a - c), tail=tail))
        rep, Hkv = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        w = synth.Workload(f"steps-{it}", dtype, dtype, rep * Hkv, Hkv, hd, g, 64, 1.5, specs, 2100 + it, top_bits=8, pin_first=0)
        bt = synth.batch(w, with_embeddings=False)
        sc = rng.standard_normal(int(bt.t.win_off[-1])).astype(np.float32)
        slack = int(rng.integers(1, 4))
        cap, off16 = H.capacities(w, slack=slack)
        splits = int(rng.integers(0, 13))
        algo = W.DECODE_AUTO | (W.DECODE_BY_LENGTH if rng.integers(2) else 0) | (W.DECODE_FIXED_SHARES if rng.integers(3) == 0 else 0)
        g_run = H.run_gpu(bt, splits=splits, algo=algo, with_scores=False, scores_override=sc, cap=cap, off16=off16)
        o = H.run_oracle(bt, scores_override=sc, with_scores=False, cap=cap, off16=off16)
        H.assert_packed_equal(g_run, o)
        assert H.attention_error(g_run.out.cpu().numpy(), o.out) <= H.ATTN_TOL
        rnd = synth.round_bf16 if dtype == synth.BF16 else synth.round_f16
        sm = 1.0 / float(np.sqrt(hd))
        max_tok = int(np.diff(bt.t.kv_off).max()) + slack + 1
        for step in range(slack + 1):
            kn = rnd(rng.standard_normal((w.B, w.Hkv, w.hd)).astype(np.float32))
            vn = rnd(rng.standard_normal((w.B, w.Hkv, w.hd)).astype(np.float32))
            qn = rnd(bt.q * (1.0 + 0.2 * rng.standard_normal(bt.q.shape).astype(np.float32)))
            out = W.wq_decode_append_attention(g_run.ctx, H.to_dev(qn, w.dtype), g_run.pk, H.to_dev(kn, w.dtype), H.to_dev(vn, w.dtype),
                                               sm, splits, max_tok, algo)
            torch.cuda.synchronize()
            assert g_run.ctx.device_status() == (2 if step == slack else 0), (it, step)
            if step < slack:
                for b in range(w.B):
                    r = int(o.pk.off16[b] + o.pk.len16[b])
                    o.pk.k16[r], o.pk.v16[r] = kn[b], vn[b]
                    o.pk.len16[b] += 1
            assert np.array_equal(g_run.pk.len16.cpu().numpy(), o.pk.len16), (it, step)
            err = H.attention_error(out.cpu().numpy(), O.decode_attention(qn, o.pk, sm))
            assert err <= H.ATTN_TOL, (it, step, err)


def test_splits_by_length_for_sequences_of_different_lengths():
    """25 sequences of 1 to 5760 tokens and more: the automatic split count is raised and every sequence uses its share of the
    splits by length (the workgroups beyond them leave at once).  Parity with the oracle; the same with a workspace that
    only has room for the plain count (the call falls back to it); fixed shares give the same bits twice."""
    H = _h()
    from paper_2605_02262_amd import binding as W
    rng = np.random.default_rng(77)
    specs = []
    for i in range(24):
        nw = int([1, 2, 3, 5, 8, 90][i % 6] if i < 18 else rng.integers(1, 40))
        a = int(rng.integers(0, nw + 1))
        c = int(rng.integers(0, nw - a + 1))
        specs.append(synth.SeqSpec(nw, 64, 64, int(rng.integers(1, 40)), (a, c, nw - a - c)))
    specs.append(synth.SeqSpec(0, 10, 4, 1, (0, 0, 0)))          # and one sequence of a single text token
    bt = _custom(77, 128, 64, 4, 2, synth.BF16, specs, pin=0)
    w = bt.w
    cap, off16 = H.capacities(w)
    max_tok = int(np.diff(bt.t.kv_off).max())
    total = sum((int(c) + 31) // 32 * 32 for c in cap) + int(off16[-1])
    plain, more = W.auto_splits(w.B, w.Hkv, max_tok), W.auto_splits_ragged(w.B, w.Hkv, max_tok, total)
    assert more > plain, (plain, more)
    by_len = W.DECODE_AUTO | W.DECODE_BY_LENGTH
    g, o, err = _check(bt, H, splits=0, algo=by_len)
    assert err <= H.ATTN_TOL
    sm = 1.0 / float(np.sqrt(w.hd))
    q = H.to_dev(bt.q, w.dtype)
    small = W.Context(W.workspace_bytes(w.B, w.Hq, w.hd, plain))
    out = W.wq_decode_attention(small, q, g.pk, sm, 0, max_tok, by_len)
    torch.cuda.synchronize()
    assert H.attention_error(out.cpu().numpy(), o.out) <= H.ATTN_TOL
    fixed = [W.wq_decode_attention(g.ctx, q, g.pk, sm, 0, max_tok, by_len | W.DECODE_FIXED_SHARES).clone() for _ in range(2)]
    torch.cuda.synchronize()
    assert torch.equal(fixed[0], fixed[1])
    assert H.attention_error(fixed[0].cpu().numpy(), o.out) <= H.ATTN_TOL
    for splits, longest in ((5, max_tok), (more, max_tok // 3), (more, 4 * max_tok)):      # a given count; wrong lengths of the longest
        out = W.wq_decode_attention(g.ctx, q, g.pk, sm, splits, longest, by_len)
        torch.cuda.synchronize()
        assert H.attention_error(out.cpu().numpy(), o.out) <= H.ATTN_TOL
    assert g.ctx.device_status() == 0 and small.device_status() == 0


def test_random_medium_caches_through_the_matrix_core_decode_kernel():
    """Seeded random caches of a few thousand tokens per sequence (many 32-token blocks per workgroup, 1-16 splits, 1-8 query
    heads per KV head, both block hand-out modes): quantization bit-exact, attention within the tolerance."""
    H = _h()
    from paper_2605_02262_amd import binding as W
    rng = np.random.default_rng(3)
    for it in range(12):
        hd, g = [(64, 32), (128, 64)][rng.integers(2)]
        dtype = [synth.BF16, synth.F16][rng.integers(2)]
        specs = []
        for _ in range(int(rng.integers(1, 5))):
            S, nw, nt, tail = int(rng.integers(16, 200)), int(rng.integers(1, 60)), int(rng.integers(0, 300)), int(rng.integers(0, 9))
            a = int(rng.integers(0, nw + 1))
            c = int(rng.integers(0, nw - a + 1))
            specs.append(synth.SeqSpec(nw, S, S, nt, (a, c, nw - a - c), tail=tail))
        rep, Hkv = int(rng.integers(1, 9)), int(rng.integers(1, 4))
        w = synth.Workload(f"medium-{it}", dtype, dtype, rep * Hkv, Hkv, hd, g, 64, 1.5, specs, 900 + it,
                           top_bits=[8, 16][rng.integers(2)], pin_first=1)
        bt = synth.batch(w, with_embeddings=False)
        sc = rng.standard_normal(int(bt.t.win_off[-1])).astype(np.float32)
        kw = dict(splits=int(rng.integers(0, 17)), algo=[W.DECODE_AUTO, W.DECODE_MFMA | W.DECODE_FIXED_SHARES][rng.integers(2)],
                  with_scores=False, scores_override=sc)
        if w.top_bits == 16:
            kw["cap"] = [sum((s.n_win * s.win_size + 31) // 32 * 32 for s in w.seqs)] * 3
            kw["off16"] = np.concatenate([[0], np.cumsum([s.n_vis + s.n_text + 4 for s in w.seqs])]).astype(np.int32)
        g_run = H.run_gpu(bt, **kw)
        o = H.run_oracle(bt, scores_override=sc, with_scores=False, **{k: v for k, v in kw.items() if k in ("cap", "off16")})
        assert np.array_equal(g_run.bits.cpu().numpy(), o.bits) and np.array_equal(g_run.perm.cpu().numpy(), o.perm)
        H.assert_packed_equal(g_run, o)
        assert H.attention_error(g_run.out.cpu().numpy(), o.out) <= H.ATTN_TOL
        assert g_run.ctx.device_status() == 0


@pytest.mark.gpu
@pytest.mark.parametrize("cfg,splits", [(1, 7), (1, 16), (1, 40), (1, 64), (3, 16)])
def test_both_merges_of_the_splits_agree_bit_for_bit(cfg, splits):
    """Alg. 2 takes one softmax over all segments; the split over tokens is merged either by the decode kernel's last
    workgroup per (sequence, KV head) or by the merge kernel.  With fixed shares the partials are the same on every run, and
    both merges weigh and sum them with the same arithmetic in the same order: every bit of out and lse must agree (the
    0.5B-shaped layer and a cache of the long-video size)."""
    H = _h()
    from paper_2605_02262_amd import binding as W
    w = synth.workload(cfg)
    bt = synth.batch(w, with_embeddings=False)
    sc = np.random.default_rng(5).standard_normal(int(bt.t.win_off[-1])).astype(np.float32)
    g = H.run_gpu(bt, splits=splits, with_scores=False, scores_override=sc)
    q = H.to_dev(bt.q, w.dtype)
    max_tok = int(np.diff(bt.t.kv_off).max())
    sm = 1.0 / float(np.sqrt(w.hd))
    res = []
    for extra in (0, W.DECODE_SEPARATE_MERGE, 0):
        lse = torch.empty(w.B, w.Hq, dtype=torch.float32, device="cuda")
        out = W.wq_decode_attention(g.ctx, q, g.pk, sm, splits, max_tok, W.DECODE_AUTO | W.DECODE_FIXED_SHARES | extra, lse=lse)
        torch.cuda.synchronize()
        res.append((out.clone(), lse.clone()))
    assert torch.equal(res[0][0], res[2][0]) and torch.equal(res[0][1], res[2][1]), "fixed shares are not reproducible"
    assert torch.equal(res[0][0], res[1][0]), "out differs between the in-kernel merge and the merge kernel"
    assert torch.equal(res[0][1], res[1][1]), "lse differs between the in-kernel merge and the merge kernel"
    if cfg == 1:
        o = H.run_oracle(bt, scores_override=sc, with_scores=False)
        assert H.attention_error(res[1][0].cpu().numpy(), o.out) <= H.ATTN_TOL


@pytest.mark.gpu
def test_decode_steps_by_length_while_the_split_count_of_a_sequence_changes():
    """Sec. 2.2 (the cache grows by one row per step) under WQ_DECODE_BY_LENGTH with more workgroups than compute units:
    a sequence uses ceil(splits * tokens / longest) splits, and tokens grows by one per step, so the count of a sequence
    changes between two steps.  Every workgroup of a launch must see the length the launch started with: the late
    workgroups of a short sequence start after its early ones have finished.  Lengths are chosen so that sequence 1 goes
    from 3 to 4 splits at the third step; outputs and len16 are checked against the oracle at every step."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    splits, steps = 24, 6
    longest = 4800                                  # tokens per split: 200
    specs = [synth.SeqSpec(23, 196, 196, 4800 - 23 * 196, (3, 8, 12))]                  # 4800 tokens: all 24 splits
    specs += [synth.SeqSpec(2, 196, 196, 598 - 2 * 196, (1, 1, 0))]                     # 598 tokens: 3 splits until it has 601
    specs += [synth.SeqSpec(int(n), 196, 196, 100 + 7 * i, (1, int(n) // 2, int(n) - 1 - int(n) // 2)) for i, n in enumerate([4, 9, 14, 19, 3, 8, 12, 20, 6, 11, 16, 5])]
    w = synth.Workload("by-length-steps", synth.BF16, synth.BF16, 28, 4, 128, 64, 64, 1.5, specs, 7100, top_bits=8, pin_first=0)
    assert w.B * w.Hkv * splits > 256
    bt = synth.batch(w, with_embeddings=False)
    sc = np.random.default_rng(8).standard_normal(int(bt.t.win_off[-1])).astype(np.float32)
    cap, off16 = H.capacities(w, slack=steps)
    algo = W.DECODE_AUTO | W.DECODE_BY_LENGTH
    g = H.run_gpu(bt, splits=splits, algo=algo, with_scores=False, scores_override=sc, cap=cap, off16=off16)
    o = H.run_oracle(bt, scores_override=sc, with_scores=False, cap=cap, off16=off16)
    assert H.attention_error(g.out.cpu().numpy(), o.out) <= H.ATTN_TOL
    sm = 1.0 / float(np.sqrt(w.hd))
    rng = np.random.default_rng(9)
    used = lambda n: max(1, min(splits, int(np.ceil(np.float32(n) * (np.float32(splits) / np.float32(longest))))))
    counts = []
    for step in range(steps):
        kn = synth.round_bf16(rng.standard_normal((w.B, w.Hkv, w.hd)).astype(np.float32))
        vn = synth.round_bf16(rng.standard_normal((w.B, w.Hkv, w.hd)).astype(np.float32))
        qn = synth.round_bf16(bt.q * (1.0 + 0.2 * rng.standard_normal(bt.q.shape).astype(np.float32)))
        tokens1 = int(sum(o.pk.cls_len[c][1] for c in range(3)) + o.pk.len16[1]) + 1       # what the launch counts for sequence 1
        counts.append(used(tokens1))
        out = W.wq_decode_append_attention(g.ctx, H.to_dev(qn, w.dtype), g.pk, H.to_dev(kn, w.dtype), H.to_dev(vn, w.dtype), sm, splits,
                                           longest, algo)
        torch.cuda.synchronize()
        assert g.ctx.device_status() == 0, step
        for b in range(w.B):
            r = int(o.pk.off16[b] + o.pk.len16[b])
            o.pk.k16[r], o.pk.v16[r] = kn[b], vn[b]
            o.pk.len16[b] += 1
        assert np.array_equal(g.pk.len16.cpu().numpy(), o.pk.len16), step
        err = H.attention_error(out.cpu().numpy(), O.decode_attention(qn, o.pk, sm))
        assert err <= H.ATTN_TOL, (step, err)
    assert counts[0] == 3 and counts[-1] == 4, counts      # the change of the split count happened inside the loop


def _edge_groups(g: int, bits: int, dtype: int, rng) -> list:
    """Groups of g values (float32 holding values of the storage type `dtype`) that reach the corners of the quantizer of
    Sec. 3.3.3: constant groups, zero minima of either sign, a range so small that the stored scale is 0 (-> 1) or an fp16
    subnormal, the largest storable magnitudes, exact ties of the rounding, data that 8 bits hold without loss."""
    qmax = 2 ** bits - 1
    big = {synth.BF16: 65280.0, synth.F16: 65504.0, synth.F32: 65504.0}[dtype]
    tiny = {synth.BF16: 2.0 ** -30, synth.F16: 2.0 ** -24, synth.F32: 2.0 ** -30}[dtype]     # a value whose range/qmax rounds to an fp16 zero
    f = lambda v: np.asarray(v, dtype=np.float32)
    pad = lambda head, fill: f(list(head) + [fill] * (g - len(head)))
    out = [np.full(g, 1.5, np.float32), np.full(g, 0.0, np.float32), np.full(g, -0.0, np.float32), np.full(g, big, np.float32),
           np.full(g, -big, np.float32),
           pad([-0.0, float(qmax)], 1.0), pad([0.0, -0.0, float(qmax)], 2.0), pad([float(qmax), -0.0, 0.0], 1.0), pad([-0.0, 0.0], 0.0),
           pad([-3.0, -0.0], -1.0),
           pad([0.0, tiny], 0.0), pad([1.0, 1.0 + 2.0 ** -7], 1.0) if dtype != synth.F32 else pad([1.0, 1.0 + 2.0 ** -20], 1.0),
           pad([0.0, qmax * 2.0 ** -20], 2.0 ** -21), pad([-2.0 ** -16, qmax * 2.0 ** -17], 0.0),
           pad([-big, big], 0.0), pad([big, big / 2], big / 4), pad([-big, -big / 2, 0.0], -1.0),
           pad([0.0, float(qmax)] + [k + 0.5 for k in range(min(qmax, g - 2))], 1.0),
           pad([-8.0, -8.0 + 2.0 * qmax] + [-8.0 + 2.0 * (k + 0.5) for k in range(min(qmax, g - 2))], -8.0)]
    ints = rng.integers(-100, -100 + qmax + 1, g).astype(np.float32)
    ints[0], ints[1] = -100.0, -100.0 + qmax
    out.append(ints)                                      # integers spanning exactly qmax: lossless
    out.append(synth.round_to(rng.standard_normal(g).astype(np.float32), dtype))
    return [synth.round_to(x, dtype) if dtype != synth.F32 else x for x in out]


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16, synth.F32])
@pytest.mark.parametrize("hd,g", [(64, 32), (128, 64)])
def test_quantizer_edge_cases(dtype, hd, g):
    """Sec. 3.3.3 on the groups a normal-distributed cache never contains, bit-exact against the oracle (codes, scales,
    minima, 16-bit rows) in all three classes: every window row of K and V is filled, group by group, from the list of
    _edge_groups, shifted per token so that every class and both planes meet every kind of group."""
    H = _h()
    Hkv, S, nw = 2, 16, 12
    dt16 = synth.BF16 if dtype == synth.BF16 else synth.F16
    sq = synth.SeqSpec(nw, S, S, 8, (4, 4, 4))
    w = synth.Workload("edges", dtype, dt16, 2 * Hkv, Hkv, hd, g, 64, 1.0, [sq], 8100 + dtype, top_bits=8, pin_first=0)
    bt = synth.batch(w, with_embeddings=False)
    rng = np.random.default_rng(81 + dtype)
    sc = np.arange(nw, dtype=np.float32)                  # windows 8..11 -> 8 bits, 4..7 -> 4 bits, 0..3 -> 2 bits
    G = hd // g
    for win in range(nw):
        bits = 2 if win < 4 else (4 if win < 8 else 8)
        groups = _edge_groups(g, bits, dtype, rng)
        for t in range(S):
            row = win * S + t
            for h in range(Hkv):
                for j in range(G):
                    k = (t * Hkv * G + h * G + j)
                    bt.K[row, h, j * g:(j + 1) * g] = groups[k % len(groups)]
                    bt.V[row, h, j * g:(j + 1) * g] = groups[(k + 7) % len(groups)]
    g_run = H.run_gpu(bt, splits=2, with_scores=False, scores_override=sc)
    o = H.run_oracle(bt, scores_override=sc, with_scores=False)
    assert o.seg[0].tolist() == [4, 4, 4, 0]
    H.assert_packed_equal(g_run, o)
    # the corners were really there: zero minima stored as +0, scales that fell back to 1, subnormal and large scales
    for c in range(3):
        sb, mb = o.pk.sbits[c][:, :, :4 * S], o.pk.mbits[c][:, :, :4 * S]
        assert (mb == 0x0000).any() and not ((mb == 0x8000) & (sb == 0x3C00)).all()
        assert ((sb > 0) & (sb < 0x0400)).any(), "no fp16-subnormal scale"
        assert (sb >= 0x6000).any(), "no large scale"


@pytest.mark.gpu
@pytest.mark.parametrize("hd,g", [(128, 64), (64, 32)])
def test_adversarial_softmax(hd, g):
    """Alg. 2 takes ONE softmax over the concatenation of all segments; the kernel keeps a running reference exponent and
    forms (weight x value scale) in fp16.  Cases built to stress exactly that, each against the fp64 oracle over the same
    dequantized values: logits that rise along the stream (the reference keeps moving), one token far above all others in
    each of the four segments (the rest of the mass sits 14 nats lower and must not be lost), a zero query and identical
    keys (uniform softmax), value groups with scales just below 16, and all of it once more with every window in the 8-bit
    class, whose value scales are the smallest, and in the 2-bit class; then values of very different magnitudes (the kernel
    places its f16 weights by the sequence's largest value scale, which the quantizer records)."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    nw, S, nt = 32, 196, 128
    rep, Hkv = 7, 2
    sm = 1.0 / float(np.sqrt(hd))
    worst = {}
    for mix_name, quota in (("mixed", (8, 16, 8)), ("all-8-bit", (32, 0, 0)), ("all-2-bit", (0, 0, 32))):
        sq = synth.SeqSpec(nw, S, S, nt, quota)
        w = synth.Workload("adv", synth.BF16, synth.BF16, rep * Hkv, Hkv, hd, g, 64, 1.0, [sq], 9100, top_bits=8, pin_first=0)
        base = synth.batch(w, with_embeddings=False)
        sc = np.random.default_rng(3).standard_normal(nw).astype(np.float32)
        n_tok = nw * S + nt
        rng = np.random.default_rng(17)
        qdir = base.q[0] / np.linalg.norm(base.q[0], axis=-1, keepdims=True)          # [Hq, hd]
        cases = {}
        # (a) the size of the keys, and with it of the logits, grows twentyfold along the stream and the query is long: the
        #     largest logit so far is overtaken again and again, by dozens of nats in all
        K = base.K * np.linspace(0.05, 1.0, n_tok, dtype=np.float32)[:, None, None]
        cases["rising"] = (synth.round_bf16(K), base.V, synth.round_bf16(base.q * 12.0))
        # (b) one token whose key points along the queries of its KV head, about 14 nats above everything else, placed in a
        #     2-bit, a 4-bit, an 8-bit window (by score rank) and in the text rows
        order = np.argsort(-sc, kind="stable")
        spots = {"dominant-top-class": int(order[0]) * S + 5, "dominant-mid-class": int(order[nw // 2]) * S + 100,
                 "dominant-low-class": int(order[-1]) * S + 190, "dominant-text": nw * S + 17}
        for name, tok in spots.items():
            K = base.K.copy()
            q = base.q.copy()
            for kvh in range(Hkv):                       # all heads of the KV head ask the same question, the token's key answers it
                d = qdir[kvh * rep]
                q[0, kvh * rep:(kvh + 1) * rep] = d * np.linalg.norm(base.q[0, kvh * rep:(kvh + 1) * rep], axis=-1).mean()
            q = synth.round_bf16(q)
            for kvh in range(Hkv):
                qh = q[0, kvh * rep].astype(np.float64)
                lg = (K[:, kvh].astype(np.float64) @ qh) * sm
                lg[tok] = -np.inf
                want = np.log(np.exp(lg - lg.max()).sum()) + lg.max() + np.log(9.0)      # the others hold a tenth of the mass
                K[tok, kvh] = (qh / (qh @ qh) * want / sm).astype(np.float32)
            cases[name] = (synth.round_bf16(K), base.V, q)
        # (c) uniform softmax: a zero query; and every key the same
        cases["zero-query"] = (base.K, base.V, np.zeros_like(base.q))
        cases["equal-keys"] = (np.broadcast_to(base.K[:1], base.K.shape).copy(), base.V, base.q)
        # (d) wide values: group scales just below 16 in every class
        Vw = base.V.copy()
        for c, (qmax, wins) in enumerate(((3, order[nw - quota[2]:] if quota[2] else []), (15, order[quota[0]:quota[0] + quota[1]]), (255, order[:quota[0]]))):
            for win in wins:
                blk = Vw[win * S:(win + 1) * S]
                blk *= np.float32(15.5 * qmax) / (blk.reshape(S, Hkv, hd // g, g).max(-1) - blk.reshape(S, Hkv, hd // g, g).min(-1)).max()
        cases["wide-values"] = (base.K, synth.round_bf16(Vw), base.q)
        for name, (K, V, q) in cases.items():
            bt = synth.Batch(w, base.t, base.E_t, base.E_v, np.ascontiguousarray(K), np.ascontiguousarray(V), np.ascontiguousarray(q))
            g_run = H.run_gpu(bt, splits=3, with_scores=False, scores_override=sc)
            o = H.run_oracle(bt, scores_override=sc, with_scores=False)
            assert g_run.ctx.device_status() == 0, (mix_name, name)
            H.assert_packed_equal(g_run, o)
            err = H.attention_error(g_run.out.cpu().numpy(), o.out)
            lse_err = float(np.abs(g_run.lse.cpu().numpy() - o.lse).max())
            worst[(mix_name, name)] = err
            assert err <= H.ATTN_TOL and lse_err <= 2e-3, (mix_name, name, err, lse_err)
            if name.startswith("dominant"):              # the case is what it says: one token holds about nine tenths of the mass
                tok = spots[name]
                lg = (K[:, 0].astype(np.float64) @ q[0, 0].astype(np.float64)) * sm
                top = 1.0 / np.exp(lg - lg[tok]).sum()
                assert 0.8 < top < 0.97 and lg[tok] - np.median(lg) > 9.0, (name, top)
    # the kernel places its f16 weights by the sequence's largest value scale: one group 400 times wider than the rest, and
    # values 2^-12 and 2^11 times the usual size under a peaked softmax, all through the matrix-core kernel
    K_dom, _, q_dom = cases["dominant-low-class"]
    Vbig = base.V.copy()
    Vbig[3, 0, :g] *= 400.0
    for name, (K, V, q) in {"one-wide-group": (base.K, Vbig, base.q), "tiny-values-peaked": (K_dom, base.V * np.float32(2.0 ** -12), q_dom),
                            "huge-values-peaked": (K_dom, base.V * np.float32(2.0 ** 11), q_dom)}.items():
        bt = synth.Batch(w, base.t, base.E_t, base.E_v, np.ascontiguousarray(K), synth.round_bf16(V), np.ascontiguousarray(q))
        g_run = H.run_gpu(bt, splits=3, with_scores=False, scores_override=sc, algo=W.DECODE_MFMA)
        o = H.run_oracle(bt, scores_override=sc, with_scores=False)
        assert g_run.ctx.device_status() == 0, name
        H.assert_packed_equal(g_run, o)
        assert H.attention_error(g_run.out.cpu().numpy(), o.out) <= H.ATTN_TOL, name


@pytest.mark.gpu
@pytest.mark.parametrize("sizes", [(5, 64, 320), (321, 7, 0, 1000), (8192, 640), (3000,)])
def test_assign_bits_few_and_many_windows(sizes):
    """wq_assign_bits on both of its ways (one workgroup per sequence up to 320 windows in the longest sequence; widths by
    several workgroups per sequence, then the class order, above that), bit for bit against the oracle: tied scores, NaN
    and infinite scores, the first-window pin on and off, both top widths, quota and threshold mode, quotas larger than
    the sequence, an empty sequence, and a bound on the windows per sequence below the real count (reported, Sec. 3.2.1,
    Sec. 3.2.2, Alg. 2 prefill loop)."""
    H = _h()
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    rng = np.random.default_rng(sum(sizes))
    win_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    nw, B, max_w = int(win_off[-1]), len(sizes), max(sizes)
    sc = np.round(rng.random(nw) * 40).astype(np.float32) / 40          # many ties
    sc[rng.integers(0, nw, max(nw // 50, 1))] = np.nan
    sc[rng.integers(0, nw, 3)] = np.inf
    sc[rng.integers(0, nw, 3)] = -np.inf
    quota = np.stack([np.array([n // 10, n // 2, n], dtype=np.int32) for n in sizes])     # (the last class takes what is left)
    quota[0] = [sizes[0] + 5, 3, 0]                                      # more top windows than the sequence has
    th = np.stack([np.array([0.3, 0.7], dtype=np.float32) for _ in sizes])
    ctx = W.Context(W.workspace_bytes(B, 0, 0, 0))
    for mode, top, pin in [(W.MODE_QUOTA, 8, 1), (W.MODE_QUOTA, 16, 0), (W.MODE_THRESHOLD, 8, 1), (W.MODE_THRESHOLD, 16, 0)]:
        bits, perm, seg = W.wq_assign_bits(ctx, torch.from_numpy(sc).cuda(), H.i32(win_off), max_w, mode,
                                           H.i32(quota) if mode == W.MODE_QUOTA else None,
                                           torch.from_numpy(th).cuda() if mode == W.MODE_THRESHOLD else None, top, pin)
        torch.cuda.synchronize()
        assert ctx.device_status() == 0
        wb, wp, ws = O.assign_bits(sc, win_off, mode, quota, th, top, pin)
        assert np.array_equal(bits.cpu().numpy(), wb) and np.array_equal(perm.cpu().numpy(), wp)
        assert np.array_equal(seg.cpu().numpy().reshape(B, 4), ws)
    # a bound below the longest sequence's count: reported; the windows inside the bound are assigned as if they were all
    if max_w > 8:
        bound = max_w - 3
        bits, perm, seg = W.wq_assign_bits(ctx, torch.from_numpy(sc).cuda(), H.i32(win_off), bound, W.MODE_QUOTA, H.i32(quota), None, 8, 1)
        torch.cuda.synchronize()
        assert ctx.device_status() & W.DEV_TOO_MANY_WINDOWS
        seg = seg.cpu().numpy().reshape(B, 4)
        for b, n in enumerate(sizes):
            m = min(n, bound)
            cut_off = np.array([0, m], dtype=np.int32)
            wb, wp, ws = O.assign_bits(sc[win_off[b]:win_off[b] + m], cut_off, W.MODE_QUOTA, quota[b:b + 1], None, 8, 1)
            assert np.array_equal(bits.cpu().numpy()[win_off[b]:win_off[b] + m], wb)
            assert np.array_equal(perm.cpu().numpy()[win_off[b]:win_off[b] + m], wp) and np.array_equal(seg[b], ws[0])


def test_device_side_validation_of_an_assignment():
    """wq_reorder_quantize gathers whatever rows perm names; wq_validate_assignment is the debug check of tables that do not
    come straight from wq_assign_bits: a permutation per sequence, class counts that add up.  Also: more windows than the
    bound given to wq_assign_bits are reported, not silently dropped."""
    H = _h()
    from paper_2605_02262_amd import binding as W
    bt = synth.batch(synth.workload(1), with_embeddings=False)
    nw = int(bt.t.win_off[-1])
    sc = np.random.default_rng(2).standard_normal(nw).astype(np.float32)
    g = H.run_gpu(bt, splits=2, with_scores=False, scores_override=sc)
    win_off = H.i32(bt.t.win_off)
    W.wq_validate_assignment(g.ctx, win_off, nw, g.perm, g.seg)
    assert g.ctx.device_status() == 0
    bad = g.perm.clone()
    bad[3] = bad[5]                                   # a window named twice, another one never
    W.wq_validate_assignment(g.ctx, win_off, nw, bad, g.seg)
    assert g.ctx.device_status() == W.DEV_BAD_ASSIGNMENT
    bad = g.perm.clone()
    bad[0] = nw                                       # out of range
    W.wq_validate_assignment(g.ctx, win_off, nw, bad, g.seg)
    assert g.ctx.device_status() == W.DEV_BAD_ASSIGNMENT
    seg = g.seg.clone()
    seg[0, 1] += 1                                    # counts that do not add up
    W.wq_validate_assignment(g.ctx, win_off, nw, g.perm, seg)
    assert g.ctx.device_status() == W.DEV_BAD_ASSIGNMENT
    W.wq_validate_assignment(g.ctx, win_off, nw - 1, g.perm, g.seg)
    assert g.ctx.device_status() == W.DEV_TOO_MANY_WINDOWS
    # wq_assign_bits with a bound below the real count: reported, the windows inside the bound assigned as if they were all
    bits, perm, seg = W.wq_assign_bits(g.ctx, torch.from_numpy(sc).cuda(), win_off, nw - 4, W.MODE_QUOTA, H.i32(bt.t.quota), None, 8, 1)
    assert g.ctx.device_status() == W.DEV_TOO_MANY_WINDOWS
    assert int(seg.sum().item()) == nw - 4
    assert g.ctx.device_status() == 0
