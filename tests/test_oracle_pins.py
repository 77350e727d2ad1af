"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU)."""
import itertools
import json
import os

import numpy as np
import pytest
from scipy.spatial.distance import cdist
from scipy.special import softmax

from oracle import wq_oracle as O
from paper_2605_02262_amd import synth

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


# ----------------------------------------------------------------------------- f16 conversion
def test_f16_conversion_matches_numpy():
    rng = np.random.default_rng(0)
    xs = np.concatenate([
        rng.standard_normal(4000).astype(np.float32) * np.float32(10.0) ** rng.integers(-9, 6, 4000),
        np.array([0.0, -0.0, 1.0, 65504.0, 65519.99, 65520.0, 1e6, -1e6, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001,
                  2.0 ** -14, 2.0 ** -14 * (1 - 2.0 ** -11), 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 6.1e-5,
                  5.96e-8, 3e-8, 2.9e-8], dtype=np.float32)])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([O.f32_to_f16_bits(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_f16_bits_to_f64_all_patterns():
    h = np.arange(65536, dtype=np.uint16)
    want = h.view(np.float16).astype(np.float64)
    got = np.array([O.f16_bits_to_f64(int(x)) for x in h])
    ok = (got == want) | (np.isnan(got) & np.isnan(want))
    assert ok.all()


# ----------------------------------------------------------------------------- O1 scores
def _tables_single(M, N, S):
    return (np.array([0, M]), np.array([0, N]), np.array([S]), np.array([0, M // S]))


def test_scores_hand_case():
    # t1=(1,0,0,0), t2=(0,2,0,0); window 0 = {(3,0,0,0),(1,1,0,0)}: cosines 1,0,1/sqrt2,1/sqrt2 -> (1+sqrt2)/4
    # window 1 = {(-1,0,0,0),(0,0,5,0)}: cosines -1,0,0,0 -> -1/4
    Et = np.array([[1, 0, 0, 0], [0, 2, 0, 0]], dtype=np.float32)
    Ev = np.array([[3, 0, 0, 0], [1, 1, 0, 0], [-1, 0, 0, 0], [0, 0, 5, 0]], dtype=np.float32)
    for form in ("pairwise", "pooled"):
        s = O.window_scores(Ev, Et, *_tables_single(4, 2, 2), form=form)
        assert s == pytest.approx([(1 + np.sqrt(2)) / 4, -0.25], abs=1e-15)


def test_scores_forms_agree_and_match_scipy():
    rng = np.random.default_rng(1)
    M, N, S, D = 24, 5, 6, 17
    Ev = rng.standard_normal((M, D)).astype(np.float32)
    Et = rng.standard_normal((N, D)).astype(np.float32)
    tb = _tables_single(M, N, S)
    a = O.window_scores(Ev, Et, *tb, form="pairwise")
    b = O.window_scores(Ev, Et, *tb, form="pooled")
    assert np.abs(a - b).max() < 1e-12
    cos = 1.0 - cdist(Ev.astype(np.float64), Et.astype(np.float64), metric="cosine")   # library routine
    want = cos.reshape(M // S, S, N).mean(axis=(1, 2))
    assert np.abs(a - want).max() < 1e-12


def test_scores_invariances():
    rng = np.random.default_rng(2)
    M, N, S, D = 12, 4, 4, 9
    Ev = rng.standard_normal((M, D)).astype(np.float32)
    Et = rng.standard_normal((N, D)).astype(np.float32)
    tb = _tables_single(M, N, S)
    base = O.window_scores(Ev, Et, *tb, form="pairwise")
    # order of tokens inside a window and of text tokens does not matter
    Ev2 = Ev.copy()
    Ev2[0:4] = Ev[[2, 0, 3, 1]]
    assert np.abs(O.window_scores(Ev2, Et[::-1].copy(), *tb, form="pairwise") - base).max() < 1e-12
    # positive rescaling of any token does not matter (powers of two: exact in fp32)
    Ev3 = Ev.copy()
    Ev3[5] *= 8.0
    Et3 = Et.copy()
    Et3[1] *= 0.25
    assert np.abs(O.window_scores(Ev3, Et3, *tb, form="pairwise") - base).max() < 1e-12
    # a window made of copies of the single text token scores 1; an orthogonal one scores 0
    t = np.array([[1.0, 2.0, -3.0]], dtype=np.float32)
    w = np.concatenate([np.repeat(t, 3, 0), np.array([[2, -1, 0]] * 3, dtype=np.float32)])
    s = O.window_scores(w, t, *_tables_single(6, 1, 3), form="pairwise")
    assert s == pytest.approx([1.0, 0.0], abs=1e-15)
    # zero-norm token: its pairs count as 0
    z = O.window_scores(np.zeros((3, 3), np.float32), t, *_tables_single(3, 1, 3), form="pooled")
    assert z[0] == 0.0


def test_scores_ragged_batch_and_tail():
    rng = np.random.default_rng(3)
    D = 8
    vis_off = np.array([0, 10, 10, 31])          # 10 tokens (S=4 -> 2 windows + tail 2), empty, 21 (S=7 -> 3)
    txt_off = np.array([0, 3, 5, 9])
    win_size = np.array([4, 4, 7])
    win_off = np.array([0, 2, 2, 5])
    Ev = rng.standard_normal((31, D)).astype(np.float32)
    Et = rng.standard_normal((9, D)).astype(np.float32)
    s = O.window_scores(Ev, Et, vis_off, txt_off, win_size, win_off, form="pairwise")
    cos = 1.0 - cdist(Ev.astype(np.float64), Et.astype(np.float64), metric="cosine")
    assert s[1] == pytest.approx(cos[4:8, 0:3].mean(), abs=1e-13)
    assert s[4] == pytest.approx(cos[10 + 14:10 + 21, 5:9].mean(), abs=1e-13)


# ----------------------------------------------------------------------------- O2 bits
def test_threshold_rule_is_strict():
    assert GOLD["bit_rule"]["strict"]
    s = np.array([0.5, 0.2, 0.8, 0.81, 0.19, np.nan], dtype=np.float32)
    th = np.array([[np.float32(0.2), np.float32(0.8)]], dtype=np.float32)
    bits, perm, seg = O.assign_bits(s, [0, 6], 1, thresholds=th, top_bits=16, pin_first=0)
    assert bits.tolist() == [4, 4, 4, 16, 2, 4]          # equality stays INT4 (Sec. 3.2.1)
    assert perm.tolist() == [4, 0, 1, 2, 5, 3] and seg.tolist() == [[1, 4, 0, 1]]
    bits, _, _ = O.assign_bits(s, [0, 6], 1, thresholds=th, top_bits=16, pin_first=1)
    assert bits[0] == 16                                    # first window pinned (Sec. 3.2.2)


def test_quota_rule_ties_and_stability():
    s = np.array([0.3, 0.9, 0.3, 0.9, 0.1, 0.3], dtype=np.float32)
    bits, perm, seg = O.assign_bits(s, [0, 6], 0, quota=[[1, 2, 3]], top_bits=8, pin_first=0)
    # order: 1,3 (0.9; lower index first), 0,2,5 (0.3), 4
    assert bits.tolist() == [4, 8, 2, 4, 2, 2]
    assert perm.tolist() == [2, 4, 5, 0, 3, 1] and seg.tolist() == [[3, 2, 1, 0]]
    # pinned first window takes the single top slot
    bits, perm, seg = O.assign_bits(s, [0, 6], 0, quota=[[1, 2, 3]], top_bits=8, pin_first=1)
    assert bits.tolist() == [8, 4, 2, 4, 2, 2] and seg.tolist() == [[3, 2, 1, 0]]
    # no top slot: the pin uses a 4-bit slot, mix stays 0/2/4 + the pinned one
    bits, _, seg = O.assign_bits(s, [0, 6], 0, quota=[[0, 2, 4]], top_bits=8, pin_first=1)
    assert bits.tolist() == [8, 4, 2, 2, 2, 2] and seg.tolist() == [[4, 1, 1, 0]]
    # top tier kept 16-bit (the paper's tiers)
    bits, perm, seg = O.assign_bits(s, [0, 6], 0, quota=[[2, 2, 2]], top_bits=16, pin_first=0)
    assert bits.tolist() == [4, 16, 4, 16, 2, 2] and perm.tolist() == [4, 5, 0, 2, 1, 3]


def test_quota_rule_against_counting_form_and_brute_force():
    rng = np.random.default_rng(4)
    for trial in range(50):
        W = int(rng.integers(1, 40))
        s = rng.choice(np.array([0.1, 0.2, 0.5, 0.7, -0.3], np.float32), W) if trial % 2 else \
            rng.standard_normal(W).astype(np.float32)
        n_top = int(rng.integers(0, W + 1))
        n4 = int(rng.integers(0, W - n_top + 1))
        pin = int(rng.integers(0, 2))
        bits, perm, seg = O.assign_bits(s, [0, W], 0, quota=[[n_top, n4, W - n_top - n4]], top_bits=8, pin_first=pin)
        first = 1 if pin else 0
        rank = O.rank_by_counting(s, first)
        a, c = n_top, n4
        if pin:
            if a > 0:
                a -= 1
            elif c > 0:
                c -= 1
        want = np.array([8 if r < a else (4 if r < a + c else 2) for r in rank], dtype=np.uint8)
        if pin:
            want[0] = 8
        assert np.array_equal(bits, want)
        assert sorted(perm.tolist()) == list(range(W)) and seg.sum() == W
        # stable partition in class order 2,4,8,16
        want_perm = [i for b in (2, 4, 8, 16) for i in range(W) if bits[i] == b]
        assert perm.tolist() == want_perm
    # brute force: the selected top set maximises the score sum among all sets of that size
    s = np.array([0.4, -1.0, 0.7, 0.1, 0.65], dtype=np.float32)
    bits, _, _ = O.assign_bits(s, [0, 5], 0, quota=[[2, 0, 3]], top_bits=8, pin_first=0)
    best = max(itertools.combinations(range(5), 2), key=lambda c: s[list(c)].sum())
    assert sorted(np.nonzero(bits == 8)[0].tolist()) == sorted(best)


def test_mix_to_counts_integer_rule():
    assert synth.mix_to_quota(8, 25, 50) == (2, 4, 2)
    assert synth.mix_to_quota(32, 25, 50) == (8, 16, 8)
    assert synth.mix_to_quota(64, 20, 50) == (13, 32, 19)
    assert synth.mix_to_quota(256, 10, 40) == (26, 102, 128)


# ----------------------------------------------------------------------------- O3 quantization
def _deq(codes, sb, mb):
    return O.f16_bits_to_f64(mb) + O.f16_bits_to_f64(sb) * codes.astype(np.float64)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantize_error_bound_and_end_points(bits):
    rng = np.random.default_rng(5 + bits)
    qmax = 2 ** bits - 1
    for trial in range(300):
        n = int(rng.choice([32, 64, 128]))
        x = synth.round_bf16((rng.standard_normal(n) * 10.0 ** rng.uniform(-3, 3)).astype(np.float32))
        if trial % 7 == 0:
            x += np.float32(rng.uniform(-50, 50))
            x = synth.round_bf16(x)
        codes, sb, mb = O.quantize_group(x, bits)
        s, m = O.f16_bits_to_f64(sb), O.f16_bits_to_f64(mb)
        lo, hi = float(x.min()), float(x.max())
        assert codes.max() <= qmax
        assert abs(m - lo) <= 2.0 ** -11 * abs(lo) + 2.0 ** -25          # m is the fp16 image of the minimum
        xhat = _deq(codes, sb, mb)
        # |x - x^| <= s/2 (round to nearest) + distance the minimum moved when stored as fp16
        assert np.abs(x - xhat).max() <= s / 2 * (1 + 2.0 ** -10) + abs(m - lo) + 1e-30
        assert codes[np.argmin(x)] == 0
        if hi > lo and s > 2.0 ** -14:
            assert codes[np.argmax(x)] == qmax


def test_quantize_special_groups():
    # constant group: all codes 0 and x^ = the constant (bf16 values are exact in fp16 here)
    x = np.full(64, 1.5, dtype=np.float32)
    codes, sb, mb = O.quantize_group(x, 4)
    assert codes.max() == 0 and O.f16_bits_to_f64(mb) == 1.5 and O.f16_bits_to_f64(sb) == 1.0
    # 8 bits on integer data spanning exactly 255 is lossless
    rng = np.random.default_rng(6)
    x = rng.integers(-100, 156, 64).astype(np.float32)
    x[0], x[1] = -100, 155
    codes, sb, mb = O.quantize_group(x, 8)
    assert np.array_equal(_deq(codes, sb, mb), x.astype(np.float64))
    assert np.array_equal(codes.astype(np.int64), x.astype(np.int64) + 100)
    # 2 bits on {0,1,2,3}
    x = np.tile(np.array([0, 1, 2, 3], np.float32), 8)
    codes, sb, mb = O.quantize_group(x, 2)
    assert np.array_equal(codes, x.astype(np.uint8))
    # ties go to even: (x-m)/s = 0.5, 1.5, 2.5 -> 0, 2, 2
    x = np.array([0.0, 3.0, 0.5, 1.5, 2.5] + [0.0] * 27, dtype=np.float32)
    codes, _, _ = O.quantize_group(x, 2)
    assert codes[:5].tolist() == [0, 3, 0, 2, 2]


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantize_zero_minimum_is_stored_as_plus_zero(bits):
    """Sec. 3.3.3 stores the group minimum.  -0 and +0 compare equal, so which of them a minimum search ends with depends on
    the order it looks at the values (a loop and a tree of pairwise minima disagree); the format therefore stores a zero
    minimum as +0 whatever its sign and wherever it stands in the group.  Only an exact zero is meant: a negative minimum
    that rounds to zero in binary16 keeps its sign."""
    qmax = 2 ** bits - 1
    rest = [float(qmax), 1.0, 2.0]
    for zeros in ([-0.0], [0.0], [-0.0, 0.0], [0.0, -0.0], [0.0, 0.0, -0.0], [-0.0, -0.0, 0.0]):
        for where in ("front", "back", "middle"):
            vals = {"front": zeros + rest, "back": rest + zeros, "middle": rest[:1] + zeros + rest[1:]}[where]
            x = np.array(vals + [1.0] * (32 - len(vals)), dtype=np.float32)
            codes, sb, mb = O.quantize_group(x, bits)
            assert mb == 0x0000, (zeros, where, hex(mb))
            assert O.f16_bits_to_f64(sb) == 1.0 and codes.tolist() == [int(v) for v in np.abs(x)]
    # nothing but zeros of either sign: constant group, m = +0, s falls back to 1
    for x in (np.full(32, -0.0, np.float32), np.array([0.0, -0.0] * 16, np.float32)):
        codes, sb, mb = O.quantize_group(x, bits)
        assert (mb, sb, int(codes.max())) == (0x0000, 0x3C00, 0)
    # a zero that is the group's largest value is not touched by the rule, and neither is a tiny negative minimum
    x = np.array([-3.0, -0.0] + [-1.0] * 30, dtype=np.float32)
    codes, sb, mb = O.quantize_group(x, bits)
    assert O.f16_bits_to_f64(mb) == -3.0 and codes[1] == qmax
    x = np.array([-1e-8, 1.0] + [0.5] * 30, dtype=np.float32)
    _, _, mb = O.quantize_group(x, bits)
    assert mb == 0x8000


def _unpack_k(img, cap, hd, bits):
    """Independent reading of the K-plane layout text: tile of 16 tokens, [quarter][token][hd/4 codes]."""
    out = np.zeros((cap, hd), dtype=np.uint8)
    per = 8 // bits
    flat = np.zeros(cap * hd, dtype=np.uint8)
    for k in range(per):
        flat[k::per] = (img >> (k * bits)) & (2 ** bits - 1)
    tiles = flat.reshape(cap // 16, 4, 16, hd // 4)          # [tile][j][m][e]
    for j in range(4):
        out.reshape(cap // 16, 16, hd)[:, :, j * (hd // 4):(j + 1) * (hd // 4)] = tiles[:, j]
    return out


def _unpack_v(img, cap, hd, bits):
    """V-plane layout text: block of 32 tokens, [jj][mm][ct][tau]; channel 16ct+mm, token 16(tau/4)+4jj+tau%4."""
    per = 8 // bits
    flat = np.zeros(cap * hd, dtype=np.uint8)
    for k in range(per):
        flat[k::per] = (img >> (k * bits)) & (2 ** bits - 1)
    blk = flat.reshape(cap // 32, 4, 16, hd // 16, 8)
    out = np.zeros((cap // 32, 32, hd), dtype=np.uint8)
    for jj in range(4):
        for tau in range(8):
            u = 16 * (tau // 4) + 4 * jj + tau % 4
            for ct in range(hd // 16):
                out[:, u, 16 * ct:16 * ct + 16] = blk[:, jj, :, ct, tau]
    return out.reshape(cap, hd)


def _small_packed(seed=7, top_bits=8, S=5, W=11, extra=9, quota=(3, 4, 4), Hkv=2, hd=64, g=32, dtype=synth.BF16):
    rng = np.random.default_rng(seed)
    rows = W * S + extra
    K = synth.round_to(rng.standard_normal((rows, Hkv, hd)).astype(np.float32) * 3, dtype)
    V = synth.round_to(rng.standard_normal((rows, Hkv, hd)).astype(np.float32), dtype)
    scores = rng.standard_normal(W).astype(np.float32)
    bits, perm, seg = O.assign_bits(scores, [0, W], 0, quota=[list(quota)], top_bits=top_bits, pin_first=1)
    pk = O.reorder_quantize(K, V, [0, rows], [S], [0, W], perm, seg, g)
    return K, V, bits, perm, seg, pk


@pytest.mark.parametrize("hd,g", [(64, 32), (128, 64), (128, 32)])
def test_pack_round_trip(hd, g):
    K, V, bits, perm, seg, pk = _small_packed(hd=hd, g=g)
    for c, b in enumerate((2, 4, 8)):
        img = pk.packed_codes(c)
        cap = pk.cap[c]
        assert cap % 32 == 0 and img.shape[-1] == cap * hd * b // 8
        for h in range(pk.Hkv):
            assert np.array_equal(_unpack_k(img[0, h], cap, hd, b), pk.codes[c][0, h])
            assert np.array_equal(_unpack_v(img[1, h], cap, hd, b), pk.codes[c][1, h])
        meta = pk.packed_meta(c).reshape(2, pk.Hkv, cap // 16, hd // g, 16)
        assert np.array_equal((meta & 0xFFFF).transpose(0, 1, 2, 4, 3).reshape(2, pk.Hkv, cap, hd // g), pk.sbits[c])
        assert np.array_equal((meta >> 16).transpose(0, 1, 2, 4, 3).reshape(2, pk.Hkv, cap, hd // g), pk.mbits[c])


def test_reorder_is_a_stable_partition_of_all_rows():
    K, V, bits, perm, seg, pk = _small_packed(top_bits=16)
    S, W = 5, 11
    rows = np.concatenate([pk.src_row[c][pk.src_row[c] >= 0] for c in range(3)] + [pk.rows16[pk.rows16 >= 0]])
    assert sorted(rows.tolist()) == list(range(K.shape[0]))          # every token lands exactly once
    for c, b in enumerate((2, 4, 8)):
        r = pk.src_row[c][: pk.cls_len[c, 0]]
        wins = r[::S] // S
        assert np.all(np.diff(wins) > 0) and np.all(bits[wins] == b)  # ascending window index inside a class
        assert np.all(pk.src_row[c][pk.cls_len[c, 0]:] == -1)
    n16 = seg[0, 3] * S
    assert np.all(bits[pk.rows16[:n16:S] // S] == 16)
    assert pk.rows16[n16:].tolist() == list(range(W * S, K.shape[0]))  # tail + text follow, in order
    assert pk.len16[0] == n16 + 9


def test_paper_memory_arithmetic():
    g = GOLD["kv_bytes_saved_per_layer"]
    S = 4
    n2, n4 = g["int2_tokens"] // S, g["int4_tokens"] // S
    assert n2 * S == g["int2_tokens"] and n4 * S == g["int4_tokens"]
    W = n2 + n4
    rows = W * S + g["fp16_tokens"]
    Hkv, hd = g["kv_heads"], g["head_dim"]
    rng = np.random.default_rng(8)
    K = rng.standard_normal((rows, Hkv, hd)).astype(np.float32)
    scores = rng.standard_normal(W).astype(np.float32)
    bits, perm, seg = O.assign_bits(scores, [0, W], 0, quota=[[0, n4, n2]], top_bits=16, pin_first=0)
    pk = O.reorder_quantize(K, K, [0, rows], [S], [0, W], perm, seg, 64)
    code_bytes = sum(int(pk.cls_len[c, 0]) * Hkv * hd * 2 * b // 8 for c, b in enumerate((2, 4, 8)))
    fp16_bytes = (g["int2_tokens"] + g["int4_tokens"]) * Hkv * hd * 2 * 2
    assert fp16_bytes - code_bytes == g["bytes_saved"]
    assert pk.len16[0] == g["fp16_tokens"]


# ----------------------------------------------------------------------------- O4 attention
def test_dense_attention_is_textbook():
    rng = np.random.default_rng(9)
    T, Hq, Hkv, hd = 37, 6, 2, 16
    q = rng.standard_normal((Hq, hd)).astype(np.float32)
    K = rng.standard_normal((T, Hkv, hd)).astype(np.float32)
    V = rng.standard_normal((T, Hkv, hd)).astype(np.float32)
    got = O.attention_dense(q, K, V, 0.25)
    for h in range(Hq):
        p = softmax(0.25 * K[:, h // 3].astype(np.float64) @ q[h].astype(np.float64))
        assert np.abs(got[h] - p @ V[:, h // 3].astype(np.float64)).max() < 1e-13


def test_reorder_invariance_of_decode_attention():
    """Sec. 3.3.2: without a mask the output does not depend on the order of the KV blocks."""
    K, V, bits, perm, seg, pk = _small_packed(top_bits=16)
    rng = np.random.default_rng(10)
    q = rng.standard_normal((6, 64)).astype(np.float32)
    order = np.concatenate([pk.src_row[c][pk.src_row[c] >= 0] for c in range(3)] + [pk.rows16])
    a = O.attention_dense(q, K, V, 0.125)
    b = O.attention_dense(q, K[order], V[order], 0.125)
    assert not np.array_equal(order, np.arange(len(order)))
    assert np.abs(a - b).max() < 1e-13


def _dequantized_cache(pk, rows, Hkv, hd):
    """fp64 cache in ORIGINAL token order rebuilt from codes and metadata (numpy, not the oracle's loop)."""
    Kh = np.zeros((rows, Hkv, hd))
    Vh = np.zeros((rows, Hkv, hd))
    g = pk.group
    for c in range(3):
        n = int(pk.cls_len[c, 0])
        src = pk.src_row[c][:n]
        for pl, dst in enumerate((Kh, Vh)):
            s = pk.sbits[c][pl, :, :n].view(np.float16).astype(np.float64)
            m = pk.mbits[c][pl, :, :n].view(np.float16).astype(np.float64)
            x = np.repeat(m, g, axis=-1) + np.repeat(s, g, axis=-1) * pk.codes[c][pl, :, :n]
            dst[src] = x.transpose(1, 0, 2)
    used = pk.rows16 >= 0
    Kh[pk.rows16[used]] = pk.k16[used]
    Vh[pk.rows16[used]] = pk.v16[used]
    return Kh, Vh


@pytest.mark.parametrize("hd,g,top", [(64, 32, 8), (128, 64, 16), (128, 32, 8)])
def test_decode_attention_equals_textbook_on_dequantized_cache(hd, g, top):
    K, V, bits, perm, seg, pk = _small_packed(top_bits=top, hd=hd, g=g, seed=11)
    rng = np.random.default_rng(12)
    Hq = 14
    q = rng.standard_normal((1, Hq, hd)).astype(np.float32)
    got, lse = O.decode_attention(q, pk, 1 / np.sqrt(hd), want_lse=True)
    Kh, Vh = _dequantized_cache(pk, K.shape[0], 2, hd)
    for h in range(Hq):
        lg = (Kh[:, h // 7] @ q[0, h].astype(np.float64)) / np.sqrt(hd)
        p = softmax(lg)
        assert np.abs(got[0, h] - p @ Vh[:, h // 7]).max() < 1e-12
        assert lse[0, h] == pytest.approx(np.log(np.exp(lg - lg.max()).sum()) + lg.max(), abs=1e-12)


def test_lossless_8bit_pipeline_equals_attention_on_original_cache():
    """Integer-valued K,V with range 255 per group are stored exactly by 8 bits, so the whole
    reorder -> quantize -> decode chain must reproduce textbook attention on the original cache."""
    rng = np.random.default_rng(13)
    S, W, Hkv, hd, g = 4, 6, 2, 64, 32
    rows = W * S + 3
    K = rng.integers(-128, 128, (rows, Hkv, hd)).astype(np.float32)
    V = rng.integers(0, 256, (rows, Hkv, hd)).astype(np.float32)
    K[..., 0::32], K[..., 1::32] = -128, 127
    V[..., 0::32], V[..., 1::32] = 0, 255
    scores = rng.standard_normal(W).astype(np.float32)
    bits, perm, seg = O.assign_bits(scores, [0, W], 0, quota=[[W, 0, 0]], top_bits=8, pin_first=0)
    pk = O.reorder_quantize(K, V, [0, rows], [S], [0, W], perm, seg, g)
    q = (rng.standard_normal((1, 14, hd)) * 0.02).astype(np.float32)
    got = O.decode_attention(q, pk, 0.125)
    want = O.attention_dense(q[0], K, V, 0.125)
    assert np.abs(got[0] - want).max() < 1e-10


def test_attention_degenerate_cases():
    K, V, bits, perm, seg, pk = _small_packed(seed=14)
    rng = np.random.default_rng(15)
    hd = 64
    # zero query -> uniform weights -> output is the mean of the dequantized values
    q0 = np.zeros((1, 14, hd), np.float32)
    got = O.decode_attention(q0, pk, 0.125)
    Kh, Vh = _dequantized_cache(pk, K.shape[0], 2, hd)
    for h in range(14):
        assert np.abs(got[0, h] - Vh[:, h // 7].mean(axis=0)).max() < 1e-12
    # a query that makes one token's logit dominate returns that token's value row
    t = 17
    qd = np.zeros((1, 14, hd), np.float32)
    qd[0, :, :] = (Kh[t, 0] * 50).astype(np.float32)
    lg = Kh[:, 0] @ qd[0, 0].astype(np.float64) * 0.125
    if np.sort(lg)[-1] - np.sort(lg)[-2] > 60:
        got = O.decode_attention(qd, pk, 0.125)
        assert np.abs(got[0, 0] - Vh[np.argmax(lg), 0]).max() < 1e-9
    # grouped-query attention = multi-head attention over KV heads repeated Hq/Hkv times
    q = rng.standard_normal((14, hd)).astype(np.float32)
    a = O.attention_dense(q, K, V, 0.125)
    b = O.attention_dense(q, np.repeat(K, 7, axis=1), np.repeat(V, 7, axis=1), 0.125)
    assert np.abs(a - b).max() < 1e-13


def test_empty_and_tail_only_sequences():
    rng = np.random.default_rng(16)
    Hkv, hd, g = 2, 64, 32
    # sequence 0: no windows at all (3 text rows); sequence 1: 2 windows of 4 + 5 tail/text rows
    kv_off = np.array([0, 3, 16])
    win_size = np.array([4, 4])
    win_off = np.array([0, 0, 2])
    K = synth.round_bf16(rng.standard_normal((16, Hkv, hd)).astype(np.float32))
    V = synth.round_bf16(rng.standard_normal((16, Hkv, hd)).astype(np.float32))
    bits, perm, seg = O.assign_bits(np.array([0.1, 0.9], np.float32), win_off, 0, quota=[[0, 0, 0], [1, 0, 1]],
                                    top_bits=8, pin_first=0)
    pk = O.reorder_quantize(K, V, kv_off, win_size, win_off, perm, seg, g)
    assert pk.len16.tolist() == [3, 5] and pk.cls_len[:, 0].tolist() == [0, 0, 0]
    q = rng.standard_normal((2, 14, hd)).astype(np.float32)
    got = O.decode_attention(q, pk, 0.125)
    want0 = O.attention_dense(q[0], K[:3], V[:3], 0.125)
    assert np.abs(got[0] - want0).max() < 1e-13


# ----------------------------------------------------------------------------------------------------------------
# Sec. 3.2.3: threshold functions and the batch-shared configuration
# ----------------------------------------------------------------------------------------------------------------
def test_threshold_functions_closed_forms():
    """What the paper states about f1, f2 (end points, f1 <= f2 on [0, 1]) and what follows from the formulas
    (f1(s) + f2(1 - s) = 1; at the default alpha = 2, f1(1/2) = 1 / (1 + e) and f2(1/2) = e / (1 + e))."""
    s = np.linspace(0.0, 1.0, 101)
    for alpha in (0.5, 1.0, 2.0, 4.0, 8.0):
        lo, hi = O.layer_thresholds(s, alpha)
        assert lo[0] == 0.0 and hi[0] == 0.0
        assert abs(lo[-1] - 1.0) < 1e-15 and abs(hi[-1] - 1.0) < 1e-15
        assert np.all(lo <= hi + 1e-15)
        assert np.all(np.diff(lo) > 0) and np.all(np.diff(hi) > 0)
        lo_r, hi_r = O.layer_thresholds(1.0 - s, alpha)
        assert np.abs(lo + hi_r - 1.0).max() < 1e-14
    lo, hi = O.layer_thresholds([0.5], 2.0)
    assert abs(lo[0] - 1.0 / (1.0 + np.e)) < 1e-15 and abs(hi[0] - np.e / (1.0 + np.e)) < 1e-15
    lo, hi = O.layer_thresholds(s, 0.0)
    assert np.array_equal(lo, s) and np.array_equal(hi, s)
    # a dropped "-1", a swapped sign of alpha or a swapped pair would each break one of the lines above
    lo, hi = O.layer_thresholds(s, 1e-9)
    assert np.abs(lo - s).max() < 1e-6 and np.abs(hi - s).max() < 1e-6


def test_vote_bits_majority_ties_and_ragged_positions():
    # three requests with 4, 4 and 2 windows
    bits = np.array([16, 2, 4, 2,   16, 4, 4, 4,   16, 4], dtype=np.uint8)
    win_off = np.array([0, 4, 8, 10])
    out, perm, seg = O.vote_bits(bits, win_off)
    # position 0: unanimous 16; position 1: 2,4,4 -> 4; position 2: 4,4 -> 4; position 3: 2 vs 4, a tie -> 4
    assert out.tolist() == [16, 4, 4, 4, 16, 4, 4, 4, 16, 4]
    assert seg.tolist() == [[0, 3, 0, 1], [0, 3, 0, 1], [0, 1, 0, 1]]
    assert perm.tolist() == [1, 2, 3, 0, 1, 2, 3, 0, 1, 0]
    # one request: the vote changes nothing; the order is the stable class order of assign_bits
    rng = np.random.default_rng(5)
    sc = rng.standard_normal(37).astype(np.float32)
    b1, p1, s1 = O.assign_bits(sc, [0, 37], 0, quota=[[5, 12, 20]], top_bits=8, pin_first=1)
    b2, p2, s2 = O.vote_bits(b1, [0, 37])
    assert np.array_equal(b1, b2) and np.array_equal(p1, p2) and np.array_equal(s1, s2)
    # brute force on random small batches: every position's result is a mode, and the widest among the modes
    for trial in range(20):
        B = int(rng.integers(1, 6))
        n = rng.integers(1, 9, size=B)
        off = np.concatenate([[0], np.cumsum(n)])
        bb = rng.choice([2, 4, 8], size=int(off[-1])).astype(np.uint8)
        out, perm, seg = O.vote_bits(bb, off)
        for p in range(int(n.max())):
            col = [int(bb[off[b] + p]) for b in range(B) if n[b] > p]
            cnt = {w: col.count(w) for w in set(col)}
            top = max(cnt.values())
            want = max(w for w, c in cnt.items() if c == top)
            assert all(int(out[off[b] + p]) == want for b in range(B) if n[b] > p)
        for b in range(B):
            pb = perm[off[b]:off[b + 1]]
            assert sorted(pb.tolist()) == list(range(int(n[b])))
            widths = out[off[b]:off[b + 1]][pb].astype(int).tolist()
            assert widths == sorted(widths)                                # classes in the order 2, 4, 8, 16 ...
            for w in set(widths):                                          # ... and index order inside a class
                idx = [int(i) for i in pb if out[off[b] + i] == w]
                assert idx == sorted(idx)
            assert seg[b].tolist() == [widths.count(w) for w in (2, 4, 8, 16)]


def test_reorder_quantize_refuses_buffers_that_are_too_small():
    """The oracle's C routines trust the capacities they are given: the wrapper refuses what does not fit (a pinned first
    window takes the top width even when the top quota is zero, so that class then needs room for it)."""
    w = synth.Workload("guard", synth.BF16, synth.BF16, 14, 2, 64, 32, 64, 1.0, [synth.SeqSpec(4, 16, 16, 8, (0, 2, 2))], 5,
                       top_bits=8, pin_first=1)
    bt = synth.batch(w)
    t = bt.t
    sc = O.window_scores(bt.E_v, bt.E_t, t.vis_off, t.txt_off, t.win_size, t.win_off, form="pooled").astype(np.float32)
    bits, perm, seg = O.assign_bits(sc, t.win_off, 0, quota=t.quota, top_bits=8, pin_first=1)
    assert seg.tolist() == [[2, 1, 1, 0]] and bits[0] == 8              # the pin took one 4-bit slot
    with pytest.raises(ValueError):
        O.reorder_quantize(bt.K, bt.V, t.kv_off, t.win_size, t.win_off, perm, seg, w.group, off16=[0], cap=[32, 32, 0], cap16=8)
    with pytest.raises(ValueError):
        O.reorder_quantize(bt.K, bt.V, t.kv_off, t.win_size, t.win_off, perm, seg, w.group, off16=[0], cap=[32, 32, 32], cap16=4)
    pk = O.reorder_quantize(bt.K, bt.V, t.kv_off, t.win_size, t.win_off, perm, seg, w.group, off16=[0], cap=[32, 32, 32], cap16=8)
    assert pk.cls_len.tolist() == [[32], [16], [16]] and pk.len16.tolist() == [8]
