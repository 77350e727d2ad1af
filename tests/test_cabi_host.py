"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and rejects bad arguments
before touching a GPU.  No compute call is made here."""
import ctypes as C
import os
import re

import numpy as np

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2605_02262_amd", "libwq.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2605_02262_amd import build
        build.build(verbose=False)
    from paper_2605_02262_amd import binding
    return binding.lib()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "wq.h")).read() + open(os.path.join(ROOT, "include", "wq_measure.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(wq_[a-z0-9_]+)\s*\(", hdr))
    assert {"wq_window_scores", "wq_assign_bits", "wq_reorder_quantize", "wq_decode_attention"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in include/*.h but not exported"
    assert {"wq_decode_attention_static", "wq_validate_assignment", "wq_probe_stream", "wq_decode_times_us"} <= names


def test_pure_size_helpers(lib):
    from paper_2605_02262_amd import binding as W
    # codes only, hd=128, 4 KV heads, K+V: 2-bit token = 2*4*32 B; padded to 32 tokens
    cb, mb = W.packed_bytes(2, 12564, 4, 128, 64)
    assert cb == 12576 * 4 * 2 * 32 and mb == 12576 * 4 * 2 * 2 * 4
    assert W.packed_bytes(4, 32, 2, 64, 32) == (32 * 2 * 2 * 32, 32 * 2 * 2 * 2 * 4)
    assert W.packed_bytes(3, 32, 2, 64, 32) == (0, 0)            # unsupported width
    assert W.packed_bytes(8, 32, 2, 96, 32) == (0, 0)            # unsupported head dim
    assert W.workspace_bytes(4, 28, 128, 64) >= 256 + 4 * 28 * 64 * 130 * 4
    assert 1 <= W.auto_splits(4, 4, 50688) <= 256
    assert W.auto_splits(1, 2, 100) == 1
    # sequences of about equal length: the same count; very different lengths: more splits (used by length), never fewer,
    # never so many that the longest sequence's splits get under 1024 tokens
    assert W.auto_splits_ragged(4, 4, 50688, 4 * 50688) == W.auto_splits(4, 4, 50688)
    assert W.auto_splits_ragged(4, 4, 50688, 3 * 50688 + 1000) == W.auto_splits(4, 4, 50688)
    assert W.auto_splits_ragged(32, 4, 25344, 32 * 25344 // 2) == 4 * W.auto_splits(32, 4, 25344) == 8
    assert W.auto_splits_ragged(32, 4, 25344, 32 * 25344 // 100) == 25
    assert W.auto_splits_ragged(32, 4, 2000, 32 * 200) == W.auto_splits(32, 4, 2000) == 2
    assert W.auto_splits_ragged(0, 4, 100, 0) == 1 and W.auto_splits_ragged(4, 4, 0, 100) == W.auto_splits(4, 4, 0)


def test_split_count_helpers_over_random_batches(lib):
    """Properties that hold for any batch: at least one split and at most 256; never more splits than 1024-token pieces of the
    longest sequence; the count for sequences of different lengths is never below the plain one, equal to it when the batch
    is at least three quarters full, and does not shrink when the batch gets emptier."""
    from paper_2605_02262_amd import binding as W
    rng = np.random.default_rng(5)
    for _ in range(2000):
        B, Hkv = int(rng.integers(1, 200)), int(rng.integers(1, 9))
        longest = int(rng.integers(1, 300000))
        plain = W.auto_splits(B, Hkv, longest)
        most = (longest + 1023) // 1024
        assert 1 <= plain <= min(256, most)
        assert plain == min(most, 256, -(-256 // (B * Hkv)))
        totals = sorted(int(rng.integers(1, B * longest + 1)) for _ in range(3))
        counts = [W.auto_splits_ragged(B, Hkv, longest, t) for t in totals]
        assert all(plain <= c <= min(256, max(most, plain)) for c in counts)
        assert counts[0] >= counts[1] >= counts[2]
        assert W.auto_splits_ragged(B, Hkv, longest, (3 * B * longest + 3) // 4) == plain


def test_argument_errors_are_reported_without_a_gpu(lib):
    from paper_2605_02262_amd import binding as W
    h = C.c_void_p()
    fake_ws = C.c_void_p(0x1000)          # never dereferenced: every call below fails validation first
    assert lib.wq_create(C.byref(h), None, fake_ws, 1 << 20) == 0
    try:
        one = C.c_void_p(0x2000)
        # unknown dtype
        rc = lib.wq_window_scores(h, one, one, 7, 1, 64, one, one, one, one, 10, 10, 1, 0, one)
        assert rc == -1 and b"dtype" in lib.wq_last_error(h)
        # matrix-core scoring refuses fp32
        rc = lib.wq_window_scores(h, one, one, W.F32, 1, 64, one, one, one, one, 10, 10, 1, W.SCORE_PAIRWISE_MFMA, one)
        assert rc == -2
        # bad top_bits / too many windows
        assert lib.wq_assign_bits(h, one, 1, one, 8, 0, one, None, 4, 1, one, one, one) == -1
        assert lib.wq_assign_bits(h, one, 1, one, 10000, 0, one, None, 8, 1, one, one, one) == -2
        assert lib.wq_assign_bits(h, one, 1, one, 8, 0, None, None, 8, 1, one, one, one) == -1   # quota mode, no quotas
        # packed descriptor checks
        d = W._PackedKV()
        d.B, d.Hkv, d.hd, d.group, d.dtype16 = 1, 4, 128, 64, W.BF16
        for c in range(3):
            d.cap[c] = 33                                               # not a multiple of 32
        rc = lib.wq_reorder_quantize(h, one, one, W.BF16, 1, one, one, one, one, one, 10, C.byref(d))
        assert rc == -1 and b"multiple of 32" in lib.wq_last_error(h)
        for c in range(3):
            d.cap[c] = 64
            d.codes[c] = 0x3000
            d.meta[c] = 0x3000
            d.cls_off[c] = 0x3000
            d.cls_len[c] = 0x3000
        d.off16, d.len16 = 0x3000, 0x3000
        assert lib.wq_decode_attention(h, one, W.BF16, 1, 28, C.byref(d), 0.1, 0, 100, 0, one, None) == -1
        assert b"v_scale_max" in lib.wq_last_error(h)
        d.v_scale_max = 0x3000
        d.hd = 96
        assert lib.wq_decode_attention(h, one, W.BF16, 1, 28, C.byref(d), 0.1, 0, 100, 0, one, None) == -2
        d.hd = 128
        assert lib.wq_decode_attention(h, one, W.BF16, 1, 30, C.byref(d), 0.1, 0, 100, 0, one, None) == -2  # Hq % Hkv
        assert lib.wq_decode_attention(h, one, W.BF16, 2, 28, C.byref(d), 0.1, 0, 100, 0, one, None) == -1  # B mismatch
        assert lib.wq_reorder_quantize(h, one, one, W.F16, 1, one, one, one, one, one, 10, C.byref(d)) == -1  # dtype16
        # dequantize: descriptors must agree; the two 16-bit segments must differ; the probe checks its sizes
        d.k16, d.v16, d.cap16 = 0x4000, 0x5000, 64
        d2 = W._PackedKV()
        C.memmove(C.byref(d2), C.byref(d), C.sizeof(d))
        assert lib.wq_dequantize(h, 1, C.byref(d), C.byref(d2)) == -1 and b"share" in lib.wq_last_error(h)
        d2.k16, d2.v16 = 0x6000, 0x7000
        d2.dtype16 = W.F16
        assert lib.wq_dequantize(h, 1, C.byref(d), C.byref(d2)) == -1 and b"differ" in lib.wq_last_error(h)
        assert lib.wq_dequantize(h, 1, C.byref(d), None) == -1
        assert lib.wq_probe_mfma(h, 1, 0, 10, None) == -1
        # the one-call decode step: new rows must match the cache's 16-bit type family, no partials-only, same checks as decode
        app = lambda new_dt, algo=0, Hq=28, kn=one: lib.wq_decode_append_attention(h, one, W.BF16, 1, Hq, C.byref(d), kn, one, new_dt,
                                                                                  0.1, 0, 100, algo, one, None)
        assert app(W.F16) == -1 and b"dtype16" in lib.wq_last_error(h)
        assert app(W.BF16, W.DECODE_PARTIALS_ONLY) == -1
        assert app(W.BF16, 0, 30) == -2
        assert app(W.BF16, 0, 28, None) == -1 and b"k_new" in lib.wq_last_error(h)
        assert app(9) == -1
        # splits by length need the longest sequence's length
        assert lib.wq_decode_attention(h, one, W.BF16, 1, 28, C.byref(d), 0.1, 0, 0, W.DECODE_BY_LENGTH, one, None) == -1
        assert b"max_seq_tokens" in lib.wq_last_error(h)
        # workspace too small
        h2 = C.c_void_p()
        assert lib.wq_create(C.byref(h2), None, fake_ws, 512) == 0
        assert lib.wq_decode_attention(h2, one, W.BF16, 1, 28, C.byref(d), 0.1, 64, 100, 0, one, None) == -4
        assert lib.wq_decode_append_attention(h2, one, W.BF16, 1, 28, C.byref(d), one, one, W.BF16, 0.1, 64, 100, 0, one, None) == -4
        lib.wq_destroy(h2)
        # empty batch is a no-op
        d.B = 0
        assert lib.wq_decode_attention(h, one, W.BF16, 0, 28, C.byref(d), 0.1, 0, 0, 0, None, None) == 0
        assert lib.wq_decode_append_attention(h, one, W.BF16, 0, 28, C.byref(d), None, None, W.BF16, 0.1, 0, 0, 0, None, None) == 0
    finally:
        lib.wq_destroy(h)


def test_layer_thresholds_match_the_oracle_and_reject_bad_input(lib):
    """Host-only call (Sec. 3.2.3 threshold functions): compared with the fp64 oracle, which the CPU pins tie to
    the closed forms."""
    import numpy as np
    from oracle import wq_oracle as O
    from paper_2605_02262_amd import binding as W
    s = np.concatenate([[0.0, 1.0, 0.5, 1e-12], np.random.default_rng(3).random(28)])
    lo, hi = W.wq_layer_thresholds(s, 1e-9)                # the written-out quotient cancels here; the limit is s
    assert np.abs(np.asarray(lo) - s).max() <= 1e-6 and np.abs(np.asarray(hi) - s).max() <= 1e-6
    for alpha in (0.0, 0.5, 2.0, 8.0, -1.0):
        lo, hi = W.wq_layer_thresholds(s, alpha)
        lo_o, hi_o = O.layer_thresholds(s, alpha)
        assert np.abs(np.asarray(lo) - lo_o).max() <= 1e-7
        assert np.abs(np.asarray(hi) - hi_o).max() <= 1e-7
    lo, hi = W.wq_layer_thresholds([0.0, 1.0], 2.0)
    assert lo == [0.0, 1.0] and hi == [0.0, 1.0]
    for bad in ([1.5], [-0.1], [float("nan")]):
        with pytest.raises(W.WQError):
            W.wq_layer_thresholds(bad, 2.0)
    with pytest.raises(W.WQError):
        W.wq_layer_thresholds([0.5], float("inf"))
    # vote: size checks before any launch
    h = C.c_void_p()
    assert lib.wq_create(C.byref(h), None, C.c_void_p(0x1000), 1 << 21) == 0
    one = C.c_void_p(0x2000)
    assert lib.wq_vote_bits(h, one, 1, one, 10000, one, one, one) == -2
    assert lib.wq_vote_bits(h, None, 1, one, 8, one, one, one) == -1
    assert lib.wq_vote_bits(h, one, 0, one, 8, one, one, one) == 0
    lib.wq_destroy(h)
