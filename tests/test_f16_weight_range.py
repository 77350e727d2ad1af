"""Range and rounding of the f16 softmax weights of the matrix-core decode kernel, emulated in numpy (CPU only).

The kernel multiplies a token's softmax weight with its value group's scale and rounds the product to f16 before the value
product (the codes themselves enter exactly).  This file restates that arithmetic for one head and one value channel
(reference exponent that moves when a logit exceeds it by more than 2^5; weights formed 2^up too large, up chosen from the
sequence's largest value scale so that the largest product lies in [2^14, 2^15]; a slot's power of two of up to 2^-6
folded in; f16 with gradual underflow; fp32 sums) and compares it with the exact softmax average in fp64 on the inputs
that stress it: logits rising along the stream, one token far above the rest, equal logits, and values of very different
magnitudes (Sec. 3.3.3 fixes the quantizer; the weights are the decode side's own).  It shares no code with the kernel: it
pins the *analysis* that include/wq.h states (no overflow at any scale, what is lost to underflow cannot be seen in the
result, and why a fixed factor would not do), the GPU tests pin the kernel.
"""
import numpy as np
import pytest

SLACK, TOP = 5.0, 15                 # the kernel's constants, restated: log2 of the largest weight, and of the largest f16 product
BLOCK = 32


def upscale(s_max):
    return float(TOP - SLACK - np.ceil(np.log2(float(s_max))))


def emulate(x_log2, codes, s_v, m_v, slot_shift, UP=None):
    """x_log2 [N] logits in log2 units; codes [N] integer value codes; s_v, m_v [N] the value group's scale and minimum
    (f16-representable); slot_shift [N] in {0, 2, 4, 6}; UP: log2 of the factor the weights are formed with (default: from
    the largest scale, as the kernel does).  Returns (emulated output, largest |f16 weight| seen)."""
    n = len(x_log2)
    if UP is None:
        UP = upscale(s_v.astype(np.float32).max())
    ref, acc, acc_m, l = -np.inf, np.float32(0), np.float32(0), np.float32(0)
    biggest = 0.0
    for b0 in range(0, n, BLOCK):
        xb = x_log2[b0:b0 + BLOCK].astype(np.float32)
        if xb.max() > ref + SLACK:                                   # the reference exponent moves: everything so far is rescaled
            new = max(ref, float(xb.max()))
            alpha = np.float32(0.0) if ref == -np.inf else np.float32(2.0 ** (ref - new))
            acc, acc_m, l, ref = acc * alpha, acc_m * alpha, l * alpha, new
        sh = slot_shift[b0:b0 + BLOCK].astype(np.float32)
        p_slot = np.exp2(xb - np.float32(ref) + np.float32(UP) - sh).astype(np.float32)       # weight with the slot's power of two folded in
        w16 = (p_slot * s_v[b0:b0 + BLOCK].astype(np.float32)).astype(np.float16)             # the f16 operand
        biggest = max(biggest, float(np.abs(w16.astype(np.float64)).max()))
        # the codes sit in the operand as code * 2^(shift - 24): the product undoes the slot's shift exactly
        prod = w16.astype(np.float64) * codes[b0:b0 + BLOCK] * np.exp2(sh.astype(np.float64))
        acc = np.float32(acc + np.float32(prod.sum() * 2.0 ** -UP))
        p = np.exp2(xb - np.float32(ref)).astype(np.float32)
        acc_m = np.float32(acc_m + np.float32((p * m_v[b0:b0 + BLOCK].astype(np.float32)).sum()))
        l = np.float32(l + p.sum())
    return float((acc + acc_m) / l), biggest


def exact(x_log2, codes, s_v, m_v):
    w = np.exp2(x_log2.astype(np.float64) - x_log2.max())
    v = m_v.astype(np.float64) + s_v.astype(np.float64) * codes
    return float((w * v).sum() / w.sum())


def _case(n, seed, s_scale):
    rng = np.random.Generator(np.random.PCG64(seed))
    codes = rng.integers(0, 4, n).astype(np.float64)                                   # 2-bit codes: the widest slot shifts
    s_v = np.full(n, s_scale, np.float16)
    m_v = np.full(n, -1.5 * s_scale, np.float16)
    shift = (2 * rng.integers(0, 4, n)).astype(np.float64)
    return rng, codes, s_v, m_v, shift


@pytest.mark.parametrize("s_scale", [2.0 ** -12, 1.0, 16.0, 2048.0])
def test_rising_logits_keep_the_weights_in_range_and_the_result_accurate(s_scale):
    n = 4096
    rng, codes, s_v, m_v, shift = _case(n, 1, s_scale)
    x = np.linspace(0.0, 40 * SLACK, n) + rng.normal(0, 1.0, n)                          # the reference moves dozens of times
    got, biggest = emulate(x, codes, s_v, m_v, shift)
    want = exact(x, codes, s_v, m_v)
    assert 2.0 ** (TOP - 7) <= biggest <= 2.0 ** TOP
    assert abs(got - want) <= 2e-3 * s_scale * 3.0                                       # (values span 3 scales)


@pytest.mark.parametrize("where", [0, 2000, 4095])
def test_one_token_far_above_the_rest(where):
    n = 4096
    rng, codes, s_v, m_v, shift = _case(n, 2, 1.0)
    x = rng.normal(0, 2.0, n)
    x[where] += 14.0 / np.log(2.0)                                                       # 14 nats above the bulk
    got, biggest = emulate(x, codes, s_v, m_v, shift)
    assert biggest <= 65504.0
    assert abs(got - exact(x, codes, s_v, m_v)) <= 2e-3 * 3.0


def test_equal_logits_over_a_long_stream():
    n = 50688
    rng, codes, s_v, m_v, shift = _case(n, 3, 1.0)
    x = np.zeros(n)
    got, _ = emulate(x, codes, s_v, m_v, shift)
    assert abs(got - exact(x, codes, s_v, m_v)) <= 2e-3 * 3.0


def test_a_fixed_factor_overflows_for_wide_values_and_loses_mass_for_narrow_ones():
    """Why the factor follows the values: with a fixed 2^6 (an earlier build) a scale of 64 overflows f16, and with values
    of scale 2^-8 a bulk of 50 688 tokens 23 octaves below one dominant token, which holds 0.6 % of the mass, is lost from
    the numerator while the denominator counts it."""
    n = 64
    rng, codes, s_v, m_v, shift = _case(n, 4, 64.0)
    x = np.zeros(n); x[40] = SLACK
    shift[:] = 0
    with np.errstate(over="ignore"):
        _, biggest = emulate(x, codes, s_v, m_v, shift, UP=6.0)
    assert not np.isfinite(biggest)
    _, biggest = emulate(x, codes, s_v, m_v, shift)
    assert biggest <= 2.0 ** TOP

    n = 50688
    rng, codes, s_v, m_v, shift = _case(n, 5, 2.0 ** -8)
    x = np.full(n, -23.0); x[0] = 0.0
    shift[:] = 6
    tol = 2e-3 * 3.0 * 2.0 ** -8
    fixed, _ = emulate(x, codes, s_v, m_v, shift, UP=6.0)
    placed, _ = emulate(x, codes, s_v, m_v, shift)
    want = exact(x, codes, s_v, m_v)
    assert abs(fixed - want) > tol
    assert abs(placed - want) <= tol


def test_what_underflows_is_too_small_to_matter():
    # placed by the largest scale, a weight is lost below 2^-29 of the reference in the slot shifted most: 50 688 such
    # tokens hold 1e-4 of the mass
    n = 50688
    rng, codes, s_v, m_v, shift = _case(n, 6, 1.0)
    x = np.full(n, -30.0); x[0] = 0.0
    shift[:] = 6
    got, _ = emulate(x, codes, s_v, m_v, shift)
    assert abs(got - exact(x, codes, s_v, m_v)) <= 2e-3 * 3.0
