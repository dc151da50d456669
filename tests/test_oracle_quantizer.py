"""Pins of the oracle's quantizer against what Eq. 2-3 (Section 3.2) and the
error-bound proof (Appendix A) fix.  CPU only."""
import numpy as np
import pytest

from oracle import mixkvq_oracle as O


def _groups(rng, n_groups, G, kind):
    if kind == "normal":
        x = rng.standard_normal((n_groups, G))
    elif kind == "outlier":
        x = rng.standard_normal((n_groups, G))
        x[np.arange(n_groups), rng.integers(0, G, n_groups)] *= 300.0
    elif kind == "extreme":
        x = rng.choice([65504.0, -65504.0, 0.0, 1.0], size=(n_groups, G))
    elif kind == "subnormal":
        x = rng.integers(-40, 40, size=(n_groups, G)) * 2.0 ** -24
    elif kind == "constant":
        x = np.repeat(rng.standard_normal((n_groups, 1)), G, axis=1)
    elif kind == "tiny_range":
        base = rng.standard_normal((n_groups, 1))
        x = base + rng.integers(0, 3, size=(n_groups, G)) * 2.0 ** -12
    return x.astype(np.float16)


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("kind", ["normal", "outlier", "extreme", "subnormal", "constant", "tiny_range"])
def test_error_bound_half_scale(bits, kind):
    """Appendix A: |x - x~| <= s/2.  With the stored fp16 scale the end of the
    range can fall short by (2^B-1)|s16 - s32| <= (2^B-1) 2^-25 when s16 is
    subnormal; inside the range the binary32 quotient adds a relative 2^-22."""
    rng = np.random.default_rng(1)
    x = _groups(rng, 500, 32, kind)
    s16, z16 = O.group_params(x, bits, axis=1)
    c = O.encode(x, s16[:, None], z16[:, None], bits)
    xt = O.decode(c, s16[:, None], z16[:, None])
    err = np.abs(x.astype(np.float64) - xt)
    bound = s16.astype(np.float64)[:, None] * 0.5 * (1 + 1e-5) + ((1 << bits) - 1) * 2.0 ** -25
    assert np.all(err <= bound), float((err - bound).max())
    assert c.max() <= (1 << bits) - 1


@pytest.mark.parametrize("bits", [2, 4])
def test_endpoints_and_monotone(bits):
    rng = np.random.default_rng(2)
    x = _groups(rng, 300, 64, "normal")
    s16, z16 = O.group_params(x, bits, axis=1)
    c = O.encode(x, s16[:, None], z16[:, None], bits)
    rows = np.arange(x.shape[0])
    # zero-point is the group minimum (Eq. 2), and it maps to code 0; the maximum maps to the top code
    assert np.array_equal(z16, x.min(axis=1))
    assert np.all(c[rows, x.argmin(axis=1)] == 0)
    assert np.all(c[rows, x.argmax(axis=1)] == (1 << bits) - 1)
    # codes are monotone in x inside a group
    order = np.argsort(x, axis=1, kind="stable")
    cs = np.take_along_axis(c, order, axis=1).astype(np.int64)
    assert np.all(np.diff(cs, axis=1) >= 0)


def test_scale_is_range_over_levels():
    """s = (max - min) / (2^B - 1), Section 3.2, to fp16 rounding."""
    rng = np.random.default_rng(3)
    x = _groups(rng, 200, 128, "normal")
    for bits in (2, 4):
        s16, _ = O.group_params(x, bits, axis=1)
        exact = (x.max(axis=1).astype(np.float64) - x.min(axis=1).astype(np.float64)) / ((1 << bits) - 1)
        assert np.all(np.abs(s16.astype(np.float64) - exact) <= exact * 2.0 ** -11 + 2.0 ** -25)
    s2, _ = O.group_params(x, 2, axis=1)
    s4, _ = O.group_params(x, 4, axis=1)
    # 4-bit error bound is a fifth of the 2-bit one (15 levels against 3)
    assert np.allclose(s4.astype(np.float64) * 5, s2.astype(np.float64), rtol=2e-3)


def test_matches_textbook_float64_quantizer():
    """With no salient channel the scheme is the plain asymmetric min/max
    quantizer.  An independent float64 rendering of Eq. 2 may differ by one code
    only where (x - z)/s sits within fp16-scale rounding of a half-integer."""
    rng = np.random.default_rng(4)
    x = _groups(rng, 400, 32, "normal")
    xf = x.astype(np.float64)
    mn, mx = xf.min(axis=1, keepdims=True), xf.max(axis=1, keepdims=True)
    s = (mx - mn) / 3.0
    ref = np.clip(np.floor((xf - mn) / s + 0.5), 0, 3).astype(np.int64)
    s16, z16 = O.group_params(x, 2, axis=1)
    c = O.encode(x, s16[:, None], z16[:, None], 2).astype(np.int64)
    diff = np.abs(c - ref)
    assert diff.max() <= 1
    assert (diff != 0).mean() < 5e-3
    y = (xf - mn) / s
    assert np.all(np.abs(y[diff != 0] - np.floor(y[diff != 0]) - 0.5) < 5e-3)


def test_round_half_to_even():
    """Ties of Eq. 2's round() go to the even code: x exactly between two levels."""
    # group {0, 3} -> s = 1, z = 0; 0.5 -> 0, 1.5 -> 2, 2.5 -> 2
    x = np.array([[0.0, 3.0, 0.5, 1.5, 2.5, 1.0]], dtype=np.float16)
    s16, z16 = O.group_params(x, 2, axis=1)
    assert float(s16[0]) == 1.0 and float(z16[0]) == 0.0
    c = O.encode(x, s16[:, None], z16[:, None], 2)
    assert c.tolist() == [[0, 3, 0, 2, 2, 1]]


def test_negative_zero_zero_point_is_canonical():
    x = np.array([[-0.0, 0.0, 1.0, 3.0]], dtype=np.float16)
    _, z16 = O.group_params(x, 2, axis=1)
    assert z16.view(np.uint16)[0] == 0


def test_key_groups_run_along_tokens_value_groups_along_channels():
    """Section 4.2: keys per channel, values per token.  A key tensor constant
    along tokens and a value tensor constant along channels are then exact;
    the transposed grouping would not be."""
    L, D = 64, 32
    K = np.tile(np.linspace(-4, 4, D, dtype=np.float32)[None, :], (L, 1)).astype(np.float16)
    V = np.tile(np.linspace(-4, 4, L, dtype=np.float32)[:, None], (1, D)).astype(np.float16)
    codes, s, z = O.quantize_keys(K, np.arange(D), 2, 32)
    assert np.all(codes == 0) and np.all(s == 0)
    assert np.array_equal(O.decode(codes, np.repeat(s, 32, 0), np.repeat(z, 32, 0)), K.astype(np.float64))
    vc, vs, vz = O.quantize_values(V, 16)
    assert np.all(vc == 0) and np.all(vs == 0)
    assert np.array_equal(O.decode(vc, np.repeat(vs, 16, 1), np.repeat(vz, 16, 1)), V.astype(np.float64))
    # and the other way round they are NOT exact
    kc2, ks2, _ = O.quantize_keys(V, np.arange(D), 2, 32)
    assert ks2.max() > 0


def test_key_groups_restart_every_gk_tokens():
    rng = np.random.default_rng(5)
    K = rng.standard_normal((96, 8)).astype(np.float16)
    codes, s, z = O.quantize_keys(K, np.arange(8), 2, 32)
    for gidx in range(3):
        sub = K[32 * gidx:32 * (gidx + 1)]
        assert np.array_equal(z[gidx], sub.min(axis=0))
        c2, s2, z2 = O.quantize_keys(sub, np.arange(8), 2, 32)
        assert np.array_equal(c2, codes[32 * gidx:32 * (gidx + 1)])
        assert np.array_equal(s2[0], s[gidx])


def test_bfloat16_inputs_enter_as_nearest_binary16():
    """bfloat16 -> binary16: exact wherever binary16 has the range (8 significant bits fit into 11), the nearest
    value with ties to even inside the binary16 subnormals, saturated at +-65504.  Checked for every finite
    bfloat16 pattern against exact rational arithmetic."""
    from fractions import Fraction
    bits = np.arange(1 << 16, dtype=np.uint32)
    exp = (bits >> 7) & 0xFF
    bits = bits[exp != 0xFF].astype(np.uint16)                     # finite patterns
    got = O.bf16_bits_to_f16(bits)
    assert got.dtype == np.float16 and np.all(np.isfinite(got))
    x32 = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    normal_range = (np.abs(x32) >= 2.0 ** -14) & (np.abs(x32) <= 65504.0)
    assert np.array_equal(got[normal_range].astype(np.float64), x32[normal_range])          # exact
    big = np.abs(x32) > 65504.0
    assert np.array_equal(got[big].astype(np.float64), np.sign(x32[big]) * 65504.0)         # saturated
    # below the normal range: a multiple of 2^-24, nearest to x, ties to the even multiple
    small = np.nonzero((np.abs(x32) < 2.0 ** -14) & (x32 != 0))[0]
    for i in small[:: max(1, len(small) // 400)]:
        x = Fraction(float(x32[i]))
        n = Fraction(float(got[i])) * (1 << 24)
        assert n.denominator == 1
        d = abs(x * (1 << 24) - n)
        assert d <= Fraction(1, 2) and (d < Fraction(1, 2) or n.numerator % 2 == 0)
    assert O.bf16_bits_to_f16(np.array([0x0000, 0x8000], dtype=np.uint16)).view(np.uint16).tolist() == [0x0000, 0x8000]
