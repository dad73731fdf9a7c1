"""Pins for the oracle's 8-bit cache format (OCP FP8 E4M3, nearest-even, saturating) and for attention over it."""
import numpy as np
import torch

from oracle import heatkv_oracle as orc


def test_decode_matches_the_values_the_format_fixes():
    d = orc.fp8_e4m3_decode
    assert d([0x00])[0] == 0.0 and np.signbit(d([0x80])[0]) and d([0x80])[0] == 0.0
    assert d([0x01])[0] == 2.0 ** -9            # smallest subnormal
    assert d([0x07])[0] == 7 * 2.0 ** -9        # largest subnormal
    assert d([0x08])[0] == 2.0 ** -6            # smallest normal
    assert d([0x38])[0] == 1.0 and d([0x39])[0] == 1.125 and d([0xB8])[0] == -1.0
    assert d([0x7E])[0] == 448.0 and d([0xFE])[0] == -448.0
    assert np.isnan(d([0x7F])[0]) and np.isnan(d([0xFF])[0])
    pos = d(np.arange(127, dtype=np.uint8))
    assert np.all(np.diff(pos) > 0)             # codes order the magnitudes
    assert not np.isinf(d(np.arange(256, dtype=np.uint8))).any()


def test_every_code_survives_the_round_trip():
    codes = np.arange(256, dtype=np.uint8)
    finite = ~np.isnan(orc.fp8_e4m3_decode(codes))
    back = orc.fp8_e4m3_encode(orc.fp8_e4m3_decode(codes))
    assert np.array_equal(back[finite], codes[finite])
    assert np.all((back[~finite] & 0x7F) == 0x7F)


def test_ties_saturation_and_underflow_by_hand():
    e = lambda v: int(orc.fp8_e4m3_encode(np.array([v]))[0])
    assert e(1.0625) == 0x38      # halfway between 1.0 (0x38) and 1.125 (0x39): the even code
    assert e(1.1875) == 0x3A      # halfway between 1.125 (0x39) and 1.25 (0x3A): the even code
    assert e(1.0626) == 0x39 and e(1.0624) == 0x38
    assert e(448.0) == 0x7E and e(1e6) == 0x7E and e(-1e6) == 0xFE and e(np.inf) == 0x7E   # saturating
    assert e(2.0 ** -10) == 0x00  # halfway between 0 and the smallest subnormal: the even code, zero
    assert e(2.0 ** -10 * 1.01) == 0x01 and e(-(2.0 ** -9)) == 0x81
    assert e(float("nan")) == 0x7F
    assert e(-0.0) == 0x80


def test_encode_matches_torch_cast_inside_the_finite_range():
    # torch's float8_e4m3fn cast rounds to nearest-even as well (it does not saturate, so stay inside +-448)
    g = torch.Generator().manual_seed(0)
    x = torch.cat([torch.randn(20000, generator=g), torch.randn(5000, generator=g) * 60.0,
                   torch.randn(5000, generator=g) * 2.0 ** -7, torch.randn(2000, generator=g) * 2.0 ** -9])
    x = x[x.abs() <= 448.0].to(torch.bfloat16).float()   # the cache stores bf16 inputs
    want = x.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = orc.fp8_e4m3_encode(x.double().numpy())
    assert np.array_equal(got, want)
    # rounding error: half a step of the 3-bit mantissa at most for normal values
    v = x.double().numpy()
    r = orc.fp8_e4m3_round(v)
    normal = np.abs(v) >= 2.0 ** -6
    assert np.all(np.abs(r - v)[normal] <= np.abs(v)[normal] * 2.0 ** -4)
    assert np.all(np.abs(r - v)[~normal] <= 2.0 ** -10)


def test_attention_over_the_8_bit_cache():
    rng = np.random.default_rng(3)
    t = orc.one_based([2, 3, 5, 4])
    c = orc.cumulative(t)
    d = 8
    q, k, v = (rng.standard_normal((c[-1], d)) for _ in range(3))
    # values that E4M3 holds exactly pass through unchanged: same result as the full-precision path
    k8, v8 = orc.fp8_e4m3_round(k), orc.fp8_e4m3_round(v)
    kk, vv = k8.copy(), v8.copy()
    got = orc.attend_scale_fp8_cache(q, kk, vv, t, 4, [1, 3], 0.3)
    assert np.array_equal(got, orc.attend_scale(q, k8, v8, t, 4, [1, 3], 0.3))
    # in general: the retained rows are rounded, the current scale's rows are not
    got = orc.attend_scale_fp8_cache(q, k, v, t, 4, [1, 3], 0.3)
    km, vm = k.copy(), v.copy()
    km[:c[3]], vm[:c[3]] = k8[:c[3]], v8[:c[3]]
    assert np.array_equal(got, orc.attend_scale(q, km, vm, t, 4, [1, 3], 0.3))
    assert not np.array_equal(got, orc.attend_scale(q, k8, v8, t, 4, [1, 3], 0.3))  # rounding the current scale too differs
    assert np.abs(got - orc.attend_scale(q, k, v, t, 4, [1, 3], 0.3)).max() < 0.2
