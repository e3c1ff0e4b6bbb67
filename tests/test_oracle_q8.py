"""Pins of the 8-bit cache format of oracle/q8.py: the code table and the rounding against an independent
library routine (PyTorch's CPU float8_e4m3fn cast), closed forms of the format, and the scale rule."""
import numpy as np
import pytest
import torch

from oracle import q8


def test_decode_table_matches_the_library_type():
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    t = q8.e4m3_decode_table()
    assert np.array_equal(np.isnan(t), np.isnan(ref)) and np.isnan(t).sum() == 2
    ok = ~np.isnan(t)
    assert np.array_equal(t[ok], ref[ok])
    assert np.array_equal(np.signbit(t[ok]), np.signbit(ref[ok]))        # code 0x80 is -0


def test_format_closed_forms():
    t = q8.e4m3_decode_table()
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0                        # largest finite
    assert t[0x01] == 2.0 ** -9 and t[0x08] == 2.0 ** -6                 # smallest subnormal, smallest normal
    assert t[0x38] == 1.0 and t[0x39] == 1.125
    pos = t[:0x7F]
    assert (np.diff(pos) > 0).all()                                      # value order = code order
    # every finite code survives a round trip, both signs
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    assert np.array_equal(q8.e4m3_encode(t[codes]), codes)


def test_rounding_is_nearest_with_ties_to_even():
    pos = q8.e4m3_decode_table()[:0x7F]
    for c in range(0x7E):
        lo, hi = pos[c], pos[c + 1]
        mid = 0.5 * (lo + hi)                                            # exact in float64
        even = c if c % 2 == 0 else c + 1
        assert q8.e4m3_encode(np.array([mid]))[0] == even
        assert q8.e4m3_encode(np.array([np.nextafter(mid, lo)]))[0] == c
        assert q8.e4m3_encode(np.array([np.nextafter(mid, hi)]))[0] == c + 1
        assert q8.e4m3_encode(np.array([-mid]))[0] == (even | 0x80)
    assert q8.e4m3_encode(np.array([1e9, -1e9, 448.0, 463.9]))[[0, 1, 2, 3]].tolist() == [0x7E, 0xFE, 0x7E, 0x7E]   # saturation
    assert q8.e4m3_encode(np.array([-0.0, -1e-9, 1e-9])).tolist() == [0x80, 0x80, 0x00]                             # the sign survives


def test_encode_matches_the_library_cast_in_range():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(200000) * 50.0, rng.standard_normal(100000) * 0.01, rng.uniform(-448, 448, 100000)])
    x = x[np.abs(x) <= 448.0].astype(np.float32)                         # the library cast does not saturate beyond the range
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = q8.e4m3_encode(x.astype(np.float64))
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("amax,expect", [(448.0, 1.0), (448.0001, 2.0), (224.0, 0.5), (224.0001, 1.0), (1.0, 2.0 ** -8), (0.0, 1.0), (3.5e-7, None)])
def test_scale_rule(amax, expect):
    s = float(q8.row_scale(np.array(amax)))
    assert s == 2.0 ** round(np.log2(s))                                 # a power of two
    if amax > 0:
        assert 224.0 < amax / s <= 448.0
    if expect is not None:
        assert s == expect


def test_quantized_rows_stay_within_half_a_step():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((64, 512)) * rng.uniform(0.01, 30.0, (64, 1))
    x[3] = 0.0
    codes, s = q8.quantize_rows(x)
    y = q8.dequantize_rows(codes, s)
    assert np.array_equal(y[3], np.zeros(512)) and s[3] == 1.0
    # normal codes: relative error at most 2^-4 (half of a 3-bit mantissa step); subnormal codes: at most 2^-10 of the scale
    err = np.abs(y - x)
    bound = np.maximum(np.abs(x) * 2.0 ** -4, s[:, None] * 2.0 ** -10)
    assert (err <= bound).all()
    # the largest element of every row uses the top binade
    assert ((np.abs(codes.astype(np.int32) & 0x7F)).max(axis=1)[np.arange(64) != 3] >= 0x70).all()
