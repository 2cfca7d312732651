"""Pins of the oracle's e4m3 weight quantiser: the format's published table through an
independent library routine (torch.float8_e4m3fn), hand-worked ties, closed forms.  CPU only."""
import numpy as np
import torch

from oracle import fp8 as Q


def test_code_table_is_ocp_e4m3():
    codes = torch.arange(256, dtype=torch.uint8)
    want = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy()
    got = np.array([Q.value(c) for c in range(256)])
    assert np.array_equal(np.isnan(got), np.isnan(want)) and np.isnan(got).sum() == 2
    ok = ~np.isnan(got)
    assert np.array_equal(got[ok], want[ok].astype(np.float64))
    assert Q.value(0x7E) == 448.0 and Q.value(0x01) == 2.0 ** -9 and Q.value(0x08) == 2.0 ** -6
    assert Q.value(0x38) == 1.0 and Q.value(0xB8) == -1.0


def test_rounding_ties_and_extremes_by_hand():
    v = lambda x: Q.value(Q.encode(x))
    assert v(1.0625) == 1.0          # halfway 1.000|1.125: mantissa 000 is even
    assert v(1.1875) == 1.25         # halfway 1.125|1.250: mantissa 010 is even
    assert v(1.06251) == 1.125 and v(1.06249) == 1.0
    assert v(2.0 ** -10) == 0.0      # halfway 0 | 2^-9: zero is even
    assert v(3 * 2.0 ** -10) == 2.0 ** -8
    assert v(15 * 2.0 ** -10) == 2.0 ** -6   # halfway between the largest subnormal and the smallest normal
    assert v(448.0) == 448.0 and v(-448.0) == -448.0 and v(447.9) == 448.0 and v(431.9) == 416.0
    assert v(1.9375 * 2) == 4.0      # rounding up carries into the exponent
    for c in list(range(127)) + list(range(128, 255)):
        assert Q.encode(Q.value(c)) == c or (c == 128 and Q.encode(-0.0) == 128)


def test_array_encoder_equals_the_scan_and_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4000) * 30, rng.standard_normal(2000) * 0.01,
                        (Q._POS[:-1] + Q._POS[1:]) / 2, -(Q._POS[:-1] + Q._POS[1:]) / 2, Q._POS, [0.0, -0.0]])
    x = np.clip(x, -448, 448)
    fast = Q.encode_array(x)
    assert all(int(fast[i]) == Q.encode(x[i]) for i in range(len(x)))
    # torch casts fp32 -> e4m3fn with round-to-nearest-even too
    t = torch.tensor(x, dtype=torch.float32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    x32 = x.astype(np.float32).astype(np.float64)                       # what torch saw
    assert np.array_equal(Q.encode_array(x32), t)


def test_row_scales_and_round_trip():
    w = np.array([[448.0, 1.0], [448.0 * 1.0001, 1.0], [0.1, -0.05], [0.0, 0.0], [2.0 ** -20, 0.0],
                  [3.5 * 2.0 ** -7, 0.0]])
    s = Q.row_scales(w)
    assert s.tolist() == [1.0, 2.0, 2.0 ** -12, 1.0, 2.0 ** -28, 2.0 ** -14]
    assert np.all(np.abs(w).max(axis=1) / s <= 448.0)
    assert np.all((np.abs(w).max(axis=1) / s > 224.0) | (np.abs(w).max(axis=1) == 0))
    codes, s, deq = Q.quantize_rows(w)
    assert deq[0].tolist() == [448.0, 1.0] and deq[3].tolist() == [0.0, 0.0]
    rng = np.random.default_rng(1)
    w = rng.standard_normal((64, 300)) * 0.02
    codes, s, deq = Q.quantize_rows(w)
    # the relative error of a normal e4m3 value is at most 2^-4; values already on the grid come back
    big = np.abs(w) >= s[:, None] * 2.0 ** -6
    assert np.all(np.abs(deq - w)[big] <= np.abs(w)[big] * 2.0 ** -4)
    assert np.all(np.abs(deq - w)[~big] <= s[:, None].repeat(300, 1)[~big] * 2.0 ** -10)
    assert np.array_equal(Q.quantize_rows(deq)[2], deq)
