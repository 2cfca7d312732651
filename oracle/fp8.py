"""Weight-only 8-bit storage (a step beyond the paper, for the decode passes that its
method leaves untouched, Appendix "Token Reuse Mechanism", last paragraph): every weight
matrix row (one output feature) is stored as OCP e4m3 codes (1 sign, 4 exponent bits with
bias 7, 3 mantissa bits; no infinities, 0x7f / 0xff are NaN, largest value 448, subnormals
down to 2^-9) times a power-of-two scale per row.  Plain definitions, test infrastructure
only: nothing in the product path may import this.

    value(code)    the number a code stands for
    round_e4m3(x)  nearest representable value, ties to the even mantissa
    quantize_rows  scale_n = the smallest power of two with max|w_n| / scale_n <= 448,
                   codes = round_e4m3(w / scale), and the dequantised matrix
"""
import numpy as np


def value(code):
    code = int(code)
    sign = -1.0 if code & 0x80 else 1.0
    e, m = (code >> 3) & 0xF, code & 0x7
    if e == 0xF and m == 0x7:
        return float("nan")
    if e == 0:
        return sign * (m / 8.0) * 2.0 ** -6
    return sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)


# the 127 finite non-negative values in code order (= ascending order)
_POS = np.array([value(c) for c in range(127)], dtype=np.float64)


def encode(x):
    """Code of the representable value nearest to x (|x| <= 448); of two equally near
    values the one with the even mantissa, i.e. the even code."""
    a = abs(float(x))
    assert a <= 448.0
    best, best_d = 0, None
    for c in range(127):
        d = abs(_POS[c] - a)
        if best_d is None or d < best_d or (d == best_d and c % 2 == 0 and best % 2 == 1):
            best, best_d = c, d
    return best | (0x80 if (x < 0 or (x == 0 and np.signbit(x))) else 0)


def encode_array(x):
    """encode() for arrays, by binary search over the value table instead of a scan."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    assert np.all(a <= 448.0)
    hi = np.clip(np.searchsorted(_POS, a, side="left"), 0, 126)        # first value >= a
    lo = np.clip(hi - 1, 0, 126)
    d_hi, d_lo = _POS[hi] - a, a - _POS[lo]
    take_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(take_lo, lo, hi).astype(np.uint8)
    return code | np.where(np.signbit(x), 0x80, 0).astype(np.uint8)


def decode_array(codes):
    table = np.array([value(c) for c in range(256)], dtype=np.float64)
    return table[np.asarray(codes, dtype=np.uint8)]


def row_scales(w):
    """Per row the smallest power of two s with max|w_row| / s <= 448 (1 for a zero row)."""
    m = np.abs(np.asarray(w, dtype=np.float64)).max(axis=1)
    s = np.ones_like(m)
    nz = m > 0
    e = np.ceil(np.log2(m[nz] / 448.0))
    # log2 is inexact near powers of two: settle the two candidates by the definition
    e = np.where(m[nz] / 2.0 ** (e - 1) <= 448.0, e - 1, e)
    e = np.where(m[nz] / 2.0 ** e <= 448.0, e, e + 1)
    s[nz] = 2.0 ** e
    return s


def quantize_rows(w):
    """Returns (codes uint8 [N, K], scales fp64 [N], dequantised fp64 [N, K])."""
    w = np.asarray(w, dtype=np.float64)
    s = row_scales(w)
    codes = encode_array(w / s[:, None])
    return codes, s, decode_array(codes) * s[:, None]
