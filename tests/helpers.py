"""Small independent helpers for the tests (exact rational rounding, golden file reader)."""
from fractions import Fraction
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


def round_f32(x: Fraction) -> np.float32:
    """Round an exact rational to the nearest binary32 (ties to even); normal range only."""
    if x == 0:
        return np.float32(0.0)
    sign = -1 if x < 0 else 1
    a = abs(x)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    assert -126 <= e <= 126
    q = a / Fraction(2) ** (e - 23)  # in [2^23, 2^24)
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    return np.float32(sign * float(n) * 2.0 ** (e - 23))


def f32_mul(a, b) -> np.float32:
    return round_f32(Fraction(float(a)) * Fraction(float(b)))


def f32_fma(a, b, c) -> np.float32:
    return round_f32(Fraction(float(a)) * Fraction(float(b)) + Fraction(float(c)))


def topk_reference(scores: np.ndarray, passing: np.ndarray, K: int):
    """Plain selection with numpy: score descending, ties by lower id (lexsort is stable)."""
    ids = np.nonzero(passing)[0]
    s = scores[ids]
    order = np.lexsort((ids, -s.astype(np.float64)))
    ids, s = ids[order][:K], s[order][:K]
    out_i = np.full(K, -1, dtype=np.int64)
    out_s = np.full(K, -np.inf, dtype=np.float32)
    out_i[: ids.size] = ids
    out_s[: ids.size] = s
    return out_i, out_s, ids.size
