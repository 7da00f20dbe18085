"""Pins of the oracle's publish-time quantisation (paper Sec. 4.2): hand-worked values, the
rounding error bound, extremes and special tables.  CPU only."""
from fractions import Fraction

import numpy as np

from oracle import st_oracle as O
from tests.helpers import round_f32


def test_hand_worked_table():
    # a = 2, s = 2/127: 2 -> 127, -2 -> -127, 0 -> 0, 1 -> 63.5 -> 64 (tie to even),
    # 0.5 -> 31.75 -> 32, -1 -> -63.5 -> -64, 1.99 -> 126.365 -> 126, 3/127*... below
    x = np.array([[2.0, -2.0, 0.0, 1.0], [0.5, -1.0, 1.99, -0.0078125]], dtype=np.float32)
    q, rs, (mn, mx) = O.quantize_global(x)
    assert (mn, mx) == (-2.0, 2.0)
    s = round_f32(Fraction(2) / Fraction(127))
    assert rs.tolist() == [float(s), float(s)]
    # -0.0078125 / s = -0.49609... -> 0
    assert q.tolist() == [[127, -127, 0, 64], [32, -64, 126, 0]]


def test_asymmetric_range_uses_the_larger_magnitude():
    x = np.array([[-3.0, 1.0, 0.25]], dtype=np.float32)
    q, rs, (mn, mx) = O.quantize_global(x)
    assert (mn, mx) == (-3.0, 1.0)
    assert q[0, 0] == -127 and q[0, 1] == 42  # 1 / (3/127) = 42.33
    assert q[0, 2] == 11                      # 10.58 -> 11
    x = np.array([[0.5, 4.0]], dtype=np.float32)
    q, _, _ = O.quantize_global(x)
    assert q.tolist() == [[16, 127]]          # 0.5 / (4/127) = 15.875


def test_error_bound_order_and_sign_symmetry():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((300, 48)) * 0.37).astype(np.float32)
    q, rs, (mn, mx) = O.quantize_global(x)
    s = rs[0]
    assert (rs == s).all() and mn == x.min() and mx == x.max()
    a = max(abs(mn), abs(mx))
    assert abs(float(s) - a / 127.0) <= 1e-7 * a
    # reconstruction within half a step (plus rounding of the division)
    err = np.abs(x.astype(np.float64) - q.astype(np.float64) * float(s))
    assert err.max() <= 0.5 * float(s) * (1 + 1e-5)
    assert np.abs(q).max() == 127 and q.min() >= -127
    # order preserved (weakly), sign symmetric
    flat, fq = x.reshape(-1), q.reshape(-1)
    order = np.argsort(flat, kind="stable")
    assert (np.diff(fq[order].astype(np.int32)) >= 0).all()
    q2, _, _ = O.quantize_global(-x)
    assert np.array_equal(q2, -q)


def test_zero_table_and_empty_table():
    q, rs, mm = O.quantize_global(np.zeros((3, 4), np.float32))
    assert (q == 0).all() and (rs == 1.0).all() and mm == (0.0, 0.0)
    q, rs, mm = O.quantize_global(np.zeros((0, 16), np.float32))
    assert q.shape == (0, 16) and rs.size == 0 and mm == (0.0, 0.0)


def test_quantised_inner_product_tracks_the_real_one():
    # the reason for the exercise: dot(q_a, q_b) * s_a * s_b approximates dot(a, b); with both
    # errors at most half a step the difference is bounded by d * (s/2) * (|a|max + |b|max + s/2)
    rng = np.random.default_rng(6)
    a = rng.standard_normal((40, 64)).astype(np.float32)
    b = rng.standard_normal((30, 64)).astype(np.float32)
    qa, sa, _ = O.quantize_global(a)
    qb, sb, _ = O.quantize_global(b)
    approx = (qa.astype(np.int32) @ qb.astype(np.int32).T).astype(np.float64) * float(sa[0]) * float(sb[0])
    exact = a.astype(np.float64) @ b.astype(np.float64).T
    bound = 64 * (0.5 * float(sa[0]) * np.abs(b).max() + 0.5 * float(sb[0]) * np.abs(a).max()
                  + 0.25 * float(sa[0]) * float(sb[0])) * (1 + 1e-4)
    assert np.abs(approx - exact).max() <= bound
