"""Pins for the oracle's PWL table builder (Section 3.2, Post-Training Approximation; Algorithm 3
step 1) against closed forms: end-point interpolation, the analytic chord error bound, exact
reproduction of affine functions, exact ReLU."""
import math

import numpy as np
import pytest
from scipy.special import erf

CASES = [  # func name, lo, hi
    ("gelu", -8.0, 8.0),
    ("exp", -16.0, 0.0),
    ("recip", 1.0, 64.0),
    ("recip", 1.0, 512.0),
    ("rsqrt", 1e-3, 64.0),
    ("sqrt", 0.25, 64.0),
]


def truth(name, x):
    x = np.asarray(x, np.float64)
    if name == "gelu":
        return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))
    if name == "exp":
        return np.exp(x)
    if name == "recip":
        return 1.0 / x
    if name == "rsqrt":
        return x ** -0.5
    if name == "sqrt":
        return np.sqrt(x)
    raise KeyError(name)


def second_derivative_max(name, a, b):
    """max |f''| over [a, b] from the closed forms."""
    if name == "exp":
        return math.exp(b)
    if name == "recip":
        return 2.0 / a ** 3
    if name == "rsqrt":
        return 0.75 * a ** -2.5
    if name == "sqrt":
        return 0.25 * a ** -1.5
    if name == "gelu":
        # f'' = phi(x) (2 - x^2); its derivative vanishes at 0 and +-2
        pts = [a, b] + [c for c in (0.0, 2.0, -2.0) if a <= c <= b]
        phi = lambda x: math.exp(-0.5 * x * x) / math.sqrt(2 * math.pi)  # noqa: E731
        return max(abs(phi(x) * (2 - x * x)) for x in pts)
    raise KeyError(name)


def func_id(O, name):
    return {"gelu": O.F_GELU, "exp": O.F_EXP, "recip": O.F_RECIP, "rsqrt": O.F_RSQRT,
            "sqrt": O.F_SQRT, "relu": O.F_RELU, "identity": O.F_IDENTITY}[name]


@pytest.mark.parametrize("name,lo,hi", CASES)
@pytest.mark.parametrize("nseg", [1, 7, 64, 128, 256])
def test_chord_interpolates_end_points(oracle, name, lo, hi, nseg):
    t = oracle.build_table(func_id(oracle, name), lo, hi, nseg)
    L, R = float(np.float32(lo)), float(np.float32(hi))
    w = (R - L) / nseg
    k = t.k.astype(np.float64)
    b = t.b.astype(np.float64)
    for i in range(nseg):
        for x in (L + i * w, L + (i + 1) * w):
            got = k[i] * x + b[i]
            slack = 4 * np.finfo(np.float32).eps * max(abs(k[i] * x), abs(b[i]), 1e-30)
            assert abs(got - truth(name, x)) <= slack, (i, x)
    # neighbouring segments meet (continuity)
    for i in range(nseg - 1):
        x = L + (i + 1) * w
        left, right = k[i] * x + b[i], k[i + 1] * x + b[i + 1]
        slack = 8 * np.finfo(np.float32).eps * max(abs(k[i] * x), abs(b[i]), abs(k[i + 1] * x),
                                                   abs(b[i + 1]))
        assert abs(left - right) <= slack
    assert t.inv_w == np.float32(nseg / (R - L))


@pytest.mark.parametrize("name,lo,hi", CASES)
@pytest.mark.parametrize("nseg", [16, 64, 128])
def test_chord_error_within_analytic_bound(oracle, name, lo, hi, nseg):
    """|f - chord| <= w^2/8 * max|f''| on every segment (plus fp32 rounding of k and b)."""
    t = oracle.build_table(func_id(oracle, name), lo, hi, nseg)
    L, R = float(np.float32(lo)), float(np.float32(hi))
    w = (R - L) / nseg
    worst_ratio = 0.0
    for i in range(nseg):
        a, c = L + i * w, L + (i + 1) * w
        xs = np.linspace(a, c, 201)
        err = np.abs(float(t.k[i]) * xs + float(t.b[i]) - truth(name, xs))
        bound = w * w / 8.0 * second_derivative_max(name, a, c)
        slack = 4 * np.finfo(np.float32).eps * (abs(float(t.k[i])) * max(abs(a), abs(c)) +
                                                abs(float(t.b[i])))
        assert err.max() <= bound + slack, (i, err.max(), bound)
        if bound > 1e-12:
            worst_ratio = max(worst_ratio, err.max() / bound)
    # the bound is attained to within a factor ~2 somewhere: the chord is not a better fit than
    # a chord can be (catches a builder that silently does something else)
    assert worst_ratio > 0.4


def test_affine_function_reproduced_exactly(oracle):
    a, c = 0.375, -1.25  # dyadic
    t = oracle.build_table_fn(lambda x: a * x + c, -4.0, 12.0, 64)
    assert np.all(t.k == np.float32(a))
    assert np.all(t.b == np.float32(c))
    t = oracle.build_table(oracle.F_IDENTITY, -8.0, 8.0, 32)
    assert np.all(t.k == 1.0) and np.all(t.b == 0.0)


def test_relu_two_segments_is_exact(oracle):
    t = oracle.build_table(oracle.F_RELU, -8.0, 8.0, 2)
    assert t.k.tolist() == [0.0, 1.0] and t.b.tolist() == [0.0, 0.0]
    xs = np.concatenate([np.linspace(-20, 20, 401), [0.0, -0.0, 1e-30, -1e-6]]).astype(np.float32)
    y, _, s = oracle.pwl_apply(xs, t)
    assert np.array_equal(y, np.maximum(xs, 0.0))
    assert np.array_equal(s, (xs >= 0).astype(np.uint16))
    # the segment is found from (x - lo) in fp32: a negative x closer to 0 than half an ulp of
    # |lo| is indistinguishable from the break point and takes the right-hand line y = x, an
    # error of at most that half ulp
    y, _, s = oracle.pwl_apply(np.array([-1e-30, -2e-7], np.float32), t)
    assert s.tolist() == [1, 1] and np.all(np.abs(y) <= 0.5 * np.spacing(np.float32(8.0)))


def test_max_error_of_uniform_chords_matches_closed_form(oracle):
    """Max abs error of uniform chords, GELU on [-8,8] and exp on [-16,0]: ~w^2/8 * max f''."""
    for name, lo, hi, nseg, expect in [("gelu", -8, 8, 64, 0.25 ** 2 / 8 * 0.7979),
                                       ("exp", -16, 0, 64, 0.25 ** 2 / 8 * 1.0),
                                       ("exp", -16, 0, 128, 0.125 ** 2 / 8 * 1.0)]:
        t = oracle.build_table(func_id(oracle, name), lo, hi, nseg)
        xs = np.linspace(lo, hi, 200001)[:-1]
        w = (hi - lo) / nseg
        idx = np.minimum(((xs - lo) / w).astype(int), nseg - 1)
        err = np.abs(t.k[idx].astype(np.float64) * xs + t.b[idx] - truth(name, xs)).max()
        assert 0.8 * expect <= err <= 1.02 * expect, (name, nseg, err, expect)


def test_bad_arguments_rejected(oracle):
    with pytest.raises(RuntimeError):
        oracle.build_table(oracle.F_EXP, 0.0, 0.0, 8)
    with pytest.raises(RuntimeError):
        oracle.build_table(99, 0.0, 1.0, 8)
