"""Pins for the oracle's run-time PWL pieces: segment search ("quantising x"), evaluation, int8
requantisation, canonical row reduction."""
import numpy as np
import pytest


def brute_segment(x, lo, hi, nseg):
    """if-chain over the break points in double: the segment whose half-open interval holds x,
    first / last segment outside the range."""
    w = (hi - lo) / nseg
    s = 0
    for i in range(1, nseg):
        if x >= lo + i * w:
            s = i
    return s


@pytest.mark.parametrize("nseg", [1, 2, 3, 4, 7, 8])
@pytest.mark.parametrize("scale", [1.0 / 16, 3.0 / 64, 0.25])
def test_segment_search_brute_force_over_all_int8(oracle, nseg, scale):
    lo, hi = -4.0, 4.0
    t = oracle.build_table(oracle.F_GELU, lo, hi, nseg)
    q = np.arange(-128, 128, dtype=np.int32)
    y, _, seg = oracle.pwl_apply(q, t, alpha=scale)
    for qi, si, yi in zip(q.tolist(), seg.tolist(), y.tolist()):
        x = float(np.float32(qi) * np.float32(scale))
        want = brute_segment(x, lo, hi, nseg)
        assert si == want, (qi, x, si, want)
        # value = that segment's line at x (one rounding)
        line = float(t.k[want]) * x + float(t.b[want])
        assert abs(yi - line) <= 2e-7 * max(1.0, abs(line))
    assert np.all(np.diff(seg.astype(int)) >= 0)  # monotone in x


def test_break_point_belongs_to_right_segment_and_clamps(oracle):
    t = oracle.build_table(oracle.F_EXP, -16.0, 0.0, 64)  # w = 0.25, exact in fp32
    for i in range(64):
        assert oracle.segidx(-16.0 + 0.25 * i, t) == i
        # just left of the break point, by more than the fp32 resolution of (x - lo)
        assert oracle.segidx(np.float32(-16.0 + 0.25 * i) - np.float32(4e-6), t) == max(i - 1, 0)
    assert oracle.segidx(0.0, t) == 63          # x == hi -> last segment
    assert oracle.segidx(5.0, t) == 63
    assert oracle.segidx(1e30, t) == 63
    assert oracle.segidx(np.inf, t) == 63
    assert oracle.segidx(-16.001, t) == 0
    assert oracle.segidx(-1e30, t) == 0
    assert oracle.segidx(-np.inf, t) == 0
    assert oracle.segidx(np.nan, t) == 0         # NaN lands in segment 0


def test_out_of_range_uses_edge_lines(oracle):
    """Inputs outside [lo, hi] share k, b with the first / last segment."""
    t = oracle.build_table(oracle.F_GELU, -8.0, 8.0, 64)
    for x in (-9.5, -100.0):
        got = float(oracle.pwl_eval(x, t))
        assert abs(got - (float(t.k[0]) * x + float(t.b[0]))) <= 1e-6 * max(1, abs(got))
    for x in (8.5, 100.0):
        got = float(oracle.pwl_eval(x, t))
        assert abs(got - (float(t.k[63]) * x + float(t.b[63]))) <= 1e-6 * max(1, abs(got))
        assert abs(got - x) < 1e-3  # GELU's last chord is y = x to table accuracy


def test_clamp_input_flag(oracle):
    t = oracle.build_table(oracle.F_EXP, -16.0, 0.0, 64, flags=oracle.FLAG_CLAMP_INPUT)
    assert oracle.pwl_eval(-50.0, t) == oracle.pwl_eval(-16.0, t)
    assert oracle.pwl_eval(3.0, t) == oracle.pwl_eval(0.0, t)
    t2 = oracle.build_table(oracle.F_EXP, -16.0, 0.0, 64)
    assert oracle.pwl_eval(-50.0, t2) < 0  # extrapolated chord goes negative: the documented hazard


def test_requant_ties_to_even_and_saturation(oracle):
    cases = {0.5: 0, 1.5: 2, 2.5: 2, 3.5: 4, -0.5: 0, -1.5: -2, -2.5: -2, 0.49999997: 0,
             0.50000006: 1, 126.5: 126, 127.49: 127, 127.5: 127, 128.0: 127, 1e9: 127,
             -126.5: -126, -127.5: -127, -128.0: -127, -1e9: -127, 0.0: 0, -0.0: 0}
    for v, want in cases.items():
        assert oracle.requant(v, 1.0) == want, v
    # the product v * inv_scale is rounded to fp32 before rint
    assert oracle.requant(3.0, 0.5) == 2          # 1.5 -> 2
    assert oracle.requant(5.0, 0.5) == 2          # 2.5 -> 2
    assert oracle.requant(np.nan, 1.0) == -127    # NaN saturates low (fmax/fmin drop the NaN)


def test_requant_exhaustive_against_numpy(oracle):
    g = np.random.default_rng(0)
    v = np.concatenate([g.uniform(-140, 140, 5000), np.arange(-130, 130.25, 0.25)]).astype(np.float32)
    want = np.clip(np.rint(v.astype(np.float32)), -127, 127).astype(int)  # numpy rint is half-even
    got = np.array([oracle.requant(x, 1.0) for x in v])
    assert np.array_equal(got, want)


# ---- canonical reduction: order pinned by hand-derived fp32 results ---------------------------

def test_canonical_sum_matches_exact_sum_when_no_rounding(oracle):
    x = np.arange(1, 1001, dtype=np.float32)
    assert oracle.canonical_sum(x) == 500500.0
    assert oracle.canonical_sumsq(np.arange(1, 101, dtype=np.float32)) == 338350.0
    assert oracle.canonical_sum(np.zeros(0, np.float32)) == 0.0


def test_canonical_sum_order_inside_one_accumulator(oracle):
    """Elements 0..3 share accumulator 0 and are added left to right starting from +0:
    ((2^24 + 1) + 1) + 1 = 2^24 (each +1 is lost), but 1 + 1 + 1 + 2^24 = 2^24 + 4 after
    rounding 2^24 + 3 to even."""
    big = np.float32(2 ** 24)
    assert oracle.canonical_sum(np.array([big, 1, 1, 1], np.float32)) == big
    assert oracle.canonical_sum(np.array([1, 1, 1, big], np.float32)) == big + 4


def test_canonical_sum_deals_groups_of_four_to_64_accumulators(oracle):
    """Element j goes to accumulator (j // 4) % 64.  Put 2^24 at j = 0 and 1 at j = 4, 8, 12:
    they sit in accumulators 0, 1, 2, 3.  The butterfly adds partner pairs first
    (mask 2: a0+a2, a1+a3; mask 1: (a0+a2)+(a1+a3)) = (2^24+1 -> 2^24) + 2 = 2^24 + 2.
    A left-to-right sum would give 2^24."""
    big = np.float32(2 ** 24)
    x = np.zeros(16, np.float32)
    x[0], x[4], x[8], x[12] = big, 1, 1, 1
    assert oracle.canonical_sum(x) == big + 2
    # element 256 wraps around to accumulator 0 again: (2^24 + 1) in one accumulator -> lost
    x = np.zeros(260, np.float32)
    x[0], x[256] = big, 1
    assert oracle.canonical_sum(x) == big
    x = np.zeros(260, np.float32)
    x[0], x[252] = big, 1  # accumulator 63: reaches accumulator 0 only at the last step
    assert oracle.canonical_sum(x) == big  # 2^24 + 1 rounds to even 2^24
    x[244] = 1  # accumulator 61 pairs with 63 at mask 2 -> 2, then 2^24 + 2 is exact
    assert oracle.canonical_sum(x) == big + 2


@pytest.mark.parametrize("first,second", [(32, 16), (16, 8), (8, 4), (4, 2), (2, 1)])
def test_canonical_sum_butterfly_mask_order(oracle, first, second):
    """Masks are applied 32, 16, 8, 4, 2, 1.  With 2^24 in accumulator 0 and 1 in accumulators
    `second` and `first|second`, the two ones meet at mask `first` (giving 2) before meeting the
    big value at mask `second`: 2^24 + 2 is exact.  In the opposite order each 1 would be added
    to 2^24 alone and be lost.  The mirrored pattern (ones in `first` and `first|second`) loses
    both ones in the canonical order."""
    big = np.float32(2 ** 24)
    x = np.zeros(256, np.float32)
    x[0], x[4 * second], x[4 * (first | second)] = big, 1, 1
    assert oracle.canonical_sum(x) == big + 2
    x = np.zeros(256, np.float32)
    x[0], x[4 * first], x[4 * (first | second)] = big, 1, 1
    assert oracle.canonical_sum(x) == big


def test_canonical_sum_close_to_exact_on_random_rows(oracle):
    g = np.random.default_rng(1)
    for n in (1, 3, 64, 128, 500, 768, 1024, 4099):
        x = g.standard_normal(n).astype(np.float32)
        exact = float(np.sum(x.astype(np.float64)))
        got = float(oracle.canonical_sum(x))
        assert abs(got - exact) <= 16 * np.finfo(np.float32).eps * float(np.sum(np.abs(x)))
        sq = float(oracle.canonical_sumsq(x))
        assert abs(sq - float(np.sum(x.astype(np.float64) ** 2))) <= 1e-5 * sq + 1e-30
