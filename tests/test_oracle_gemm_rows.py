"""Pins for the oracle's integer GEMM + epilogue, softmax-PWL and LayerNorm-PWL."""
import math

import numpy as np
import pytest
import torch

import workloads as W


# ---- integer GEMM -------------------------------------------------------------------------------

@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (5, 7, 3), (33, 65, 130), (64, 48, 768)])
def test_int_gemm_equals_int64_library_matmul(oracle, M, N, K):
    d = W.gemm_inputs(M, N, K, seed=M + N + K)
    r = oracle.gemm_pwl(d["A"], d["W"])
    want = d["A"].astype(np.int64) @ d["W"].astype(np.int64).T
    assert np.array_equal(r["acc"].astype(np.int64), want)
    # extreme operands: K * 127 * 127 fits int32 and is reproduced exactly
    A = np.full((2, K), -127, np.int8)
    Wm = np.full((3, K), 127, np.int8)
    assert np.all(oracle.gemm_pwl(A, Wm)["acc"] == -127 * 127 * K)


def test_gemm_is_not_transposed_or_misindexed(oracle):
    """One-hot operands: acc[m, n] = A[m, k0] * W[n, k0] picks single entries."""
    A = np.zeros((4, 6), np.int8)
    Wm = np.zeros((5, 6), np.int8)
    A[2, 3] = 7
    Wm[4, 3] = -5
    acc = oracle.gemm_pwl(A, Wm)["acc"]
    want = np.zeros((4, 5), np.int32)
    want[2, 4] = -35
    assert np.array_equal(acc, want)


def test_epilogue_terms(oracle):
    d = W.gemm_inputs(9, 11, 32, seed=3)
    acc = d["A"].astype(np.int64) @ d["W"].astype(np.int64).T
    alpha = 2.0 ** -9
    # dequantise + bias: dyadic alpha makes acc*alpha exact, so fp32 y = fl(acc*alpha + bias)
    r = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha)
    want = (acc.astype(np.float64) * alpha + d["bias"].astype(np.float64)).astype(np.float32)
    assert np.array_equal(r["y"], want)
    # residual: + resid * resid_scale (dyadic, exact product), second rounding
    r2 = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha, resid=d["resid"],
                         resid_scale=0.25)
    want2 = (want.astype(np.float64) + d["resid"].astype(np.float64) * 0.25).astype(np.float32)
    assert np.array_equal(r2["y"], want2)
    # per-column scales
    r3 = oracle.gemm_pwl(d["A"], d["W"], alpha_vec=d["alpha_vec"],
                         out_inv_scale_vec=d["out_inv_scale_vec"])
    y3 = (acc.astype(np.float32) * d["alpha_vec"][None, :]).astype(np.float32)
    assert np.array_equal(r3["y"], y3)
    q3 = np.clip(np.rint((y3 * d["out_inv_scale_vec"][None, :]).astype(np.float32)), -127, 127)
    assert np.array_equal(r3["q"].astype(np.float32), q3)


def test_epilogue_table_is_elementwise_pwl(oracle):
    d = W.gemm_inputs(8, 16, 64, seed=5, full_range=False)
    t = oracle.build_table(oracle.F_GELU, -8.0, 8.0, 64)
    alpha = 1.0 / 256
    pre = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha)["y"]
    r = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha, table=t, out_inv_scale=16.0)
    y, q, s = oracle.pwl_apply(pre.ravel(), t, out_inv_scale=16.0)
    assert np.array_equal(r["y"].ravel(), y)
    assert np.array_equal(r["q"].ravel(), q)
    assert np.array_equal(r["seg"].ravel(), s)
    # and close to the true GELU (table bound 0.25^2/8*0.8 ~ 6.2e-3)
    g = torch.nn.functional.gelu(torch.from_numpy(pre.astype(np.float64))).numpy()
    assert np.abs(r["y"] - g).max() < 6.5e-3


def test_int_to_float_conversion_rounds_to_nearest_even(oracle):
    """acc = 16777217 (2^24 + 1) must convert to 16777216.0f."""
    # 16777217 = 127*127*1040 + 3057 ; 3057 = 127*24 + 9
    K = 1040 + 24 + 1
    A = np.zeros((1, K), np.int8)
    Wm = np.zeros((1, K), np.int8)
    A[0, :1040] = 127
    Wm[0, :1040] = 127
    A[0, 1040:1064] = 127
    Wm[0, 1040:1064] = 1
    A[0, 1064] = 9
    Wm[0, 1064] = 1
    r = oracle.gemm_pwl(A, Wm, alpha=1.0)
    assert r["acc"][0, 0] == 2 ** 24 + 1
    assert r["y"][0, 0] == np.float32(2 ** 24)


# ---- softmax-PWL ------------------------------------------------------------------------------

def tables(oracle, nseg=128, recip_hi=128.0):
    return (oracle.build_table(oracle.F_EXP, -16.0, 0.0, nseg),
            oracle.build_table(oracle.F_RECIP, 1.0, recip_hi, nseg))


@pytest.mark.parametrize("cols", [1, 5, 64, 128, 200, 512])
def test_softmax_shift_invariance_is_exact(oracle, cols):
    te, tr = tables(oracle, 64, float(max(64, cols)))
    a = W.score_rows(16, cols, seed=cols)
    r0 = oracle.softmax_pwl(a, 1e-3, te, tr, 127.0)
    r1 = oracle.softmax_pwl(a + 123456, 1e-3, te, tr, 127.0)
    for key in ("p", "q", "seg_exp", "seg_recip"):
        assert np.array_equal(r0[key], r1[key])


@pytest.mark.parametrize("cols", [4, 64, 128, 512])
def test_softmax_constant_row(oracle, cols):
    """A constant row: every t_j = 0, e_j = PWL_exp(0) = 1 (the last chord ends at exp(0)), the
    denominator is cols (exact), p_j = PWL_recip(cols) = 1/cols up to fp32 rounding because cols
    sits on a break point of the recip table when (hi - lo) / nseg divides cols - lo."""
    te = oracle.build_table(oracle.F_EXP, -16.0, 0.0, 64)
    tr = oracle.build_table(oracle.F_RECIP, 0.0 + 1.0, 1.0 + 1024.0, 1024)  # unit segments
    a = np.full((3, cols), -77, np.int32)
    r = oracle.softmax_pwl(a, 0.01, te, tr, 127.0)
    assert np.all(r["seg_exp"] == 63)
    assert np.all(r["seg_recip"] == cols - 1)
    assert np.allclose(r["p"], 1.0 / cols, rtol=4e-7, atol=0)
    assert np.all(r["p"] == r["p"][0, 0])
    assert np.all(r["q"] == int(np.rint(np.float32(r["p"][0, 0]) * np.float32(127.0))))


def test_softmax_close_to_true_softmax(oracle):
    cols, nseg = 128, 128
    te, tr = tables(oracle, nseg, 128.0)
    g = np.random.default_rng(0)
    a = np.rint(3000 * g.standard_normal((64, cols))).astype(np.int32)
    alpha = 2.0e-4  # logits std 0.6: denominators well inside the recip range
    r = oracle.softmax_pwl(a, alpha, te, tr, 127.0)
    t = (a - a.max(axis=1, keepdims=True)).astype(np.float64) * alpha
    e_true = np.exp(t)
    S_true = e_true.sum(axis=1, keepdims=True)
    p_true = e_true / S_true
    w_e = 16.0 / nseg
    eps_e = w_e * w_e / 8.0          # max f'' of exp on [-16, 0] is 1
    w_r = 127.0 / nseg
    S_lo = S_true - cols * eps_e
    eps_r = w_r * w_r / 8.0 * 2.0 / np.maximum(S_lo - w_r, 1.0) ** 3
    # |p - p*| <= |e - e*| r + e* |r - 1/S*|,  |r - 1/S*| <= eps_r + |S - S*| / (S S*)
    r_up = 1.0 / S_lo + eps_r
    bound = eps_e * r_up + e_true * (eps_r + cols * eps_e / (S_lo * S_true)) + 1e-6
    assert np.all(np.abs(r["p"] - p_true) <= bound)
    assert np.abs(r["p"] - p_true).max() < 5e-4
    assert np.abs(r["p"].sum(axis=1) - 1.0).max() < 2e-2
    # int8 codes are the RNE codes of p
    want_q = np.clip(np.rint((r["p"] * np.float32(127.0)).astype(np.float32)), -127, 127)
    assert np.array_equal(r["q"].astype(np.float32), want_q)


def test_softmax_fp32_input_form(oracle):
    te, tr = tables(oracle, 64, 64.0)
    g = np.random.default_rng(2)
    x = g.standard_normal((8, 64)).astype(np.float32)
    r = oracle.softmax_pwl(x, 1.0, te, tr, 127.0)
    p_true = torch.softmax(torch.from_numpy(x.astype(np.float64)), dim=1).numpy()
    assert np.abs(r["p"] - p_true).max() < 2e-3
    # integer-valued fp32 input behaves exactly like the int32 form
    a = np.rint(50 * x).astype(np.int32)
    ri = oracle.softmax_pwl(a, 0.02, te, tr, 127.0)
    rf = oracle.softmax_pwl(a.astype(np.float32), 0.02, te, tr, 127.0)
    assert np.array_equal(ri["p"], rf["p"]) and np.array_equal(ri["seg_exp"], rf["seg_exp"])


# ---- LayerNorm-PWL ----------------------------------------------------------------------------

@pytest.mark.parametrize("cols", [4, 128, 1024, 768, 1000])
def test_layernorm_constant_row_gives_beta(oracle, cols):
    t = oracle.build_table(oracle.F_RSQRT, 1e-3, 64.0, 64)
    g = np.random.default_rng(cols)
    gamma = (1 + 0.1 * g.standard_normal(cols)).astype(np.float32)
    beta = g.standard_normal(cols).astype(np.float32)
    x = np.full((2, cols), 0.75, np.float32)  # 0.75 * cols / cols is exact -> d = 0
    r = oracle.layernorm_pwl(x, gamma, beta, 1e-5, t, 32.0)
    if cols & (cols - 1) == 0:   # 1/cols exact in fp32 -> mean exact -> d = 0 -> y = beta
        assert np.array_equal(r["y"], np.broadcast_to(beta, (2, cols)))
    else:                        # mean off by at most one rounding of 0.75
        assert np.abs(r["y"] - beta).max() < 1e-4
    assert np.all(r["seg"] == 0)


def test_layernorm_variance_on_break_point_is_exact(oracle):
    """Row of +-a: mean 0, variance a^2; with eps = 0 and a^2 on a break point, PWL_rsqrt is
    exact there (chords interpolate the break points), so y = +-1 * gamma + beta to rounding."""
    t = oracle.build_table_fn(lambda v: v ** -0.5, 0.25, 16.25, 64)  # break points 0.25 + i/4
    cols = 256
    x = np.tile(np.array([2.0, -2.0], np.float32), cols // 2)[None, :]  # variance 4 = 0.25+15*0.25
    gamma = np.ones(cols, np.float32)
    beta = np.zeros(cols, np.float32)
    r = oracle.layernorm_pwl(x, gamma, beta, 0.0, t, 1.0)
    assert r["seg"][0] == 15
    assert np.allclose(np.abs(r["y"]), 1.0, rtol=1e-6, atol=0)
    assert np.array_equal(np.sign(r["y"]), np.sign(x))


def test_layernorm_close_to_library_layer_norm(oracle):
    nseg, lo, hi = 256, 1e-3, 64.0
    t = oracle.build_table(oracle.F_RSQRT, lo, hi, nseg)
    cols = 768
    x = W.float_rows(32, cols, seed=7, std=1.5)
    g = np.random.default_rng(8)
    gamma = (1 + 0.1 * g.standard_normal(cols)).astype(np.float32)
    beta = (0.1 * g.standard_normal(cols)).astype(np.float32)
    eps = 1e-5
    r = oracle.layernorm_pwl(x, gamma, beta, eps, t, 30.0)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x.astype(np.float64)), (cols,),
                                         torch.from_numpy(gamma.astype(np.float64)),
                                         torch.from_numpy(beta.astype(np.float64)), eps).numpy()
    var = x.astype(np.float64).var(axis=1) + eps
    w = (float(np.float32(hi)) - float(np.float32(lo))) / nseg
    for i in range(x.shape[0]):
        if i == 1:   # constant row: y = beta exactly
            assert np.array_equal(r["y"][i], beta)
            continue
        if var[i] < lo or var[i] >= hi:  # outside the table: edge segment's line, no accuracy claim
            assert int(r["seg"][i]) == (0 if var[i] < lo else nseg - 1)
            continue
        left = lo + math.floor((var[i] - lo) / w) * w
        assert int(r["seg"][i]) == int(math.floor((var[i] - lo) / w))
        eps_r = w * w / 8.0 * 0.75 * max(left, lo) ** -2.5    # chord bound on this segment
        rel = eps_r * math.sqrt(var[i])                        # relative error of r
        d = x[i].astype(np.float64) - x[i].astype(np.float64).mean()
        bound = np.abs(d / math.sqrt(var[i]) * gamma) * rel + 1e-5 * (1 + np.abs(ref[i]))
        assert np.all(np.abs(r["y"][i] - ref[i]) <= bound), i
    want_q = np.clip(np.rint((r["y"] * np.float32(30.0)).astype(np.float32)), -127, 127)
    assert np.array_equal(r["q"].astype(np.float32), want_q)


# ---- LayerNorm with a square-root table followed by a reciprocal table ----------------------------

def test_layernorm2_break_points_are_exact(oracle):
    """Row of +-2: variance 4.  sqrt table with break points at k/2 ... contains 4 -> sd = 2 exactly;
    reciprocal table with break points at 1 + k/4 contains 2 -> r = 0.5 exactly; y = +-1."""
    ts = oracle.build_table(oracle.F_SQRT, 0.0, 16.0, 32)
    tr = oracle.build_table(oracle.F_RECIP, 1.0, 5.0, 16)
    cols = 256
    x = np.tile(np.array([2.0, -2.0], np.float32), cols // 2)[None, :]
    r = oracle.layernorm_pwl2(x, np.ones(cols, np.float32), np.zeros(cols, np.float32), 0.0, ts, tr, 1.0)
    assert r["seg_sqrt"][0] == 8 and r["seg_recip"][0] == 4
    assert np.allclose(np.abs(r["y"]), 1.0, rtol=1e-6, atol=0)
    assert np.array_equal(np.sign(r["y"]), np.sign(x))


def test_layernorm2_is_the_composition_of_the_two_tables(oracle):
    """r = PWL_recip(PWL_sqrt(var + eps)) with the same mean / variance as the one-table form: the
    two forms differ only in r, so y2 - beta = (y1 - beta) * r2 / r1 up to one rounding each."""
    cols = 200
    x = W.float_rows(9, cols, seed=3, std=1.3)
    gamma = np.ones(cols, np.float32)
    beta = np.zeros(cols, np.float32)
    t1 = oracle.build_table(oracle.F_RSQRT, 0.05, 16.0, 4096)
    ts = oracle.build_table(oracle.F_SQRT, 0.05, 16.0, 4096)
    tr = oracle.build_table(oracle.F_RECIP, 0.2, 4.0, 4096)
    a = oracle.layernorm_pwl(x, gamma, beta, 1e-5, t1, 10.0)
    b = oracle.layernorm_pwl2(x, gamma, beta, 1e-5, ts, tr, 10.0)
    var = x.astype(np.float64).var(axis=1) + 1e-5
    inside = (var > 0.1) & (var < 15.0)   # the generator also makes constant and extreme rows
    assert inside.sum() >= 4
    for i in np.nonzero(inside)[0]:
        u = np.float32(var[i])
        r2 = oracle.pwl_eval(float(oracle.pwl_eval(float(u), ts)), tr)
        assert abs(float(r2) - var[i] ** -0.5) < 1e-4 * var[i] ** -0.5
    live = (np.abs(a["y"]) > 1e-3) & inside[:, None]
    assert np.allclose(b["y"][live], a["y"][live], rtol=2e-4)


def test_layernorm2_close_to_library_layer_norm(oracle):
    cols = 768
    x = W.float_rows(16, cols, seed=11, std=1.5)
    g = np.random.default_rng(12)
    gamma = (1 + 0.1 * g.standard_normal(cols)).astype(np.float32)
    beta = (0.1 * g.standard_normal(cols)).astype(np.float32)
    ts = oracle.build_table(oracle.F_SQRT, 0.0, 16.0, 1024)
    tr = oracle.build_table(oracle.F_RECIP, 0.25, 4.0, 1024)
    r = oracle.layernorm_pwl2(x, gamma, beta, 1e-5, ts, tr, 30.0)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x.astype(np.float64)), (cols,),
                                         torch.from_numpy(gamma.astype(np.float64)),
                                         torch.from_numpy(beta.astype(np.float64)), 1e-5).numpy()
    sd = np.sqrt(x.astype(np.float64).var(axis=1) + 1e-5)
    ok = (sd > 0.3) & (sd < 3.9)   # rows whose standard deviation lies well inside both tables
    assert ok.sum() >= 8
    # chord errors: sqrt w^2/8 * |f''| = (1/64)^2/8 * sd^-3/4, recip (3.75/1024)^2/8 * 2/sd^3: relative ~1e-5
    assert np.abs(r["y"][ok] - ref[ok]).max() < 2e-3
    const = oracle.layernorm_pwl2(np.full((1, 64), 0.5, np.float32), np.ones(64, np.float32),
                                  np.full(64, 0.25, np.float32), 1e-5, ts, tr, 1.0)
    assert np.all(const["y"] == 0.25)   # constant row: d = 0 -> y = beta
