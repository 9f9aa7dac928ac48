"""Pins for the oracle's encoder layer: (1) its wiring equals the composition of the separately
pinned stage functions with the attention products done by an int64 library einsum; (2) its
exact-function binary64 mode equals a library (PyTorch CPU, float64) transformer layer; (3) the PWL
layer stays within the tables' accuracy of the exact-function layer."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as W

FUNC = {"gelu": 0, "exp": 1, "recip": 2, "rsqrt": 3}


def make_tables(oracle, cfg):
    return {n: oracle.build_table(FUNC[f], lo, hi, nseg)
            for n, (f, lo, hi, nseg) in W.table_ranges(cfg).items()}


@pytest.mark.parametrize("name", ["tiny", "ragged"])
def test_layer_equals_composition_of_pinned_stages(oracle, name):
    cfg = W.config(name)
    p = W.layer_params(name, 0)
    tb = make_tables(oracle, cfg)
    out = oracle.encoder_layer(p, tb, p["x"])
    B, S, H, nh = cfg["B"], cfg["S"], cfg["H"], cfg["heads"]
    d = H // nh
    M = B * S
    x = p["x"]
    osv = np.concatenate([np.full(H, p["inv_s_q"]), np.full(H, p["inv_s_k"]),
                          np.full(H, p["inv_s_v"])]).astype(np.float32)
    qkv = oracle.gemm_pwl(x, p["Wqkv"], bias=p["bqkv"], alpha=p["alpha_qkv"],
                          out_inv_scale_vec=osv)["q"]
    assert np.array_equal(out["qkv"], qkv)
    q4 = qkv[:, :H].reshape(B, S, nh, d).astype(np.int64)
    k4 = qkv[:, H:2 * H].reshape(B, S, nh, d).astype(np.int64)
    v4 = qkv[:, 2 * H:].reshape(B, S, nh, d).astype(np.int64)
    scores = np.einsum("bihc,bjhc->bhij", q4, k4)
    assert np.array_equal(out["scores"].astype(np.int64), scores)
    sm = oracle.softmax_pwl(scores.reshape(-1, S).astype(np.int32), p["alpha_scores"], tb["exp"],
                            tb["recip"], p["inv_s_p"])
    P = sm["q"].reshape(B, nh, S, S)
    assert np.array_equal(out["p"], P)
    cacc = np.einsum("bhij,bjhc->bihc", P.astype(np.int64), v4).reshape(M, H)
    assert np.abs(cacc).max() < 2 ** 24  # so the int->fp32 conversion below is exact
    cv = (cacc.astype(np.float32) * np.float32(p["alpha_ctx"])).astype(np.float32)
    ctx = np.clip(np.rint((cv * np.float32(p["inv_s_ctx"])).astype(np.float32)), -127, 127)
    assert np.array_equal(out["ctx"].astype(np.float32), ctx)
    attn = oracle.gemm_pwl(out["ctx"], p["Wo"], bias=p["bo"], alpha=p["alpha_o"], resid=x,
                           resid_scale=p["resid1_scale"])["y"]
    assert np.array_equal(out["attn"], attn)
    ln1 = oracle.layernorm_pwl(attn, p["gamma1"], p["beta1"], p["eps1"], tb["rsqrt"],
                               p["inv_s_ln1"])["q"]
    assert np.array_equal(out["ln1"], ln1)
    ffn1 = oracle.gemm_pwl(ln1, p["W1"], bias=p["b1"], alpha=p["alpha_1"], table=tb["gelu"],
                           out_inv_scale=p["inv_s_ffn1"])["q"]
    assert np.array_equal(out["ffn1"], ffn1)
    ffn2 = oracle.gemm_pwl(ffn1, p["W2"], bias=p["b2"], alpha=p["alpha_2"], resid=ln1,
                           resid_scale=p["resid2_scale"])["y"]
    assert np.array_equal(out["ffn2"], ffn2)
    ln2 = oracle.layernorm_pwl(ffn2, p["gamma2"], p["beta2"], p["eps2"], tb["rsqrt"],
                               p["inv_s_out"])
    assert np.array_equal(out["y_q"], ln2["q"])
    assert np.array_equal(out["y_f32"], ln2["y"])


def torch_layer(p, x_codes, quantise):
    """A float64 post-LN transformer encoder layer from library ops, fed the same int8 weights."""
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))  # noqa: E731
    B, S, H, nh = p["B"], p["S"], p["H"], p["heads"]
    d = H // nh
    f32 = lambda v: float(np.float32(v))  # noqa: E731

    def q8(v, inv):
        if not quantise:
            return v * f32(inv)
        return torch.clamp(torch.round(v * f32(inv)), -127, 127)

    x = t(x_codes)
    qkv = F.linear(x, t(p["Wqkv"])) * f32(p["alpha_qkv"]) + t(p["bqkv"])
    q = q8(qkv[:, :H], p["inv_s_q"]).reshape(B, S, nh, d).transpose(1, 2)
    k = q8(qkv[:, H:2 * H], p["inv_s_k"]).reshape(B, S, nh, d).transpose(1, 2)
    v = q8(qkv[:, 2 * H:], p["inv_s_v"]).reshape(B, S, nh, d).transpose(1, 2)
    logits = (q @ k.transpose(-1, -2)) * f32(p["alpha_scores"])
    P = q8(torch.softmax(logits, dim=-1), p["inv_s_p"])
    ctx = (P @ v) * f32(p["alpha_ctx"])
    ctx = q8(ctx, p["inv_s_ctx"]).transpose(1, 2).reshape(B * S, H)
    attn = F.linear(ctx, t(p["Wo"])) * f32(p["alpha_o"]) + t(p["bo"]) + x * f32(p["resid1_scale"])
    ln1 = F.layer_norm(attn, (H,), t(p["gamma1"]), t(p["beta1"]), f32(p["eps1"]))
    ln1 = q8(ln1, p["inv_s_ln1"])
    h = F.linear(ln1, t(p["W1"])) * f32(p["alpha_1"]) + t(p["b1"])
    g = q8(F.gelu(h), p["inv_s_ffn1"])
    ffn2 = F.linear(g, t(p["W2"])) * f32(p["alpha_2"]) + t(p["b2"]) + ln1 * f32(p["resid2_scale"])
    y = F.layer_norm(ffn2, (H,), t(p["gamma2"]), t(p["beta2"]), f32(p["eps2"]))
    if quantise:
        y = q8(y, p["inv_s_out"]) / f32(p["inv_s_out"])
    return y.numpy()


@pytest.mark.parametrize("name", ["tiny", "ragged"])
def test_exact_mode_equals_library_transformer_layer(oracle, name):
    cfg = W.config(name)
    p = W.layer_params(name, 0)
    tb = make_tables(oracle, cfg)
    y, obs = oracle.encoder_layer_exact(p, tb, p["x"], quantise=False)
    ref = torch_layer(p, p["x"], quantise=False)
    assert np.abs(y - ref).max() < 1e-9
    # quantised: identical up to rare ties decided by the last bits of a float64 sum
    yq, _ = oracle.encoder_layer_exact(p, tb, p["x"], quantise=True)
    refq = torch_layer(p, p["x"], quantise=True)
    step = 1.0 / float(np.float32(p["inv_s_out"]))
    diff = np.abs(yq - refq)
    assert diff.max() <= 1.0001 * step
    assert (diff > 0.5 * step).mean() < 2e-3
    # the calibration record reports what the library run sees
    assert obs["x"] == pytest.approx(np.abs(p["x"]).max() * p["resid1_scale"], rel=1e-6)
    assert obs["out"] == pytest.approx(np.abs(ref).max(), rel=1e-9)
    assert 1.0 <= obs["softmax_den_max"] <= cfg["S"]


def test_stack_is_the_layers_one_after_the_other(oracle):
    """encoder_stack against the pinned single layer: a stack of one layer is that layer; a stack of
    three distinct layers ends where feeding each layer's int8 output to the next one by hand ends
    (and not where the layers in another order, or the first input fed to every layer, end)."""
    stack = W.stack_params("tiny", 3)
    tables = make_tables(oracle, W.config("tiny"))
    x = stack[0]["x"]
    one = oracle.encoder_stack(stack[:1], tables, x)
    assert np.array_equal(one["y_q"], oracle.encoder_layer(stack[0], tables, x)["y_q"])
    by_hand = x
    for p in stack:
        by_hand = oracle.encoder_layer(p, tables, by_hand, want_taps=False)["y_q"]
    got = oracle.encoder_stack(stack, tables, x)
    assert np.array_equal(got["y_q"], by_hand)
    assert got["y_q"].dtype == np.int8 and got["y_q"].shape == x.shape
    swapped = oracle.encoder_stack([stack[1], stack[0], stack[2]], tables, x)["y_q"]
    unchained = oracle.encoder_layer(stack[2], tables, x, want_taps=False)["y_q"]
    assert not np.array_equal(got["y_q"], swapped) and not np.array_equal(got["y_q"], unchained)


def test_stored_scales_are_the_calibration_output(oracle):
    """The stored scale file is what the calibration run of the exact-function layer produces."""
    from oracle import make_scales
    for name in ("tiny", "ragged"):
        got = make_scales.calibrate(name, 0)
        want = W.stored_scales(name, 0)
        for n in W.ACT_NAMES:
            assert got[n] == pytest.approx(want[n], rel=1e-12)


def test_pwl_layer_converges_to_exact_function_layer(oracle):
    """With the workload's own coarse tables (64 uniform segments; rsqrt on [1e-3, 64] has its
    first break point at 1.0, right where the LayerNorm variances of N(0,1) inputs lie) the PWL
    layer is only a rough approximation; with finer tables on tighter ranges it converges to the
    exact-function layer.  A mistake in how the layer uses its tables would break the second."""
    cfg = W.config("tiny")
    p = W.layer_params("tiny", 0)
    coarse = make_tables(oracle, cfg)
    fine = dict(gelu=oracle.build_table(0, -8.0, 8.0, 256), exp=oracle.build_table(1, -16.0, 0.0, 256),
                recip=oracle.build_table(2, 1.0, 65.0, 256), rsqrt=oracle.build_table(3, 0.25, 4.25, 256))
    yq, _ = oracle.encoder_layer_exact(p, coarse, p["x"], quantise=True)
    step = 1.0 / float(np.float32(p["inv_s_out"]))

    def rel_rms(tb):
        out = oracle.encoder_layer(p, tb, p["x"], want_taps=False)
        assert np.isfinite(out["y_f32"]).all()
        err = out["y_f32"].astype(np.float64) - yq
        return math.sqrt((err ** 2).mean() / (yq ** 2).mean())

    assert rel_rms(coarse) < 0.5
    # residual error of the fine tables: int8 rounding flips (one output step = 0.03) dominate
    assert rel_rms(fine) < 0.03
    assert step < 0.05
