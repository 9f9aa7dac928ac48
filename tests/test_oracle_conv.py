"""Pins of the oracle's convolution and pooling operators (CPU only).

Convolution (Section 3.1: a linear operation that becomes a matrix product): pinned against an
independent library routine (torch.nn.functional.conv2d on float64 tensors, exact for these
integer magnitudes), against the oracle's own matrix product on an explicitly gathered patch
matrix built here with numpy indexing, and against closed-form special cases (one-hot kernels
shift the image; a 1x1 kernel is a matrix product; padding contributes zeros)."""
import numpy as np
import pytest
import torch


def rand_i8(g, shape, lim=127):
    return g.integers(-lim, lim + 1, shape, dtype=np.int64).astype(np.int8)


CASES = [  # B, H, W, Cin, Cout, kh, kw, stride, pad
    (2, 9, 11, 5, 7, 3, 3, 1, 1),
    (1, 12, 12, 16, 8, 3, 3, 2, 1),
    (2, 8, 8, 6, 10, 1, 1, 1, 0),
    (2, 9, 9, 4, 6, 1, 1, 2, 0),
    (1, 17, 15, 3, 5, 7, 7, 2, 3),
    (1, 6, 7, 2, 3, 5, 3, 1, 2),
]


@pytest.mark.parametrize("B,H,W,Cin,Cout,kh,kw,stride,pad", CASES)
def test_conv_accumulators_equal_library_convolution(oracle, B, H, W, Cin, Cout, kh, kw, stride, pad):
    g = np.random.default_rng(B + H + Cin + kh)
    x = rand_i8(g, (B, H, W, Cin))
    w = rand_i8(g, (Cout, kh, kw, Cin))
    r = oracle.conv2d_pwl(x, w, stride=stride, pad=pad)
    want = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2),
                                      torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2),
                                      stride=stride, padding=pad).permute(0, 2, 3, 1).numpy()
    assert r["acc"].shape == want.shape
    assert np.array_equal(r["acc"].astype(np.int64), np.rint(want).astype(np.int64))


@pytest.mark.parametrize("B,H,W,Cin,Cout,kh,kw,stride,pad", CASES[:4])
def test_conv_equals_matrix_product_on_gathered_patches(oracle, B, H, W, Cin, Cout, kh, kw, stride, pad):
    """The matrix form: one row per output position, K = kh*kw*Cin with the tap major and the
    channel minor, padding as zeros; epilogue included (per-channel scale, bias, residual, table)."""
    g = np.random.default_rng(7 * B + H)
    x = rand_i8(g, (B, H, W, Cin), 40)
    w = rand_i8(g, (Cout, kh, kw, Cin), 40)
    Ho, Wo = oracle.conv_out_hw(H, W, kh, kw, stride, pad)
    xp = np.zeros((B, H + 2 * pad, W + 2 * pad, Cin), np.int8)
    xp[:, pad:pad + H, pad:pad + W] = x
    A = np.empty((B, Ho, Wo, kh, kw, Cin), np.int8)
    for i in range(kh):
        for j in range(kw):
            A[:, :, :, i, j] = xp[:, i:i + stride * Ho:stride, j:j + stride * Wo:stride]
    A = A.reshape(B * Ho * Wo, kh * kw * Cin)
    alpha_vec = (1e-3 * (1 + g.random(Cout))).astype(np.float32)
    bias = g.standard_normal(Cout).astype(np.float32)
    resid = rand_i8(g, (B, Ho, Wo, Cout))
    t = oracle.build_table(oracle.F_RELU, -8.0, 8.0, 2)
    kw_ = dict(bias=bias, alpha_vec=alpha_vec, resid_scale=0.02, table=t, out_inv_scale=11.0)
    rc = oracle.conv2d_pwl(x, w, stride=stride, pad=pad, resid=resid, **kw_)
    rg = oracle.gemm_pwl(A, w.reshape(Cout, -1), resid=resid.reshape(-1, Cout), **kw_)
    assert np.array_equal(rc["acc"].reshape(-1, Cout), rg["acc"])
    assert np.array_equal(rc["y"].reshape(-1, Cout).view(np.uint32), rg["y"].view(np.uint32))
    assert np.array_equal(rc["q"].reshape(-1, Cout), rg["q"])
    assert (rc["q"] == 0).mean() > 0.2 and (rc["q"] > 0).mean() > 0.2  # both ReLU segments used


def test_one_hot_kernel_shifts_the_image(oracle):
    """w[n, i, j, c] = [n == c][i == a][j == b]: output (ho, wo, n) = x(ho - 1 + a, wo - 1 + b, n),
    zero outside the image."""
    g = np.random.default_rng(3)
    B, H, W, Cc = 1, 6, 5, 4
    x = rand_i8(g, (B, H, W, Cc))
    for a in range(3):
        for b in range(3):
            w = np.zeros((Cc, 3, 3, Cc), np.int8)
            for n in range(Cc):
                w[n, a, b, n] = 1
            acc = oracle.conv2d_pwl(x, w, stride=1, pad=1)["acc"]
            want = np.zeros((B, H, W, Cc), np.int64)
            for ho in range(H):
                for wo in range(W):
                    hi, wi = ho - 1 + a, wo - 1 + b
                    if 0 <= hi < H and 0 <= wi < W:
                        want[0, ho, wo] = x[0, hi, wi]
            assert np.array_equal(acc, want)


def test_conv_extreme_accumulator(oracle):
    """All -127 against all +127 over the largest K of the CNN workload (3*3*512 = 4608):
    |acc| = 4608 * 127^2 = 74 322 432 < 2^31, converted to fp32 with round-to-nearest-even."""
    x = np.full((1, 3, 3, 512), -127, np.int8)
    w = np.full((2, 3, 3, 512), 127, np.int8)
    r = oracle.conv2d_pwl(x, w, stride=1, pad=0, alpha=1.0)
    assert r["acc"].shape == (1, 1, 1, 2) and int(r["acc"][0, 0, 0, 0]) == -4608 * 127 * 127
    assert r["y"][0, 0, 0, 0] == np.float32(-4608 * 127 * 127)


@pytest.mark.parametrize("B,H,W,Cc,k,stride,pad", [(2, 9, 10, 5, 3, 2, 1), (1, 8, 8, 3, 2, 2, 0), (1, 7, 7, 4, 3, 1, 1)])
def test_maxpool_equals_library(oracle, B, H, W, Cc, k, stride, pad):
    g = np.random.default_rng(H * W)
    x = rand_i8(g, (B, H, W, Cc))
    y = oracle.maxpool_i8(x, k, stride, pad)
    want = torch.nn.functional.max_pool2d(torch.from_numpy(x.astype(np.float32)).permute(0, 3, 1, 2), k, stride,
                                          pad).permute(0, 2, 3, 1).numpy()
    assert np.array_equal(y.astype(np.float32), want)


def test_maxpool_all_negative_border(oracle):
    """Padding never wins: an all-(-100) image pools to -100 everywhere, borders included."""
    x = np.full((1, 5, 5, 2), -100, np.int8)
    assert np.array_equal(oracle.maxpool_i8(x, 3, 2, 1), np.full((1, 3, 3, 2), -100, np.int8))


def test_avgpool_is_the_scaled_integer_sum(oracle):
    g = np.random.default_rng(11)
    x = rand_i8(g, (3, 49, 10))
    s_x = 0.037
    alpha = float(np.float32(s_x / 49))
    r = oracle.avgpool_i8(x, alpha, 20.0)
    acc = x.astype(np.int64).sum(axis=1)
    want = (acc.astype(np.float32) * np.float32(alpha)).astype(np.float32)
    assert np.array_equal(r["y"].view(np.uint32), want.view(np.uint32))
    assert np.allclose(r["y"], x.astype(np.float64).mean(axis=1) * s_x, rtol=1e-6, atol=1e-7)
    wq = np.clip(np.rint((want * np.float32(20.0)).astype(np.float32)), -127, 127).astype(np.int8)
    assert np.array_equal(r["q"], wq)
    const = np.full((1, 16, 4), 64, np.int8)  # a constant image averages to itself: 16 * 64 / 16
    assert np.all(oracle.avgpool_i8(const, 1.0 / 16, 1.0)["y"] == 64.0)


@pytest.mark.parametrize("name", ["resnet_odd", "resnet_tiny"])
def test_resnet_forward_tracks_a_float64_library_network(oracle, name):
    """The oracle's int8 residual network against the same network in float64 with library
    operators and no activation rounding (weights dequantised, batch-norm gain and bias applied
    per channel, ReLU, residual sums, pooling, classifier): the wiring (strides, shortcuts,
    which tensor feeds which) must agree, so the logits differ only by quantisation noise."""
    import workloads as W
    p = W.resnet_params(name, 0)
    got = oracle.resnet_forward(p)["logits"]
    F = torch.nn.functional
    cur = {"x": torch.from_numpy(p["x"].astype(np.float64) * p["s_x"]).permute(0, 3, 1, 2)}
    for op in p["graph"]:
        n = op["name"]
        if op["op"] == "conv":
            w = torch.from_numpy(p["w"][n].astype(np.float64) * p["s_w"][n]).permute(0, 3, 1, 2)
            y = F.conv2d(cur[op["src"]], w, stride=op["stride"], padding=op["pad"])
            y = y * torch.from_numpy(p["gain"][n]).view(1, -1, 1, 1) + \
                torch.from_numpy(p["bias"][n].astype(np.float64)).view(1, -1, 1, 1)
            if op["resid"]:
                y = y + cur[op["resid"]]
            cur[op["dst"]] = torch.relu(y) if op["relu"] else y
        elif op["op"] == "maxpool":
            cur[op["dst"]] = F.max_pool2d(cur[op["src"]], op["k"], op["stride"], op["pad"])
        elif op["op"] == "avgpool":
            cur[op["dst"]] = cur[op["src"]].mean(dim=(2, 3))
        elif op["op"] == "fc":
            w = torch.from_numpy(p["w"][n].astype(np.float64) * p["s_w"][n])
            want = (cur[op["src"]] @ w.T + torch.from_numpy(p["bias"][n].astype(np.float64))).numpy()
    assert got.shape == want.shape
    rel = np.sqrt(((got - want) ** 2).mean() / (want ** 2).mean())
    assert rel < 0.05, rel
    assert np.abs(want).max() > 0.05  # the logits are not degenerate
