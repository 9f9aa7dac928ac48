"""Seeded synthetic workloads: the only module shared by the GPU library's harness and the CPU
oracle's tests (a package of its own, outside both).  It generates INPUTS (int8 tensors, fp32 vectors, scale numbers, table ranges); it
holds none of the method's arithmetic (no GEMM, no PWL evaluation, no reductions).

The tensors stand in for the workloads the paper evaluates (BERT / RoBERTa encoders on GLUE):
random-initialised weights and random inputs with the shapes of those models.  Recipe:

* one ``numpy`` PCG64 stream per (workload, seed), drawn in the fixed order
  x, Wqkv, bqkv, Wo, bo, gamma1, beta1, W1, b1, W2, b2, gamma2, beta2;
* weights ~ N(0, 0.02^2), input x ~ N(0, 1), biases and beta ~ N(0, 0.02^2),
  gamma ~ 1 + N(0, 0.02^2)  (non-trivial so that every epilogue term is exercised);
* int8 tensors are per-tensor symmetric: scale = absmax / 127, code = clip(rint(v / scale));
* activation scales are static.  They come from ``workload_scales.json`` (written once by the
  calibration script that sits with the CPU oracle: one run of the true-function network over the
  same seeded input, scale = observed absmax / 127; this is step 1 of the paper's Section 3.2,
  "obtain the input range by running the model", applied to scales as well as to table ranges).
"""
from __future__ import annotations

import json
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SCALES_JSON = os.path.join(_HERE, "workload_scales.json")

# name -> dims, segment count, PWL ranges (function name, lo, hi)
CONFIGS = {
    # benchmark configuration 0: the small case the oracle finishes in well under a second
    "tiny": dict(B=1, S=64, H=128, heads=2, F=512, nseg=64),
    # benchmark configuration 1: the configuration the headline metric is quoted on
    "bert_base_layer": dict(B=32, S=128, H=768, heads=12, F=3072, nseg=128),
    # one layer of benchmark configuration 2 (12-layer BERT-base, batch 16, sequence 512)
    "bert_base_s512": dict(B=16, S=512, H=768, heads=12, F=3072, nseg=128),
    # one layer of benchmark configuration 4 (24-layer BERT-large, batch 32, sequence 512)
    "bert_large_s512": dict(B=32, S=512, H=1024, heads=16, F=4096, nseg=64),
    # a sequence longer than the fused attention kernel covers (parity tests only: three-kernel attention)
    "long_seq": dict(B=1, S=640, H=128, heads=2, F=256, nseg=64),
    # ragged shapes that fit no tile exactly (parity tests only)
    "ragged": dict(B=3, S=40, H=96, heads=3, F=200, nseg=37),
}

ACT_NAMES = ("q", "k", "v", "p", "ctx", "ln1", "ffn1", "out")

LAYER_FLOATS = ("alpha_qkv", "inv_s_q", "inv_s_k", "inv_s_v", "alpha_scores", "inv_s_p",
                "alpha_ctx", "inv_s_ctx", "alpha_o", "resid1_scale", "inv_s_ln1", "alpha_1",
                "inv_s_ffn1", "alpha_2", "resid2_scale", "inv_s_out")


def config(name: str) -> dict:
    return dict(CONFIGS[name])


def table_ranges(cfg: dict) -> dict:
    """PWL ranges of the benchmark's configurations: GELU on [-8, 8], exp on [-16, 0], reciprocal on
    [1, max(64, S)] (a softmax denominator lies in [1, S]), rsqrt on [1e-3, 64]."""
    n = int(cfg["nseg"])
    return {
        "gelu": ("gelu", -8.0, 8.0, n),
        "exp": ("exp", -16.0, 0.0, n),
        "recip": ("recip", 1.0, float(max(64, cfg["S"])), n),
        "rsqrt": ("rsqrt", 1e-3, 64.0, n),
    }


def quantize_sym(v: np.ndarray):
    """Per-tensor symmetric int8 code of a synthetic tensor: (codes, scale)."""
    amax = float(np.max(np.abs(v)))
    scale = amax / 127.0 if amax > 0 else 1.0
    q = np.clip(np.rint(v.astype(np.float64) / scale), -127, 127).astype(np.int8)
    return q, scale


def layer_tensors(cfg: dict, seed: int = 0) -> dict:
    """All tensors of one encoder layer and its input, quantised, plus their scales."""
    g = np.random.Generator(np.random.PCG64(seed))
    B, S, H, F = cfg["B"], cfg["S"], cfg["H"], cfg["F"]
    M = B * S

    def normal(shape, std, mean=0.0):
        return (mean + std * g.standard_normal(shape, dtype=np.float32)).astype(np.float32)

    t = dict(B=B, S=S, H=H, heads=cfg["heads"], F=F)
    x = normal((M, H), 1.0)
    t["x"], t["s_x"] = quantize_sym(x)
    t["Wqkv"], t["s_wqkv"] = quantize_sym(normal((3 * H, H), 0.02))
    t["bqkv"] = normal((3 * H,), 0.02)
    t["Wo"], t["s_wo"] = quantize_sym(normal((H, H), 0.02))
    t["bo"] = normal((H,), 0.02)
    t["gamma1"] = normal((H,), 0.02, 1.0)
    t["beta1"] = normal((H,), 0.02)
    t["W1"], t["s_w1"] = quantize_sym(normal((F, H), 0.02))
    t["b1"] = normal((F,), 0.02)
    t["W2"], t["s_w2"] = quantize_sym(normal((H, F), 0.02))
    t["b2"] = normal((H,), 0.02)
    t["gamma2"] = normal((H,), 0.02, 1.0)
    t["beta2"] = normal((H,), 0.02)
    t["eps1"] = 1e-5
    t["eps2"] = 1e-5
    return t


def with_scales(t: dict, act: dict) -> dict:
    """Add the fp32 multipliers both implementations receive, formed in binary64 from the tensor
    scales and rounded once to fp32.  ``act`` maps q,k,v,p,ctx,ln1,ffn1,out -> scale."""
    p = dict(t)
    d = t["H"] // t["heads"]
    f32 = lambda v: float(np.float32(v))  # noqa: E731
    p["alpha_qkv"] = f32(t["s_x"] * t["s_wqkv"])
    p["inv_s_q"] = f32(1.0 / act["q"])
    p["inv_s_k"] = f32(1.0 / act["k"])
    p["inv_s_v"] = f32(1.0 / act["v"])
    p["alpha_scores"] = f32(act["q"] * act["k"] / np.sqrt(float(d)))
    p["inv_s_p"] = f32(1.0 / act["p"])
    p["alpha_ctx"] = f32(act["p"] * act["v"])
    p["inv_s_ctx"] = f32(1.0 / act["ctx"])
    p["alpha_o"] = f32(act["ctx"] * t["s_wo"])
    p["resid1_scale"] = f32(t["s_x"])
    p["inv_s_ln1"] = f32(1.0 / act["ln1"])
    p["alpha_1"] = f32(act["ln1"] * t["s_w1"])
    p["inv_s_ffn1"] = f32(1.0 / act["ffn1"])
    p["alpha_2"] = f32(act["ffn1"] * t["s_w2"])
    p["resid2_scale"] = f32(act["ln1"])
    p["inv_s_out"] = f32(1.0 / act["out"])
    p["act_scales"] = dict(act)
    return p


def unit_scales() -> dict:
    return {n: 1.0 for n in ACT_NAMES}


def stored_scales(name: str, seed: int = 0) -> dict:
    """Calibrated activation scales of a named workload, from the stored calibration file."""
    with open(SCALES_JSON) as f:
        table = json.load(f)
    key = f"{name}/seed{seed}"
    if key not in table:
        raise KeyError(f"no stored activation scales for {key}; run oracle/make_scales.py")
    return {n: float(table[key][n]) for n in ACT_NAMES}


def layer_params(name: str, seed: int = 0) -> dict:
    """Tensors + calibrated multipliers of a named workload."""
    return with_scales(layer_tensors(config(name), seed), stored_scales(name, seed))


def stored_stack_scales(name: str, n_layers: int) -> list:
    """Calibrated activation scales of every layer of a stack, from the stored calibration file."""
    with open(SCALES_JSON) as f:
        table = json.load(f)
    key = f"{name}/stack"
    if key not in table or len(table[key]) < n_layers:
        raise KeyError(f"no stored activation scales for {n_layers} layers of {name}; run "
                       f"python -m oracle.make_scales stack:{name}:{n_layers}")
    return [{n: float(s[n]) for n in ACT_NAMES} for s in table[key][:n_layers]]


def stack_params(name: str, n_layers: int) -> list:
    """A stack of ``n_layers`` layers of a named workload: layer l has its own weights (seed l), its
    own calibrated activation scales, and reads the int8 output of layer l-1, so its input scale is
    that layer's output scale.  Element 0 also carries the stack input ``x``."""
    cfg, acts = config(name), stored_stack_scales(name, n_layers)
    out = []
    for l in range(n_layers):
        t = layer_tensors(cfg, l)
        if l > 0:
            del t["x"]
            t["s_x"] = acts[l - 1]["out"]
        out.append(with_scales(t, acts[l]))
    return out


# ---------------------------------------------------------------------------------------------
# Inputs for the single-kernel tests and for the stress distribution (values that sweep the whole
# table range, fall outside it, sit on break points, constant rows).
# ---------------------------------------------------------------------------------------------

def gemm_inputs(M: int, N: int, K: int, seed: int = 0, full_range: bool = True) -> dict:
    g = np.random.Generator(np.random.PCG64(seed))
    lim = 127 if full_range else 20
    return dict(
        A=g.integers(-lim, lim + 1, size=(M, K), dtype=np.int8),
        W=g.integers(-lim, lim + 1, size=(N, K), dtype=np.int8),
        bias=(0.5 * g.standard_normal(N)).astype(np.float32),
        resid=g.integers(-127, 128, size=(M, N), dtype=np.int8),
        alpha_vec=np.exp(0.25 * g.standard_normal(N)).astype(np.float32),
        out_inv_scale_vec=np.exp(0.25 * g.standard_normal(N)).astype(np.float32),
    )


def score_rows(rows: int, cols: int, seed: int = 0, spread: float = 4000.0) -> np.ndarray:
    """int32 attention-score-like rows; a few rows are constant, a few have outliers far below
    the exp table's range."""
    g = np.random.Generator(np.random.PCG64(seed))
    a = np.rint(spread * g.standard_normal((rows, cols))).astype(np.int32)
    if rows >= 4:
        a[1, :] = 1234
        a[2, :: max(1, cols // 7)] -= 10_000_000
        a[3, 0] += 5_000_000
    return a


def float_rows(rows: int, cols: int, seed: int = 0, std: float = 1.5) -> np.ndarray:
    """fp32 LayerNorm-input-like rows; includes a constant row, a tiny-variance row and a
    large-variance row."""
    g = np.random.Generator(np.random.PCG64(seed))
    a = (std * g.standard_normal((rows, cols))).astype(np.float32)
    if rows >= 4:
        a[1, :] = 0.75
        a[2, :] = 3.0 + 1e-3 * a[2, :]
        a[3, :] *= 9.0
    return a


def sweep_values(lo: float, hi: float, n: int, seed: int = 0) -> np.ndarray:
    """fp32 values that cover [lo - 10%, hi + 10%] densely, plus the exact break points of an
    n-independent dyadic grid and a few specials (0, -0, huge)."""
    g = np.random.Generator(np.random.PCG64(seed))
    span = hi - lo
    v = g.uniform(lo - 0.1 * span, hi + 0.1 * span, size=n).astype(np.float32)
    grid = np.linspace(lo, hi, 257, dtype=np.float64).astype(np.float32)
    specials = np.array([0.0, -0.0, lo, hi, 1e30, -1e30, np.nextafter(np.float32(hi), np.float32(0))],
                        dtype=np.float32)
    return np.concatenate([v, grid, specials]).astype(np.float32)


# ---------------------------------------------------------------------------------------------
# Residual CNN workload (benchmark configuration 3: ResNet-50-shaped network as int8 convolutions in
# their matrix form, batch normalisation folded into a per-channel scale and bias, ReLU as a
# two-segment PWL table).  Stand-in for the paper's ResNet-50 / ImageNet experiments: random
# weights, inputs U(0, 1).
# ---------------------------------------------------------------------------------------------

RESNET_CONFIGS = {
    # the real layer shapes: 224 x 224 x 3 input, bottleneck stages (3, 4, 6, 3), 1000 classes
    "resnet50": dict(B=64, HW=224, stages=(3, 4, 6, 3), widths=(64, 128, 256, 512), classes=1000),
    # the same channel widths on 32 x 32 images, one block per stage (parity tests: every kernel
    # path of the big network at sizes the oracle finishes in a second)
    "resnet_tiny": dict(B=2, HW=32, stages=(1, 1, 1, 1), widths=(64, 128, 256, 512), classes=10),
    # channel counts that are multiples of nothing convenient (fallback paths)
    "resnet_odd": dict(B=3, HW=20, stages=(1, 2), widths=(12, 20), classes=7),
}
RELU_TABLE = ("relu", -8.0, 8.0, 2)  # chords of max(x, 0) on a symmetric range: k = {0, 1}, b = {0, 0}


def resnet_graph(cfg: dict) -> list:
    """The network as a list of operations over named NHWC tensors (shapes only)."""
    ops = []
    hw = cfg["HW"]
    w0 = cfg["widths"][0]

    def conv(name, src, dst, cin, cout, k, stride, pad, h, relu, resid=None):
        ho = (h + 2 * pad - k) // stride + 1
        ops.append(dict(op="conv", name=name, src=src, dst=dst, Cin=cin, Cout=cout, k=k, stride=stride,
                        pad=pad, H=h, Ho=ho, relu=relu, resid=resid))
        return ho

    h = conv("conv1", "x", "c1", 3, w0, 7, 2, 3, hw, True)
    ho = (h + 2 - 3) // 2 + 1
    ops.append(dict(op="maxpool", name="pool1", src="c1", dst="p1", C=w0, k=3, stride=2, pad=1, H=h, Ho=ho))
    h, cur, cin = ho, "p1", w0
    for si, (nblocks, mid) in enumerate(zip(cfg["stages"], cfg["widths"])):
        for bi in range(nblocks):
            stride = 2 if (bi == 0 and si > 0) else 1
            pre = f"s{si}b{bi}"
            cout = 4 * mid
            conv(pre + "a", cur, pre + "a", cin, mid, 1, 1, 0, h, True)
            h2 = conv(pre + "b", pre + "a", pre + "b", mid, mid, 3, stride, 1, h, True)
            short = cur
            if bi == 0:  # projection shortcut (channel count and / or resolution change)
                conv(pre + "d", cur, pre + "d", cin, cout, 1, stride, 0, h, False)
                short = pre + "d"
            conv(pre + "c", pre + "b", pre + "c", mid, cout, 1, 1, 0, h2, True, resid=short)
            h, cur, cin = h2, pre + "c", cout
    ops.append(dict(op="avgpool", name="avgpool", src=cur, dst="gap", C=cin, H=h))
    ops.append(dict(op="fc", name="fc", src="gap", dst="logits", Cin=cin, Cout=cfg["classes"]))
    return ops


def resnet_tensors(name: str, seed: int = 0, batch: int | None = None) -> dict:
    """Weights (one PCG64 stream, drawn in graph order: weight, folded-BN gain, bias per
    convolution; then the classifier) and the input image batch (its own stream, so that the
    weights do not depend on the batch size).  Weights ~ N(0, 2 / fan_in) quantised per tensor;
    folded batch-norm gain ~ 1 + N(0, 0.1^2) (0.25 + ... on the last convolution of a block and
    on projection shortcuts, which keeps the residual sums O(1)), bias ~ N(0, 0.1^2);
    images ~ U(0, 1) with scale 1/127."""
    cfg = dict(RESNET_CONFIGS[name])
    B = batch if batch is not None else cfg["B"]
    g = np.random.Generator(np.random.PCG64(seed))
    t = dict(cfg=cfg, B=B, graph=resnet_graph(cfg), w={}, s_w={}, gain={}, bias={})
    for op in t["graph"]:
        if op["op"] == "conv":
            k, cin, cout = op["k"], op["Cin"], op["Cout"]
            std = np.sqrt(2.0 / (k * k * cin))
            wt = (std * g.standard_normal((cout, k, k, cin), dtype=np.float32)).astype(np.float32)
            t["w"][op["name"]], t["s_w"][op["name"]] = quantize_sym(wt)
            base = 1.0 if op["relu"] and op["resid"] is None else 0.25
            t["gain"][op["name"]] = (base * (1.0 + 0.1 * g.standard_normal(cout))).astype(np.float64)
            t["bias"][op["name"]] = (0.1 * g.standard_normal(cout)).astype(np.float32)
        elif op["op"] == "fc":
            wt = (np.sqrt(1.0 / op["Cin"]) * g.standard_normal((op["Cout"], op["Cin"]), dtype=np.float32))
            t["w"]["fc"], t["s_w"]["fc"] = quantize_sym(wt.astype(np.float32))
            t["bias"]["fc"] = (0.1 * g.standard_normal(op["Cout"])).astype(np.float32)
    gi = np.random.Generator(np.random.PCG64(seed + 1000))
    img = gi.random((B, cfg["HW"], cfg["HW"], 3), dtype=np.float32)
    t["x"] = np.clip(np.rint(img.astype(np.float64) * 127.0), -127, 127).astype(np.int8)
    t["s_x"] = 1.0 / 127.0
    return t


def resnet_with_scales(t: dict, act: dict) -> dict:
    """Adds, per operation, the fp32 numbers both implementations receive (formed in binary64,
    rounded once): per-channel dequantisation scale alpha_vec = s_in * s_w * gain, residual scale,
    inverse output scale.  ``act`` maps tensor name -> scale (the input 'x' included)."""
    p = dict(t)
    p["alpha_vec"], p["resid_scale"], p["inv_s"], p["alpha"] = {}, {}, {}, {}
    f32 = lambda v: float(np.float32(v))  # noqa: E731
    for op in t["graph"]:
        n = op["name"]
        if op["op"] == "conv":
            p["alpha_vec"][n] = (act[op["src"]] * t["s_w"][n] * t["gain"][n]).astype(np.float32)
            p["resid_scale"][n] = f32(act[op["resid"]]) if op["resid"] else 0.0
            p["inv_s"][n] = f32(1.0 / act[op["dst"]])
        elif op["op"] == "avgpool":
            p["alpha"][n] = f32(act[op["src"]] / (op["H"] * op["H"]))
            p["inv_s"][n] = f32(1.0 / act[op["dst"]])
        elif op["op"] == "fc":
            p["alpha"][n] = f32(act[op["src"]] * t["s_w"][n])
    p["act_scales"] = dict(act)
    return p


def resnet_params(name: str, seed: int = 0, batch: int | None = None) -> dict:
    with open(SCALES_JSON) as f:
        table = json.load(f)
    key = f"{name}/seed{seed}"
    if key not in table:
        raise KeyError(f"no stored activation scales for {key}; run oracle/make_scales.py")
    return resnet_with_scales(resnet_tensors(name, seed, batch), table[key])
