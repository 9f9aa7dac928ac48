"""Calibration of the synthetic workloads' static activation scales (test infrastructure).

Runs the oracle's binary64 true-function encoder layer, without rounding any activation, over the
seeded input of each named workload and records the largest magnitude of every activation that
the int8 pipeline quantises (Section 3.2 step 1 of the paper: the input range of an operator is
obtained by running the model).  scale = absmax / 127.  The softmax output P is the exception: it
lies in [0, 1] whatever the input, so its scale is fixed at 1 / 127.

A stack of layers is calibrated layer by layer: layer l's calibration run reads the true-function
output of layer l-1, quantised with that layer's calibrated output scale (as layer 0 reads a
quantised input), so every layer gets activation scales of its own.

Writes ``workloads/workload_scales.json``.  Calls nothing but the oracle and the input
generator.  Usage: python -m oracle.make_scales [workload ...] [stack:<workload>:<layers> ...]
"""
from __future__ import annotations

import json
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

from oracle import oracle as O  # noqa: E402
import workloads as W  # noqa: E402

_FUNC = {"gelu": O.F_GELU, "exp": O.F_EXP, "recip": O.F_RECIP, "rsqrt": O.F_RSQRT}
# batch used for calibration: activations are i.i.d. over sequences, a few are enough
CALIB_BATCH = {"bert_base_s512": 2, "bert_large_s512": 1}
DEFAULT = ("tiny", "ragged", "long_seq", "bert_base_layer", "bert_base_s512", "bert_large_s512",
           "resnet_tiny", "resnet_odd", "resnet50")
RESNET_CALIB_BATCH = {"resnet50": 2}


def oracle_tables(cfg):
    return {n: O.build_table(_FUNC[f], lo, hi, nseg)
            for n, (f, lo, hi, nseg) in W.table_ranges(cfg).items()}


def calibrate_resnet(name: str, seed: int = 0) -> dict:
    """The residual CNN: its only nonlinearity, ReLU, is exact as a PWL table, so the calibration
    run is the oracle's own network with each tensor's scale taken from its fp32 values as it goes."""
    t = W.resnet_tensors(name, seed, RESNET_CALIB_BATCH.get(name))
    return O.resnet_forward(t, calibrate=True)["scales"]


def calibrate(name: str, seed: int = 0) -> dict:
    if name in W.RESNET_CONFIGS:
        return calibrate_resnet(name, seed)
    cfg = W.config(name)
    t = W.layer_tensors(cfg, seed)
    if name in CALIB_BATCH:
        nb = CALIB_BATCH[name]
        t["x"] = t["x"][: nb * cfg["S"]].copy()
        t["B"] = nb
    p = W.with_scales(t, W.unit_scales())
    _, obs = O.encoder_layer_exact(p, oracle_tables(cfg), t["x"], quantise=False)
    scales = {n: obs[n] / 127.0 for n in W.ACT_NAMES}
    scales["p"] = 1.0 / 127.0
    scales["observed"] = obs
    return scales


# stacks the tests and the benchmark run: workload -> depth
STACKS = {"tiny": 3, "ragged": 2, "bert_base_layer": 2, "bert_base_s512": 12, "bert_large_s512": 24}


def calibrate_stack(name: str, n_layers: int) -> list:
    """Per-layer activation scales of a stack (layer l has the weights of seed l)."""
    import numpy as np
    cfg = W.config(name)
    nb = CALIB_BATCH.get(name)
    out = []
    x, s_x = None, None
    for l in range(n_layers):
        t = W.layer_tensors(cfg, l)
        if nb:
            t["x"] = t["x"][: nb * cfg["S"]].copy()
            t["B"] = nb
        if l > 0:
            t["x"], t["s_x"] = x, s_x
        p = W.with_scales(t, W.unit_scales())
        y, obs = O.encoder_layer_exact(p, oracle_tables(cfg), t["x"], quantise=False)
        scales = {n: obs[n] / 127.0 for n in W.ACT_NAMES}
        scales["p"] = 1.0 / 127.0
        out.append(scales)
        # the next layer's input: this layer's output as the int8 code the pipeline would pass on
        s_x = scales["out"]
        x = np.clip(np.rint(y / s_x), -127, 127).astype(np.int8)
    return out


def main(argv):
    stacks = [a for a in argv if a.startswith("stack:")]
    argv = [a for a in argv if not a.startswith("stack:")]
    names = argv or (DEFAULT if not stacks else ())
    table = {}
    if os.path.exists(W.SCALES_JSON):
        with open(W.SCALES_JSON) as f:
            table = json.load(f)
    for name in names:
        t0 = time.time()
        table[f"{name}/seed0"] = calibrate(name, 0)
        print(f"{name}: {time.time() - t0:.1f} s", {k: round(v, 5) for k, v in
                                                    table[f'{name}/seed0'].items()
                                                    if k != "observed"}, flush=True)
    if not argv and not stacks:
        stacks = [f"stack:{n}:{d}" for n, d in STACKS.items()]
    for spec in stacks:
        _, name, depth = spec.split(":")
        t0 = time.time()
        table[f"{name}/stack"] = calibrate_stack(name, int(depth))
        print(f"stack {name} x{depth}: {time.time() - t0:.1f} s; output scales",
              [round(s["out"], 5) for s in table[f"{name}/stack"]], flush=True)
    with open(W.SCALES_JSON, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)


if __name__ == "__main__":
    main(sys.argv[1:])
