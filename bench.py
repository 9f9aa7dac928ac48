"""Benchmark of the PWL int8 encoder layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload bert_base_layer]
                    [--layers L] [--nseg N]

A step is one pass of the whole hot path (nm_encoder_layer: QKV GEMM, scores, softmax-PWL, context,
output projection, LayerNorm-PWL, FFN1 + GELU-PWL, FFN2, LayerNorm-PWL; with --layers L > 1 the
L-layer stack, nm_encoder_stack) over one batch of seeded synthetic input that already sits in HBM.
The 512-token workloads default to their stack depth (bert_base_s512: 12, bert_large_s512: 24);
--nseg overrides the segment count of every table (the accuracy of the layer output against the
oracle's true-function mode is then reported next to the throughput).  Prints ONE JSON line: sequences/s, per-kernel roofline
figures measured live with HIP events on the launch stream, and the CPU oracle timed on the host
cores over the same workload (a reported baseline, not a target).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0   # MI355X dense int8 MFMA, published: 5.0 POP/s
PEAK_HBM_GBS = 8000.0     # MI355X HBM3E, published: 8 TB/s
# Plain vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-operations/s (one
# operation per lane per clock; the published 157.3 TFLOP/s counts packed two-wide FMAs, which this
# build does not emit).  The fused attention kernel is bound by it: per score the method's
# definition needs 18 scalar operations (row max 1; subtract, convert, scale 3; segment index:
# subtract, multiply, two-sided clamp, floor 5; k*t+b 1; row-sum add 1; e*r 1; requantisation:
# multiply, round, two-sided clamp, convert 5; the look-up itself not counted).
PEAK_VALU_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
ATTN_OPS_PER_SCORE = 18.0

# HBM-side traffic per launch comes from two rocprofv3 --pmc runs of this script (FETCH_SIZE, then
# WRITE_SIZE; KiB per dispatch), each scaled by what the same counter reads for a plain 64 MiB device
# copy.  Counters cannot be read from inside this process, so the figures are taken from the
# committed summary of those runs, which also records a hash of the kernel sources it was measured
# on: when the sources have changed since, the figure is stale and null is reported instead.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "encoder_layer_bert_base_layer_pmc_traffic.txt")
KERNEL_SOURCES = os.path.join(ROOT, "paper_2305_14405_amd", "csrc")


# the sources the encoder layer's kernels are built from (the convolution path is not among them)
LAYER_KERNEL_SOURCES = ("nm_device.h", "nm_internal.h", "nm_gemm_common.h", "nm_gemm_tile.h", "nm_gemm.hip",
                        "nm_rows.hip", "nm_attention.hip", "nm_layer.cpp")


def kernel_source_hash():
    import hashlib
    h = hashlib.sha256()
    for name in LAYER_KERNEL_SOURCES:
        with open(os.path.join(KERNEL_SOURCES, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def load_traffic():
    """kernel -> HBM bytes per launch, or {} when the recorded figures do not belong to these sources."""
    try:
        lines = open(TRAFFIC_FILE).read().splitlines()
    except OSError:
        return {}
    meta, rows = {}, {}
    for ln in lines:
        f = ln.split()
        if f[:1] == ["TRAFFIC_META"]:
            meta = dict(kv.split("=", 1) for kv in f[1:])
        elif f[:1] == ["TRAFFIC"]:
            kv = dict(x.split("=", 1) for x in f[1:])
            rows[kv["kernel"]] = (float(kv["fetch_kib"]), float(kv["write_kib"]))
    if meta.get("source_sha") != kernel_source_hash():
        return {}
    scale = float(meta["fetch_scale"])
    return {k: int(round((f * scale + w) * 1024)) for k, (f, w) in rows.items()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="bert_base_layer")
    ap.add_argument("--layers", type=int, default=0, help="stack depth (0: the workload's own)")
    ap.add_argument("--nseg", type=int, default=0, help="segments per table (0: the workload's own)")
    ap.add_argument("--table-flags", type=int, default=0,
                    help="table construction flags for every table (2: the paper's Algorithm 3 bias correction)")
    ap.add_argument("--dk-th", type=float, default=0.0,
                    help="slope threshold of the paper's Algorithm 2 (with --table-flags 4: neighbouring "
                         "primary segments whose slopes differ by less are merged)")
    ap.add_argument("--kernel-reps", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layernorm", choices=("auto", "fold", "separate"), default="auto",
                    help="LayerNorm inside the out-projection / FFN2 kernels (fold), as kernels of its own "
                         "(separate), or the library's choice (auto)")
    ap.add_argument("--graph", action="store_true", help="replay a HIP graph holding one step instead of launching it from the host")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 64 MiB device copy (reference for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE runs of this script)")
    ap.add_argument("--also", default="bert_base_s512,resnet50",
                    help="with the default workload and the CPU leg on: further workloads measured briefly "
                         "(few steps, one oracle run each) and reported under other_workloads; 'none' to skip")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    out = run_workload(args)
    if args.workload == "bert_base_layer" and not args.no_cpu_baseline and args.also != "none":
        others = []
        for name in args.also.split(","):
            a = argparse.Namespace(**vars(args))
            a.workload, a.steps, a.warmup, a.kernel_reps, a.brief = name, 10, 2, 10, True
            try:   # a problem in a side measurement must not cost the run its headline line
                o = run_workload(a)
                others.append({k: o[k] for k in ("value", "unit", "ms_per_step", "steps", "config", "roofline",
                                                 "cpu_baseline", "parity")})
            except Exception as e:  # noqa: BLE001
                others.append(dict(config=dict(workload=name), error=f"{type(e).__name__}: {e}"))
        out["other_workloads"] = others
    print(json.dumps(out))


def run_workload(args):
    if args.workload.startswith("resnet"):
        return bench_resnet(args)
    return bench_encoder(args)


def bench_encoder(args):
    import numpy as np
    import torch

    from paper_2305_14405_amd import binding as nm
    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = W.config(args.workload)
    if args.nseg:
        cfg["nseg"] = args.nseg
    n_layers = args.layers or {"bert_base_s512": 12, "bert_large_s512": 24}.get(args.workload, 1)
    stack = W.stack_params(args.workload, n_layers)
    p = stack[0]
    B, S, H, nh, F = (cfg[k] for k in ("B", "S", "H", "heads", "F"))
    M, d = B * S, cfg["H"] // cfg["heads"]
    order = ("gelu", "exp", "recip", "rsqrt")
    specs = [tuple(W.table_ranges(cfg)[n]) + (args.table_flags, 0.0, args.dk_th) for n in order]
    # distinct {k, b} pairs per table: what Algorithm 2's merging leaves of the primary segments
    distinct = {n: int(nm.nm_table_build_host(sp)[3]) for n, sp in zip(order, specs)}
    tables = nm.nm_build_tables(specs)          # the library's own table builder
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)  # noqa: E731
    devws = [{n: t(q[n]) for n in nm.LAYER_PTRS} for q in stack]
    ln_flags = {"auto": 0, "fold": nm.NM_LAYER_FOLD_LAYERNORM, "separate": nm.NM_LAYER_NO_FOLD_LAYERNORM}[args.layernorm]
    descs = [nm.make_layer_desc(q, dw, tables, flags=ln_flags) for q, dw in zip(stack, devws)]
    devw, desc = devws[0], descs[0]
    ws = torch.empty(nm.nm_encoder_stack_workspace(descs), dtype=torch.uint8, device=dev)
    x = t(p["x"])
    yq = torch.empty((M, H), dtype=torch.int8, device=dev)
    taps = dict(qkv=torch.empty((M, 3 * H), dtype=torch.int8, device=dev),
                scores=torch.empty((B, nh, S, S), dtype=torch.int32, device=dev),
                p=torch.empty((B, nh, S, S), dtype=torch.int8, device=dev),
                ctx=torch.empty((M, H), dtype=torch.int8, device=dev),
                attn=torch.empty((M, H), dtype=torch.float32, device=dev),
                ln1=torch.empty((M, H), dtype=torch.int8, device=dev),
                ffn1=torch.empty((M, F), dtype=torch.int8, device=dev),
                ffn2=torch.empty((M, H), dtype=torch.float32, device=dev))

    def step():
        # the hot path proper: intermediates live in the workspace, nothing optional is written
        if n_layers == 1:
            nm.nm_encoder_layer(desc, x, yq, None, ws)
        else:
            nm.nm_encoder_stack(descs, x, yq, None, ws)

    nm.nm_encoder_layer(desc, x, yq, None, ws, taps=taps)  # fills the buffers the per-kernel timings read

    if args.copy_calibration:
        src = torch.ones(64 << 20, dtype=torch.int8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)  # a plain copy kernel of known size: reads 64 MiB, writes 64 MiB
        torch.cuda.synchronize()
        del src, dst

    # A step is one call of the entry point from the host (the host runs ahead of the GPU, so the
    # kernels queue back to back).  --graph replays a HIP graph holding the call instead (the library
    # allocates nothing and never waits for the GPU, so the call can be captured); measured here it
    # is no faster (0.082 vs 0.078 ms per layer), so it is not the default.
    launch = "eager"
    run_step = step
    if args.graph:
        try:
            for _ in range(2):
                step()
            torch.cuda.synchronize()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step_graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(step_graph, stream=side):
                    step()
            torch.cuda.current_stream().wait_stream(side)
            want_q = yq.clone()
            for _ in range(3):  # every replay must reproduce the eager result
                yq.zero_()
                step_graph.replay()
                torch.cuda.synchronize()
                assert torch.equal(yq, want_q), "graph replay differs from the eager result"
            run_step, launch = step_graph.replay, "hip_graph"
        except AssertionError:
            raise
        except Exception as e:  # capture not available: host launches
            print(f"bench.py: graph capture failed ({e}); timing eager launches", file=sys.stderr)
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    seq_per_s = B / (ms_per_step * 1e-3)

    # ---- per-kernel durations, HIP events on the launch stream (torch's current stream) ------
    def timed(fn, reps):
        """Average duration of one launch of fn, HIP events on the launch stream.  The launches
        are recorded into a HIP graph once and replayed, so that the host-side cost of a launch
        through Python (~8 us) does not inflate kernels that run for only a few microseconds."""
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        graph = None
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    for _ in range(reps):
                        fn()
            torch.cuda.current_stream().wait_stream(side)
            graph.replay()
            torch.cuda.synchronize()
        except Exception:  # capture not available: plain back-to-back launches
            graph = None
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        if graph is not None:
            graph.replay()
        else:
            for _ in range(reps):
                fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps  # ms

    traffic = load_traffic() if args.workload == "bert_base_layer" else {}
    stages = [
        # the projection exactly as the layer launches it: one output scale per column third
        ("qkv_gemm", "mfma", 2.0 * M * 3 * H * H,
         lambda: nm.nm_gemm_pwl(x, devw["Wqkv"], bias=devw["bqkv"], alpha=p["alpha_qkv"], split_cols=H,
                                out_inv_scale3=(p["inv_s_q"], p["inv_s_k"], p["inv_s_v"]),
                                out_q=taps["qkv"])),
        ("attention_fused", "alu", float(B * nh * S * S),
         lambda: nm.nm_attention_pwl(taps["qkv"], B, S, H, nh, p["alpha_scores"], tables, 1, 2,
                                     p["inv_s_p"], p["alpha_ctx"], p["inv_s_ctx"], taps["ctx"])),
        ("softmax_pwl", "hbm", float(B * nh * S * S * 5),
         lambda: nm.nm_softmax_pwl(taps["scores"].view(-1, S), p["alpha_scores"], tables, 1, 2,
                                   p["inv_s_p"], out_q=taps["p"].view(-1, S))),
        ("out_proj_gemm", "mfma", 2.0 * M * H * H,
         lambda: nm.nm_gemm_pwl(taps["ctx"], devw["Wo"], bias=devw["bo"], alpha=p["alpha_o"],
                                resid=x, resid_scale=p["resid1_scale"], out_f32=taps["attn"])),
        ("layernorm_pwl", "hbm", float(M * H * 5),
         lambda: nm.nm_layernorm_pwl(taps["attn"], devw["gamma1"], devw["beta1"], p["eps1"], tables,
                                     3, p["inv_s_ln1"], out_q=taps["ln1"])),
        ("ffn1_gelu_gemm", "mfma", 2.0 * M * F * H,
         lambda: nm.nm_gemm_pwl(taps["ln1"], devw["W1"], bias=devw["b1"], alpha=p["alpha_1"],
                                tables=tables, table_idx=0, out_inv_scale=p["inv_s_ffn1"],
                                out_q=taps["ffn1"])),
        # the same GEMM with pre-activations spread over the whole GELU table (the workload's own
        # values touch only a few segments): shows what the LDS gather costs under bank conflicts
        ("ffn1_gelu_gemm_stress", "mfma", 2.0 * M * F * H,
         lambda: nm.nm_gemm_pwl(taps["ln1"], devw["W1"], bias=devw["b1"], alpha=p["alpha_1"] * 12.0,
                                tables=tables, table_idx=0, out_inv_scale=p["inv_s_ffn1"] / 12.0,
                                out_q=stress_out)),
        ("ffn2_gemm", "mfma", 2.0 * M * H * F,
         lambda: nm.nm_gemm_pwl(taps["ffn1"], devw["W2"], bias=devw["b2"], alpha=p["alpha_2"],
                                resid=taps["ln1"], resid_scale=p["resid2_scale"],
                                out_f32=taps["ffn2"])),
    ]
    stress_out = torch.empty((M, F), dtype=torch.int8, device=dev)
    kernels = []
    for name, bound, work, fn in stages:
        try:
            ms = timed(fn, args.kernel_reps)
        except nm.NmError as e:  # e.g. the fused attention kernel does not cover this shape
            if e.status != nm.NM_ERR_UNSUPPORTED:
                raise
            continue
        if bound == "mfma":
            ach, peak, unit = work / (ms * 1e-3) / 1e12, PEAK_INT8_TOPS, "TOP/s"
        elif bound == "alu":
            ach, peak, unit = work * ATTN_OPS_PER_SCORE / (ms * 1e-3) / 1e12, PEAK_VALU_TOPS, "Tops/s"
        else:
            ach, peak, unit = work / (ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
        kernels.append(dict(kernel=name, bound=bound, ms=round(ms, 5), achieved=round(ach, 2),
                            peak=peak, unit=unit, frac=round(ach / peak, 4),
                            traffic=traffic.get(name)))
    brief = getattr(args, "brief", False)
    # the HBM-bound row kernels again at shapes beyond the last-level cache (the softmax shape is
    # that of the 12-layer BERT-base workload: 16 x 12 x 512 rows of 512 scores)
    big, rot = [], []
    if not brief:
        big, rot = row_kernel_sections(torch, nm, timed, tables, devw, p, dev, M, H, F, B, nh, S)
    # the slowest kernel the layer really launches (at shapes the fused attention kernel covers, the
    # stand-alone softmax row kernel is timed for its bandwidth figure only)
    fused_attn = H // nh == 64 and S <= 512 and H % 16 == 0
    for k in kernels:
        k["in_layer"] = k["kernel"] not in (("softmax_pwl" if fused_attn else "attention_fused"),
                                            "ffn1_gelu_gemm_stress")
    dom = max((k for k in kernels if k["in_layer"]), key=lambda k: k["ms"])
    roofline = dict(bound=dom["bound"], achieved=dom["achieved"], peak=dom["peak"], unit=dom["unit"],
                    frac=dom["frac"], traffic=dom["traffic"], kernel=dom["kernel"],
                    note="int8 MFMA rate (2 operations per multiply-accumulate)" if dom["bound"] == "mfma"
                    else "plain vector ALU, 18 scalar operations per attention score")
    gemm_ops = sum(2.0 * M * n * k for n, k in ((3 * H, H), (H, H), (F, H), (H, F)))
    gemm_ms = sum(k["ms"] for k in kernels if k["bound"] == "mfma" and k["in_layer"])
    row_bytes = float(B * nh * S * S * 5 + 2 * M * H * 5)
    ln_ms = next(k["ms"] for k in kernels if k["kernel"] == "layernorm_pwl")
    row_ms = next(k["ms"] for k in kernels if k["kernel"] == "softmax_pwl") + 2 * ln_ms
    summary = dict(int8_mfma_util_pct=round(100 * gemm_ops / (gemm_ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 2),
                   nonlinear_hbm_gbs=round(row_bytes / (row_ms * 1e-3) / 1e9, 1),
                   nonlinear_hbm_gbs_large=round(sum(k["achieved"] for k in big[:3]) / 3, 1) if big else None,
                   sum_kernel_ms=round(sum(k["ms"] for k in kernels if k["in_layer"]) + ln_ms, 4),
                   note="softmax_pwl is the stand-alone row kernel (timed on its own; the layer uses the "
                        "fused attention kernel at this shape); layernorm_pwl runs twice per layer")

    # ---- CPU oracle on the host cores: the same workload, bounded sample ----------------------
    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        oid = {"gelu": O.F_GELU, "exp": O.F_EXP, "recip": O.F_RECIP, "rsqrt": O.F_RSQRT}
        if args.table_flags & 4:
            ot = {n: O.build_table_merged(oid[s[0]], s[1], s[2], s[3], args.dk_th, flags=args.table_flags & ~4)[0]
                  for n, s in zip(order, specs)}
        else:
            ot = {n: O.build_table(oid[s[0]], s[1], s[2], s[3], flags=args.table_flags) for n, s in zip(order, specs)}
        # bounded sample: whole batch for the 128-token layer, two sequences of layer 0 otherwise
        # (sequences are independent, so a batch subset is the same computation on fewer rows)
        b_sub = B if (n_layers == 1 and M * H <= 4096 * 768) else min(B, 2)
        p_sub = dict(p, B=b_sub)
        x_sub = np.ascontiguousarray(p["x"][:b_sub * S])
        n_runs, c0 = 0, time.perf_counter()
        while True:
            want = O.encoder_layer(p_sub, ot, x_sub, want_taps=False)
            n_runs += 1
            if brief or time.perf_counter() - c0 > 12.0 or n_runs >= 64:
                break
        cpu_s = (time.perf_counter() - c0) / n_runs
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        sample = (f"{n_runs} run(s) of layer 0 of {args.workload} on {b_sub} of {B} sequences, "
                  f"{cpu_s:.2f} s per run")
        if n_layers > 1:
            sample += f"; value = {b_sub} / ({n_layers} layers x {cpu_s:.2f} s), extrapolated linearly over layers"
        cpu_baseline = dict(value=round(b_sub / (cpu_s * n_layers), 4), unit="sequences/s", cores=cores,
                            kind="oracle", sample=sample)
        # the same on one thread (one sequence, one run), for the per-core figure
        try:
            if brief:
                raise OSError("skipped in a brief run")
            import ctypes
            gomp = ctypes.CDLL("libgomp.so.1")
            gomp.omp_set_num_threads(1)
            p_one = dict(p, B=1)
            c1 = time.perf_counter()
            O.encoder_layer(p_one, ot, np.ascontiguousarray(p["x"][:S]), want_taps=False)
            one_s = time.perf_counter() - c1
            gomp.omp_set_num_threads(cores)
            cpu_baseline["value_1_thread"] = round(1.0 / (one_s * n_layers), 4)
        except OSError:
            pass
        # layer 0 on the GPU (library-built tables) against the oracle's layer 0 (oracle-built tables:
        # may differ in the last bit), and against the oracle's true-function mode (same quantised
        # network, exact GELU / exp / 1/x / rsqrt in binary64): the PWL approximation error
        yq0 = torch.empty((M, H), dtype=torch.int8, device=dev)
        yf0 = torch.empty((M, H), dtype=torch.float32, device=dev)
        nm.nm_encoder_layer(desc, x, yq0, yf0, ws)
        torch.cuda.synchronize()
        rows = b_sub * S
        diff = np.abs(yq0[:rows].cpu().numpy().astype(int) - want["y_q"].astype(int))
        exact, _ = O.encoder_layer_exact(p_sub, ot, x_sub, quantise=True)
        err = np.abs(yf0[:rows].cpu().numpy().astype(np.float64) - exact)
        parity = dict(int8_max_abs_diff=int(diff.max()), int8_mismatch_frac=float((diff > 0).mean()),
                      note="layer 0, library-built tables vs oracle-built tables (may differ in the last bit)",
                      pwl_vs_exact_f=dict(nseg=int(cfg["nseg"]), max_abs=float(err.max()),
                                          mean_abs=float(err.mean()),
                                          rel_rms=float(np.sqrt((err ** 2).mean() / (exact ** 2).mean())),
                                          note="fp32 layer-0 output vs the oracle's true-function mode "
                                               "of the same quantised layer"))

    out = dict(metric="PWL encoder-layer sequences/s + int8 MFMA util % + nonlinear-kernel HBM GB/s",
               value=round(seq_per_s, 1), unit="sequences/s", n_gpus=1, steps=args.steps,
               warmup=args.warmup, ms_per_step=round(ms_per_step, 5), higher_is_better=True,
               scaling="weak", vs_baseline=None, dtype="int8", dtype_note="int8 operands, int32 accumulation, fp32 epilogue",
               data="synthetic", config=dict(workload=args.workload, B=B, S=S, H=H, heads=nh, F=F,
                                             nseg=cfg["nseg"], layers=n_layers,
                                             table_flags=args.table_flags, dk_th=args.dk_th,
                                             distinct_segments=distinct, launch=launch, layernorm=args.layernorm),
               roofline=roofline, cpu_baseline=cpu_baseline, kernels=kernels, row_kernels_large=big,
               row_kernels_layer_shape_rotated=rot,
               summary=summary,
               parity=parity)
    return out


def row_kernel_sections(torch, nm, timed, tables, devw, p, dev, M, H, F, B, nh, S):
    """the HBM-bound row kernels at shapes beyond the last-level cache, and at the layer's own shapes
    over rotated buffer sets"""
    def rotated(make, call, bytes_per_launch, n_sets=0):
        n_sets = n_sets or max(2, -(-(320 << 20) // bytes_per_launch))
        sets = [make() for _ in range(n_sets)]
        turn = [0]

        def fn():
            call(*sets[turn[0] % n_sets])
            turn[0] += 1
        ms = timed(fn, 4 * n_sets if n_sets <= 4 else 2 * n_sets)
        return ms, n_sets

    # beyond-cache shapes, three buffer sets in rotation: a launch never finds its input in the 256 MB
    # last-level cache (one 200 MB buffer timed back to back is partly served from there and reads
    # 0.83 of the HBM peak instead of 0.65)
    big = []
    ms, n_sets = rotated(lambda: (torch.randn((65536, H), device=dev), torch.empty((65536, H), dtype=torch.int8, device=dev)),
                         lambda a, o: nm.nm_layernorm_pwl(a, devw["gamma1"], devw["beta1"], p["eps1"], tables, 3,
                                                          p["inv_s_ln1"], out_q=o), 0, 3)
    big.append(dict(kernel="layernorm_pwl", shape=[65536, H], buffer_sets=n_sets, ms=round(ms, 5),
                    achieved=round(65536 * H * 5 / (ms * 1e-3) / 1e9, 1)))
    n_big = 16 * 12 * 512
    ms, n_sets = rotated(lambda: (torch.randint(-3000, 3000, (n_big, 512), dtype=torch.int32, device=dev),
                                  torch.empty((n_big, 512), dtype=torch.int8, device=dev)),
                         lambda a, o: nm.nm_softmax_pwl(a, p["alpha_scores"], tables, 1, 2, p["inv_s_p"], out_q=o), 0, 3)
    big.append(dict(kernel="softmax_pwl", shape=[n_big, 512], buffer_sets=n_sets, ms=round(ms, 5),
                    achieved=round(n_big * 512 * 5 / (ms * 1e-3) / 1e9, 1)))
    ms, n_sets = rotated(lambda: (torch.randn((1 << 26,), device=dev), torch.empty((1 << 26,), dtype=torch.int8, device=dev)),
                         lambda a, o: nm.nm_pwl_apply(a, 1.0, tables, 0, p["inv_s_ffn1"], out_q=o), 0, 3)
    big.append(dict(kernel="pwl_apply", shape=[1 << 26], buffer_sets=n_sets, ms=round(ms, 5),
                    achieved=round((1 << 26) * 5 / (ms * 1e-3) / 1e9, 1)))
    # context: a plain device copy of the same footprint (2^26 fp32 values read and written)
    ms, n_sets = rotated(lambda: (torch.randn((1 << 26,), device=dev), torch.empty((1 << 26,), device=dev)),
                         lambda a, o: o.copy_(a), 0, 3)
    big.append(dict(kernel="device copy (torch copy_, for comparison)", shape=[1 << 26], buffer_sets=n_sets, ms=round(ms, 5),
                    achieved=round((1 << 26) * 8 / (ms * 1e-3) / 1e9, 1)))
    # the layer's own row shapes again, each launch on a different copy of the buffers: the copies
    # together exceed the last-level cache (timed back to back on one buffer, these shapes are served
    # from cache and say nothing about HBM)
    rot = []
    ms, n_sets = rotated(lambda: (torch.randn((M, H), device=dev), torch.empty((M, H), dtype=torch.int8, device=dev)),
                         lambda a, o: nm.nm_layernorm_pwl(a, devw["gamma1"], devw["beta1"], p["eps1"], tables, 3,
                                                          p["inv_s_ln1"], out_q=o), M * H * 5)
    rot.append(dict(kernel="layernorm_pwl", shape=[M, H], buffer_sets=n_sets, ms=round(ms, 5),
                    achieved=round(M * H * 5 / (ms * 1e-3) / 1e9, 1)))
    n_sc = B * nh * S
    ms, n_sets = rotated(lambda: (torch.randint(-3000, 3000, (n_sc, S), dtype=torch.int32, device=dev),
                                  torch.empty((n_sc, S), dtype=torch.int8, device=dev)),
                         lambda a, o: nm.nm_softmax_pwl(a, p["alpha_scores"], tables, 1, 2, p["inv_s_p"], out_q=o),
                         n_sc * S * 5)
    rot.append(dict(kernel="softmax_pwl", shape=[n_sc, S], buffer_sets=n_sets, ms=round(ms, 5),
                    achieved=round(n_sc * S * 5 / (ms * 1e-3) / 1e9, 1)))
    ms, n_sets = rotated(lambda: (torch.randn((M * F,), device=dev), torch.empty((M * F,), dtype=torch.int8, device=dev)),
                         lambda a, o: nm.nm_pwl_apply(a, 1.0, tables, 0, p["inv_s_ffn1"], out_q=o), M * F * 5)
    rot.append(dict(kernel="pwl_apply", shape=[M * F], buffer_sets=n_sets, ms=round(ms, 5),
                    achieved=round(M * F * 5 / (ms * 1e-3) / 1e9, 1)))
    for k in big + rot:
        k.update(bound="hbm", peak=PEAK_HBM_GBS, unit="GB/s", frac=round(k["achieved"] / PEAK_HBM_GBS, 4))
    return big, rot


def graph_timed(torch, fn, reps):
    """Average duration (ms) of one call of fn: recorded reps times into a HIP graph, the replay
    bracketed by events on the launch stream."""
    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(reps):
                fn()
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    graph.replay()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def bench_resnet(args):
    """benchmark configuration 3: the ResNet-50-shaped int8 network (convolutions in matrix form, folded
    batch norm, ReLU as a two-segment PWL table), one C-ABI call per operation.  value = images/s."""
    import numpy as np
    import torch

    from paper_2305_14405_amd import binding as nm
    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    p = W.resnet_params(args.workload, 0)
    B = p["B"]
    tables = nm.nm_build_tables([W.RELU_TABLE])
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)  # noqa: E731
    cur = {"x": t(p["x"])}
    calls, keep, convs = [], [], []
    ws_need = 256
    for op in p["graph"]:
        n = op["name"]
        if op["op"] == "conv":
            y = torch.empty((B, op["Ho"], op["Ho"], op["Cout"]), dtype=torch.int8, device=dev)
            wt, bi, av = t(p["w"][n]), t(p["bias"][n]), t(p["alpha_vec"][n])
            keep += [wt, bi, av]
            d = nm.make_conv_desc(cur[op["src"]], wt, op["stride"], op["pad"], bias=bi, alpha_vec=av,
                                  resid=cur[op["resid"]] if op["resid"] else None,
                                  resid_scale=p["resid_scale"][n], tables=tables,
                                  table_idx=0 if op["relu"] else -1, out_inv_scale=p["inv_s"][n], out_q=y)
            ws_need = max(ws_need, nm.nm_conv2d_workspace(d))
            convs.append((op, d))
            calls.append(("conv", n, d))
            cur[op["dst"]] = y
        elif op["op"] == "maxpool":
            y = torch.empty((B, op["Ho"], op["Ho"], op["C"]), dtype=torch.int8, device=dev)
            calls.append(("maxpool", n, (cur[op["src"]], y, op["k"], op["stride"], op["pad"])))
            cur[op["dst"]] = y
        elif op["op"] == "avgpool":
            y = torch.empty((B, op["C"]), dtype=torch.int8, device=dev)
            calls.append(("avgpool", n, (cur[op["src"]].view(B, -1, op["C"]), p["alpha"][n], p["inv_s"][n], y)))
            cur[op["dst"]] = y
        elif op["op"] == "fc":
            logits = torch.empty((B, op["Cout"]), dtype=torch.float32, device=dev)
            wt, bi = t(p["w"][n]), t(p["bias"][n])
            keep += [wt, bi]
            calls.append(("fc", n, (cur[op["src"]], wt, bi, p["alpha"][n], logits)))
    ws = torch.empty(ws_need, dtype=torch.uint8, device=dev)

    def run(call):
        kind, _, a = call
        if kind == "conv":
            nm.nm_conv2d_pwl(a, ws)
        elif kind == "maxpool":
            nm.nm_maxpool_i8(a[0], a[1], a[2], a[3], a[4])
        elif kind == "avgpool":
            nm.nm_avgpool_i8(a[0], a[1], a[2], out_q=a[3])
        else:
            nm.nm_gemm_pwl(a[0], a[1], bias=a[2], alpha=a[3], out_f32=a[4])

    # the whole network as one C-ABI call (nm_cnn_run over the list of steps)
    ops = []
    for kind, _, a in calls:
        if kind == "conv":
            ops.append(nm.cnn_op_conv(a))
        elif kind == "maxpool":
            ops.append(nm.cnn_op_maxpool(a[0], a[1], a[2], a[3], a[4]))
        elif kind == "avgpool":
            ops.append(nm.cnn_op_avgpool(a[0], a[1], a[2], out_q=a[3]))
        else:
            ops.append(nm.cnn_op_gemm(nm.make_gemm_desc(a[0], a[1], bias=a[2], alpha=a[3], out_f32=a[4])))
    assert nm.nm_cnn_workspace(ops) <= ws_need
    op_array = nm._op_array(ops)

    def step():
        nm.nm_cnn_run(ops, ws, op_array=op_array)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_eager = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_per_step, launch_mode = ms_eager, "eager"
    # The 57 launches of a batch leave dispatch gaps; the same call recorded once into a HIP graph
    # and replayed closes most of them.  Every replay is checked against the eager result (with
    # eager work and synchronisation in between) before its timing is used.
    eager_logits = logits.clone()
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        same = True
        for _ in range(3):
            logits.zero_()
            graph.replay()
            torch.cuda.synchronize()
            same = same and bool(torch.equal(logits, eager_logits))
            step()
            torch.cuda.synchronize()
        if not same:
            print("graph replay differs from the eager result: not used", file=sys.stderr)
        if same:
            t0 = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            ms_graph = (time.perf_counter() - t0) * 1e3 / args.steps
            print(f"graph replay {ms_graph:.4f} ms vs eager {ms_eager:.4f} ms", file=sys.stderr)
            if ms_graph < ms_per_step:
                ms_per_step, launch_mode = ms_graph, "hip graph replay (checked against eager on 3 replays)"
    except Exception as e:  # capture not available: keep the eager figure
        launch_mode = f"eager (graph capture failed: {type(e).__name__})"

    kernels = []
    for c in calls:
        ms = graph_timed(torch, lambda c=c: run(c), max(2, args.kernel_reps // 5))
        entry = dict(kernel=c[1], kind=c[0], ms=round(ms, 5))
        if c[0] == "conv":
            op = next(o for o, d in convs if o["name"] == c[1])
            ops = 2.0 * B * op["Ho"] ** 2 * op["Cout"] * op["k"] ** 2 * op["Cin"]
            ach = ops / (ms * 1e-3) / 1e12
            entry.update(bound="mfma", achieved=round(ach, 1), peak=PEAK_INT8_TOPS, unit="TOP/s",
                         frac=round(ach / PEAK_INT8_TOPS, 4),
                         shape=f"M={B * op['Ho'] ** 2} N={op['Cout']} K={op['k'] ** 2 * op['Cin']} "
                               f"k{op['k']} s{op['stride']}")
        kernels.append(entry)
    conv_k = [k for k in kernels if k["kind"] == "conv"]
    dom = max(conv_k, key=lambda k: k["ms"])
    total_ops = sum(2.0 * B * o["Ho"] ** 2 * o["Cout"] * o["k"] ** 2 * o["Cin"] for o, _ in convs)
    conv_ms = sum(k["ms"] for k in conv_k)
    roofline = dict(bound="mfma", achieved=dom["achieved"], peak=PEAK_INT8_TOPS, unit="TOP/s", frac=dom["frac"],
                    traffic=None, kernel=dom["kernel"] + " (" + dom["shape"] + ")",
                    note="int8 MFMA rate in TOP/s (2 ops per multiply-accumulate); slowest convolution")
    summary = dict(int8_mfma_util_pct=round(100 * total_ops / (conv_ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 2),
                   conv_gop_per_image=round(total_ops / B / 1e9, 3), sum_kernel_ms=round(sum(k["ms"] for k in kernels), 4))

    cpu_baseline = parity = None
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        b_sub = B   # the whole batch: about ten seconds of oracle time at batch 64
        p_sub = W.resnet_params(args.workload, 0, batch=b_sub)
        c0 = time.perf_counter()
        want = O.resnet_forward(p_sub)["logits"]
        cpu_s = time.perf_counter() - c0
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu_baseline = dict(value=round(b_sub / cpu_s, 3), unit="images/s", cores=cores, kind="oracle",
                            sample=f"one pass of the whole network on {b_sub} of {B} images, {cpu_s:.2f} s")
        step()
        torch.cuda.synchronize()
        got = logits[:b_sub].cpu().numpy()
        parity = dict(logits_bit_identical=bool(np.array_equal(got.view(np.uint32), want.view(np.uint32))),
                      max_abs_diff=float(np.abs(got - want).max()),
                      note=f"fp32 logits of the first {b_sub} images, GPU vs oracle (library-built ReLU table)")

    cfg = p["cfg"]
    out = dict(metric="PWL encoder-layer sequences/s + int8 MFMA util % + nonlinear-kernel HBM GB/s",
               value=round(B / (ms_per_step * 1e-3), 1), unit="images/s", n_gpus=1, steps=args.steps,
               warmup=args.warmup, ms_per_step=round(ms_per_step, 5), higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="int8", dtype_note="int8 operands, int32 accumulation, fp32 epilogue", data="synthetic",
               config=dict(workload=args.workload, B=B, image=cfg["HW"], stages=list(cfg["stages"]),
                           widths=list(cfg["widths"]), classes=cfg["classes"], launch=launch_mode,
                           ms_per_step_eager=round(ms_eager, 5)),
               roofline=roofline, cpu_baseline=cpu_baseline, kernels=kernels, summary=summary, parity=parity)
    return out


if __name__ == "__main__":
    main()
