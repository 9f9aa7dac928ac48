"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, its host table
builder agrees with the oracle's, and argument validation returns errors without touching a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2305_14405_amd import binding as nm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return nm.load(preload_torch=False)


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "nm.h")).read()
    declared = set(re.findall(r"^(?:int32_t|void|const char\*)\s+(nm_[a-z_0-9]+)\(", header, re.M))
    assert declared == set(nm.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.nm_version() >= 1000
    assert nm.nm_last_error() is not None


def test_no_torch_types_in_signatures():
    header = open(os.path.join(ROOT, "include", "nm.h")).read()
    assert "torch" not in header and "at::" not in header and 'extern "C"' in header


FUNCS = ["gelu", "exp", "recip", "rsqrt", "sqrt", "relu", "identity"]
RANGE = {"gelu": (-8.0, 8.0), "exp": (-16.0, 0.0), "recip": (1.0, 128.0), "rsqrt": (1e-3, 64.0),
         "sqrt": (0.25, 64.0), "relu": (-8.0, 8.0), "identity": (-3.0, 5.0)}
OID = {"gelu": 0, "exp": 1, "recip": 2, "rsqrt": 3, "relu": 4, "sqrt": 5, "identity": 6}


def ulps(a, b):
    a = np.asarray(a, np.float32)
    b = np.asarray(b, np.float32)
    return np.abs(a.astype(np.float64) - b.astype(np.float64)) / np.maximum(
        np.spacing(np.maximum(np.abs(a), np.abs(b))).astype(np.float64), 1e-45)


@pytest.mark.parametrize("name", FUNCS)
@pytest.mark.parametrize("nseg", [1, 2, 64, 128, 1000])
@pytest.mark.parametrize("flags", [0, nm.NM_TABLE_BIAS_CORRECT])
def test_host_table_builder_matches_oracle(lib, oracle, name, nseg, flags):
    lo, hi = RANGE[name]
    k, b, inv_w, nd = nm.nm_table_build_host((name, lo, hi, nseg, flags))
    t = oracle.build_table(OID[name], lo, hi, nseg, flags=oracle.FLAG_BIAS_CORRECT if flags else 0)
    assert inv_w == t.inv_w
    assert nd == nseg
    # two independent binary64 evaluations rounded to fp32: equal up to the last bit, except where
    # b is a tiny difference of large terms (GELU's tails), bounded absolutely instead
    tol_abs = 4e-7 * max(abs(lo), abs(hi)) * np.maximum(np.abs(t.k), 1e-3)
    assert np.all((ulps(k, t.k) <= 1) | (np.abs(k - t.k) <= 1e-9))
    assert np.all((ulps(b, t.b) <= 1) | (np.abs(b - t.b) <= tol_abs))


@pytest.mark.parametrize("name,dk", [("gelu", 0.1), ("exp", 0.05), ("recip", 0.02)])
def test_host_merged_table_matches_oracle(lib, oracle, name, dk):
    lo, hi = {"gelu": (-4.0, 4.0), "exp": (-8.0, 0.0), "recip": (1.0, 9.0)}[name]
    nprim = 16
    k, b, inv_w, nd = nm.nm_table_build_host((name, lo, hi, nprim, nm.NM_TABLE_MERGE, 0.0, dk))
    t, n = oracle.build_table_merged(OID[name], lo, hi, nprim, dk)
    assert nd == n
    assert np.all(ulps(k, t.k) <= 1) and np.all((ulps(b, t.b) <= 1) | (np.abs(b - t.b) < 1e-6))
    assert inv_w == t.inv_w


def test_validation_errors_without_gpu(lib):
    E = nm.NmError
    for spec in [("exp", 0.0, 0.0, 8), ("exp", 0.0, 1.0, 0), (99, 0.0, 1.0, 8), ("recip", 0.0, 1.0, 8),
                 ("rsqrt", -1.0, 1.0, 8)]:
        with pytest.raises(E) as ei:
            nm.nm_table_build_host(spec)
        assert ei.value.status == nm.NM_ERR_INVALID_ARG
    with pytest.raises(E) as ei:
        nm.nm_table_build_host(("exp", 0.0, 1.0, 5000))
    assert ei.value.status == nm.NM_ERR_UNSUPPORTED
    assert "NM_MAX_SEGMENTS" in nm.nm_last_error()
    # table objects: bad descriptors are rejected before any HIP call
    with pytest.raises(E) as ei:
        nm.nm_build_tables([("exp", 1.0, 0.0, 8)], stream=0)
    assert ei.value.status == nm.NM_ERR_INVALID_ARG
    with pytest.raises(E) as ei:
        nm.nm_build_tables([("exp", -1.0, 0.0, 8)] * 17, stream=0)
    assert ei.value.status == nm.NM_ERR_INVALID_ARG
    assert nm.nm_tables_count(None) == 0
    lib.nm_tables_destroy(None)  # null-safe


def test_compute_entry_points_validate_before_launch(lib):
    z = C.c_void_p(0)
    one = C.c_void_p(256)  # a non-null dummy; never dereferenced because validation fails first
    d = nm.GemmDesc()
    assert lib.nm_gemm_pwl(None, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_gemm_pwl(C.byref(d), z) == nm.NM_ERR_INVALID_ARG         # M = N = K = 0
    d.M, d.N, d.K = 4, 4, 4
    assert lib.nm_gemm_pwl(C.byref(d), z) == nm.NM_ERR_INVALID_ARG         # NULL operands
    d.A, d.W = 256, 256
    assert lib.nm_gemm_pwl(C.byref(d), z) == nm.NM_ERR_INVALID_ARG         # no output
    d.out_q = 256
    d.K = 70000
    assert lib.nm_gemm_pwl(C.byref(d), z) == nm.NM_ERR_UNSUPPORTED
    d.K = 4
    d.table_idx = 0                                                          # table without tables
    assert lib.nm_gemm_pwl(C.byref(d), z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_softmax_pwl(None, 0, 1.0, 1, 1, None, 0, 1, 1.0, one, None, None, None, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_softmax_pwl(one, 7, 1.0, 1, 1, None, 0, 1, 1.0, one, None, None, None, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_softmax_pwl(one, 0, 1.0, 1, 5000, None, 0, 1, 1.0, one, None, None, None, z) == nm.NM_ERR_UNSUPPORTED
    assert lib.nm_softmax_pwl(one, 0, 1.0, 1, 8, None, 0, 1, 1.0, None, None, None, None, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_softmax_pwl(one, 0, 1.0, 1, 8, None, 0, 1, 1.0, one, None, None, None, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_layernorm_pwl(one, one, None, 1e-5, 1, 8, None, 0, 1.0, one, None, None, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_layernorm_pwl(one, one, one, 1e-5, 1, 0, None, 0, 1.0, one, None, None, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_pwl_apply(one, 0, 1.0, -1, None, 0, 1.0, one, None, None, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_attn_scores(one, 1, 8, 10, 3, one, z) == nm.NM_ERR_INVALID_ARG  # H % heads
    assert lib.nm_attn_context(one, one, 1, 5000, 8, 1, 1.0, 1.0, one, z) == nm.NM_ERR_UNSUPPORTED
    ld = nm.LayerDesc()
    n = C.c_size_t()
    assert lib.nm_encoder_layer_workspace(C.byref(ld), C.byref(n)) == nm.NM_ERR_INVALID_ARG
    ld.B, ld.S, ld.H, ld.heads, ld.F = 32, 128, 768, 12, 3072
    assert lib.nm_encoder_layer_workspace(C.byref(ld), C.byref(n)) == nm.NM_OK
    M, H, F, SS = 4096, 768, 3072, 32 * 12 * 128 * 128
    # head size 64 and S <= 512: the fused attention kernel keeps scores and probabilities in registers
    need = M * 3 * H + M * H + M * H * 4 + M * H + M * F + M * H * 4
    assert need <= n.value <= need + 8 * 256
    ld2 = nm.LayerDesc()
    ld2.B, ld2.S, ld2.H, ld2.heads, ld2.F = 2, 640, 128, 2, 256      # S > 512: three-kernel attention
    n2 = C.c_size_t()
    assert lib.nm_encoder_layer_workspace(C.byref(ld2), C.byref(n2)) == nm.NM_OK
    M2, SS2 = 1280, 2 * 2 * 640 * 640
    need2 = M2 * 3 * 128 + SS2 * 4 + SS2 + M2 * 128 + M2 * 128 * 4 + M2 * 128 + M2 * 256 + M2 * 128 * 4
    assert need2 <= n2.value <= need2 + 8 * 256
    assert lib.nm_encoder_layer(C.byref(ld), one, one, None, one, n, None, z) == nm.NM_ERR_INVALID_ARG
    # scales and multipliers are checked before any GPU call: finite, score scale positive
    for name in nm.LAYER_FLOATS:
        setattr(ld, name, 1.0)
    ld.eps1 = ld.eps2 = 1e-5
    for name, bad in (("alpha_scores", float("inf")), ("alpha_scores", 0.0), ("alpha_1", float("nan")),
                      ("inv_s_out", float("-inf")), ("eps2", float("nan"))):
        keep = getattr(ld, name)
        setattr(ld, name, bad)
        assert lib.nm_encoder_layer(C.byref(ld), one, one, None, one, n, None, z) == nm.NM_ERR_INVALID_ARG
        assert b"multiplier" in lib.nm_last_error() or b"alpha_scores" in lib.nm_last_error()
        setattr(ld, name, keep)
    # the entry point that allocates nothing: validation and the size limit come before any GPU call
    assert lib.nm_encoder_layer_noalloc(None, one, one, None, z) == nm.NM_ERR_INVALID_ARG
    ld3 = nm.LayerDesc()
    ld3.B, ld3.S, ld3.H, ld3.heads, ld3.F = 16, 512, 768, 12, 3072
    assert lib.nm_encoder_layer_noalloc(C.byref(ld3), one, one, None, z) == nm.NM_ERR_WORKSPACE
    assert b"built-in buffer" in lib.nm_last_error()
    assert n.value <= nm.NM_NOALLOC_MAX_WORKSPACE
    # stack: two activation buffers on top of the largest layer workspace; layers must agree on B, S, H
    arr = (nm.LayerDesc * 3)()
    for i in range(3):
        arr[i].B, arr[i].S, arr[i].H, arr[i].heads, arr[i].F = 32, 128, 768, 12, 3072 if i != 1 else 1024
    ns = C.c_size_t()
    assert lib.nm_encoder_stack_workspace(arr, 3, C.byref(ns)) == nm.NM_OK
    assert ns.value == n.value + 2 * M * H
    assert lib.nm_encoder_stack_workspace(arr, 0, C.byref(ns)) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_encoder_stack_workspace(None, 3, C.byref(ns)) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_encoder_stack(arr, 3, None, one, None, one, ns, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_encoder_stack(arr, 3, one, None, None, one, ns, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_encoder_stack(arr, 3, one, one, None, None, ns, z) == nm.NM_ERR_WORKSPACE
    arr[2].S = 64
    assert lib.nm_encoder_stack_workspace(arr, 3, C.byref(ns)) == nm.NM_ERR_INVALID_ARG
    assert b"layer 2" in lib.nm_last_error()
    ld.heads = 7
    assert lib.nm_encoder_layer_workspace(C.byref(ld), C.byref(n)) == nm.NM_ERR_INVALID_ARG


def test_conv_and_pool_entry_points_validate_before_launch(lib):
    """nm_conv2d_workspace / nm_conv2d_pwl / pooling: geometry and pointer checks happen on the
    host before any HIP call; the workspace size follows the route the shape takes."""
    z = C.c_void_p(0)
    one = C.c_void_p(256)
    n = C.c_size_t()
    d = nm.ConvDesc()
    assert lib.nm_conv2d_workspace(None, C.byref(n)) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_conv2d_workspace(C.byref(d), C.byref(n)) == nm.NM_ERR_INVALID_ARG   # all zero
    d.B, d.H, d.W, d.Cin, d.Cout, d.kh, d.kw, d.stride, d.pad = 2, 8, 8, 3, 4, 3, 3, 1, 1
    d.table_idx = -1
    assert lib.nm_conv2d_workspace(C.byref(d), None) == nm.NM_ERR_INVALID_ARG
    # odd channel count: patch matrix (K = 27 -> 64 bytes per row) plus the padded filter rows
    assert lib.nm_conv2d_workspace(C.byref(d), C.byref(n)) == nm.NM_OK
    assert n.value == 2 * 8 * 8 * 64 + 4 * 64
    assert lib.nm_conv2d_pwl(C.byref(d), None, 0, z) == nm.NM_ERR_INVALID_ARG        # no output
    d.out_q = 256
    assert lib.nm_conv2d_pwl(C.byref(d), None, 0, z) == nm.NM_ERR_INVALID_ARG        # NULL x / w
    d.x, d.w = 256, 256
    assert lib.nm_conv2d_pwl(C.byref(d), None, 0, z) == nm.NM_ERR_WORKSPACE
    assert lib.nm_conv2d_pwl(C.byref(d), one, 16, z) == nm.NM_ERR_WORKSPACE          # too small
    assert b"workspace" in lib.nm_last_error()
    d.table_idx = 0                                                                    # table without tables
    assert lib.nm_conv2d_pwl(C.byref(d), one, n, z) == nm.NM_ERR_INVALID_ARG
    d.table_idx = -1
    # a 1x1 / stride 1 convolution and a 64-channel 3x3 convolution need no workspace
    d.Cin, d.kh, d.kw, d.pad = 3, 1, 1, 0
    assert lib.nm_conv2d_workspace(C.byref(d), C.byref(n)) == nm.NM_OK and n.value == 0
    d.Cin, d.kh, d.kw, d.pad = 64, 3, 3, 1
    assert lib.nm_conv2d_workspace(C.byref(d), C.byref(n)) == nm.NM_OK and n.value == 0
    d.kh, d.kw, d.pad = 9, 9, 0                                                        # filter larger than the image
    assert lib.nm_conv2d_workspace(C.byref(d), C.byref(n)) == nm.NM_ERR_INVALID_ARG
    d.kh, d.kw, d.Cin = 40, 40, 64                                                     # kh*kw*Cin > 65536
    d.H = d.W = 64
    assert lib.nm_conv2d_workspace(C.byref(d), C.byref(n)) == nm.NM_ERR_UNSUPPORTED
    d.B = 0                                                                            # empty batch: nothing to do
    d.kh = d.kw = 3
    assert lib.nm_conv2d_pwl(C.byref(d), None, 0, z) == nm.NM_OK
    # pooling
    assert lib.nm_maxpool_i8(one, 1, 8, 8, 4, 3, 2, 3, one, z) == nm.NM_ERR_INVALID_ARG      # pad >= k
    assert lib.nm_maxpool_i8(one, 1, 8, 8, 4, 0, 2, 0, one, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_maxpool_i8(None, 1, 8, 8, 4, 3, 2, 1, one, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_maxpool_i8(None, 0, 8, 8, 4, 3, 2, 1, None, z) == nm.NM_OK
    assert lib.nm_avgpool_i8(one, 1, 49, 8, 1.0, 1.0, None, None, z) == nm.NM_ERR_INVALID_ARG  # no output
    assert lib.nm_avgpool_i8(one, 1, 0, 8, 1.0, 1.0, one, None, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_avgpool_i8(None, 1, 49, 8, 1.0, 1.0, one, None, z) == nm.NM_ERR_INVALID_ARG
    assert lib.nm_avgpool_i8(one, 1, 1 << 24, 8, 1.0, 1.0, one, None, z) == nm.NM_ERR_UNSUPPORTED


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus N with N > 1 exits with a message (before it
    touches torch or the GPU)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=60)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
