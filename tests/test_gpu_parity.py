"""GPU parity: every C-ABI compute entry point against the CPU oracle, element by element, on the
same seeded inputs (teacher forcing: each kernel is fed the oracle's inputs for that stage).

Bar: int32 accumulators, segment indices and int8 codes bit-exact; fp32 values within 1e-5
relative (the normative operation order makes them bit-reproducible in practice; the test also
records how many differ at all)."""
import numpy as np
import pytest
import torch

from paper_2305_14405_amd import binding as nm
import workloads as W

pytestmark = pytest.mark.gpu

OID = {"gelu": 0, "exp": 1, "recip": 2, "rsqrt": 3, "relu": 4, "sqrt": 5, "identity": 6}
DEV = "cuda:0"


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def both_tables(oracle, specs, flags=0):
    """Oracle tables and a device table object holding exactly the oracle's k, b."""
    ot = [oracle.build_table(OID[f], lo, hi, n, flags=flags) for (f, lo, hi, n) in specs]
    dt = nm.nm_tables_from_arrays([(f, lo, hi, n, flags) for (f, lo, hi, n) in specs],
                                  [t.k for t in ot], [t.b for t in ot])
    return ot, dt


def assert_f32_close(got, want, what):
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape
    tol = 1e-5 * np.abs(want) + 1e-30
    with np.errstate(invalid="ignore"):
        bad = ~((np.abs(got.astype(np.float64) - want.astype(np.float64)) <= tol) | (got == want) |
                (np.isnan(got) & np.isnan(want)))
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} beyond 1e-5 relative"
    nbits = int((got.view(np.uint32) != want.view(np.uint32)).sum())
    print(f"[parity] {what}: fp32 within 1e-5 relative; {nbits} of {got.size} not bit-identical")


def assert_exact(got, want, what):
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, what
    n = int((got != want).sum())
    assert n == 0, f"{what}: {n} of {got.size} differ"


# ---- element-wise PWL -----------------------------------------------------------------------

SPECS = [("gelu", -8.0, 8.0, 64), ("exp", -16.0, 0.0, 128), ("recip", 1.0, 64.0, 64),
         ("rsqrt", 1e-3, 64.0, 37), ("relu", -8.0, 8.0, 2), ("gelu", -8.0, 8.0, 4096)]


@pytest.mark.parametrize("ti", range(len(SPECS)))
def test_pwl_apply_fp32_and_int32(oracle, ti):
    ot, dt = both_tables(oracle, SPECS)
    f, lo, hi, n = SPECS[ti]
    x = W.sweep_values(lo, hi, 100003, seed=ti)
    x = np.concatenate([x, np.array([np.nan, np.inf, -np.inf], np.float32)])
    for inv in (1.0, 17.5):
        y, q, s = oracle.pwl_apply(x, ot[ti], alpha=1.0, out_inv_scale=inv)
        xd = dev(x)
        yq, yf, ys = (torch.empty(x.size, dtype=torch.int8, device=DEV),
                      torch.empty(x.size, dtype=torch.float32, device=DEV),
                      torch.empty(x.size, dtype=torch.int16, device=DEV))
        nm.nm_pwl_apply(xd, 1.0, dt, ti, inv, out_q=yq, out_f32=yf, dbg_seg=ys)
        assert_exact(host(ys).view(np.uint16), s, f"pwl_apply seg {f}")
        assert_exact(host(yq), q, f"pwl_apply int8 {f}")
        assert_f32_close(host(yf), y, f"pwl_apply fp32 {f}")
        # fp32 in, int8 out alone (the kernel variant the layer's activations take), guard bytes behind
        yq1 = torch.full((x.size + 16,), 55, dtype=torch.int8, device=DEV)
        nm.nm_pwl_apply(xd, 1.0, dt, ti, inv, out_q=yq1, n=x.size)
        assert_exact(host(yq1)[:x.size], q, f"pwl_apply int8 alone {f}")
        assert np.all(host(yq1)[x.size:] == 55)
    # int32 input with a dequantisation scale
    g = np.random.default_rng(ti)
    a = g.integers(-40000, 40000, size=70001, dtype=np.int32)
    alpha = float(np.float32((hi - lo) / 60000.0))
    y, q, s = oracle.pwl_apply(a, ot[ti], alpha=alpha, out_inv_scale=9.0)
    yq = torch.empty(a.size, dtype=torch.int8, device=DEV)
    ys = torch.empty(a.size, dtype=torch.int16, device=DEV)
    nm.nm_pwl_apply(dev(a), alpha, dt, ti, 9.0, out_q=yq, dbg_seg=ys)
    assert_exact(host(ys).view(np.uint16), s, "pwl_apply i32 seg")
    assert_exact(host(yq), q, "pwl_apply i32 int8")


def test_pwl_apply_edge_sizes_and_misaligned(oracle):
    ot, dt = both_tables(oracle, SPECS[:1])
    x = W.sweep_values(-8.0, 8.0, 64, seed=9)
    for n in (0, 1, 3, 4, 5, 63, 64, 65):
        big = dev(np.concatenate([np.zeros(1, np.float32), x[:n]]))
        src = big[1:]                          # 4-byte but not 16-byte aligned
        yq = torch.full((n + 9,), 77, dtype=torch.int8, device=DEV)
        yf = torch.full((n + 9,), -5.0, dtype=torch.float32, device=DEV)
        nm.nm_pwl_apply(src, 1.0, dt, 0, 8.0, out_q=yq[1:], out_f32=yf[1:], n=n)
        y, q, _ = oracle.pwl_apply(x[:n], ot[0], out_inv_scale=8.0)
        assert_exact(host(yq)[1:n + 1], q, "misaligned int8")
        assert_f32_close(host(yf)[1:n + 1], y, "misaligned fp32")
        assert np.all(host(yq)[n + 1:] == 77) and host(yq)[0] == 77   # nothing outside [0, n)
        assert np.all(host(yf)[n + 1:] == -5.0)


def test_clamp_input_flag(oracle):
    ot, dt = both_tables(oracle, [("exp", -16.0, 0.0, 64)], flags=1)
    x = np.concatenate([W.sweep_values(-16.0, 0.0, 5000, seed=2),
                        np.array([np.nan, np.inf, -np.inf, -16.0, 0.0], np.float32)])
    y, q, s = oracle.pwl_apply(x, ot[0], out_inv_scale=100.0)
    yf = torch.empty(x.size, dtype=torch.float32, device=DEV)
    ys = torch.empty(x.size, dtype=torch.int16, device=DEV)
    nm.nm_pwl_apply(dev(x), 1.0, dt, 0, 100.0, out_f32=yf, dbg_seg=ys)
    assert_exact(host(ys).view(np.uint16), s, "clamp seg")
    assert_f32_close(host(yf), y, "clamp fp32")


# ---- tables built with Algorithm 3 (bias correction) and Algorithm 2 (segment merging) ---------

# (label, library flags, e_th, dk_th)
ELASTIC = [("bias", nm.NM_TABLE_BIAS_CORRECT, 0.0, 0.0),
           ("bias_threshold", nm.NM_TABLE_BIAS_CORRECT, 2e-3, 0.0),
           ("merge", nm.NM_TABLE_MERGE, 0.0, 0.02),
           ("merge_bias", nm.NM_TABLE_MERGE | nm.NM_TABLE_BIAS_CORRECT, 0.0, 0.02),
           ("merge_two_level", nm.NM_TABLE_MERGE | nm.NM_TABLE_COMPACT, 0.0, 0.02)]


def elastic_tables(oracle, specs, flags, e_th, dk_th):
    """Oracle tables built with the given options, a device object holding exactly their k, b, and
    a device object the library built itself from the same descriptors."""
    oflags = oracle.FLAG_BIAS_CORRECT if flags & nm.NM_TABLE_BIAS_CORRECT else 0
    ot = []
    for (f, lo, hi, n) in specs:
        if flags & nm.NM_TABLE_MERGE:
            t, n_merged = oracle.build_table_merged(OID[f], lo, hi, n, dk_th, flags=oflags, e_th=e_th)
            assert 1 <= n_merged <= n
        else:
            t = oracle.build_table(OID[f], lo, hi, n, flags=oflags, e_th=e_th)
        ot.append(t)
    # injected arrays are the expanded form; with the two-level flag the library folds them back into
    # runs of equal lines (the same values, looked up through the cell map)
    iflags = (nm.NM_TABLE_MERGE | nm.NM_TABLE_COMPACT) if flags & nm.NM_TABLE_COMPACT else 0
    injected = nm.nm_tables_from_arrays([(f, lo, hi, n, iflags) for (f, lo, hi, n) in specs],
                                        [t.k for t in ot], [t.b for t in ot])
    built = nm.nm_build_tables([(f, lo, hi, n, flags, e_th, dk_th) for (f, lo, hi, n) in specs])
    return ot, injected, built


ELASTIC_SPECS = [("gelu", -8.0, 8.0, 128), ("exp", -16.0, 0.0, 64), ("recip", 1.0, 64.0, 64),
                 ("rsqrt", 1e-3, 64.0, 256)]


@pytest.mark.parametrize("label,flags,e_th,dk_th", ELASTIC)
def test_elastic_tables_pwl_apply(oracle, label, flags, e_th, dk_th):
    """nm_pwl_apply on tables built with Algorithm 3 / Algorithm 2: exact with the oracle's arrays
    injected, within one int8 code with the tables the library builds itself."""
    ot, injected, built = elastic_tables(oracle, ELASTIC_SPECS, flags, e_th, dk_th)
    plain = [oracle.build_table(OID[f], lo, hi, n) for (f, lo, hi, n) in ELASTIC_SPECS]
    changed = 0
    for ti, (f, lo, hi, n) in enumerate(ELASTIC_SPECS):
        changed += int(not (np.array_equal(ot[ti].k, plain[ti].k) and np.array_equal(ot[ti].b, plain[ti].b)))
        x = W.sweep_values(lo, hi, 50021, seed=40 + ti)
        y, q, s = oracle.pwl_apply(x, ot[ti], out_inv_scale=11.0)
        yq = torch.empty(x.size, dtype=torch.int8, device=DEV)
        yf = torch.empty(x.size, dtype=torch.float32, device=DEV)
        ys = torch.empty(x.size, dtype=torch.int16, device=DEV)
        nm.nm_pwl_apply(dev(x), 1.0, injected, ti, 11.0, out_q=yq, out_f32=yf, dbg_seg=ys)
        assert_exact(host(ys).view(np.uint16), s, f"{label} {f} segments")
        assert_exact(host(yq), q, f"{label} {f} int8")
        assert_f32_close(host(yf), y, f"{label} {f} fp32")
        nm.nm_pwl_apply(dev(x), 1.0, built, ti, 11.0, out_q=yq, dbg_seg=ys)
        assert_exact(host(ys).view(np.uint16), s, f"{label} {f} segments, library-built table")
        d = np.abs(host(yq).astype(int) - q.astype(int))
        assert d.max() <= 1 and (d > 0).mean() < 1e-3, f"{label} {f}: library-built table off by {d.max()}"
    # the options did change the tables (with a threshold only where a segment's bias exceeds it)
    assert changed == len(ELASTIC_SPECS) or (e_th > 0 and changed >= 1)


@pytest.mark.parametrize("label,flags,e_th,dk_th", ELASTIC)
def test_elastic_tables_gemm_epilogue(oracle, label, flags, e_th, dk_th):
    """nm_gemm_pwl with a GELU table built with Algorithm 3 / Algorithm 2 (streaming and generic
    kernels)."""
    ot, injected, built = elastic_tables(oracle, [("gelu", -8.0, 8.0, 128)], flags, e_th, dk_th)
    for (M, N, K) in [(256, 384, 256), (70, 50, 96)]:
        d = W.gemm_inputs(M, N, K, seed=M + K, full_range=False)
        alpha = float(np.float32(6.0 / (20 * 20 * np.sqrt(K))))
        r = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha, table=ot[0], out_inv_scale=25.0)
        oq = torch.empty((M, N), dtype=torch.int8, device=DEV)
        seg = torch.empty((M, N), dtype=torch.int16, device=DEV)
        nm.nm_gemm_pwl(dev(d["A"]), dev(d["W"]), bias=dev(d["bias"]), alpha=alpha, tables=injected,
                       table_idx=0, out_inv_scale=25.0, out_q=oq, dbg_seg=seg)
        assert_exact(host(seg).view(np.uint16), r["seg"], f"{label} gemm segments")
        assert_exact(host(oq), r["q"], f"{label} gemm int8")
        oq2 = torch.empty_like(oq)
        nm.nm_gemm_pwl(dev(d["A"]), dev(d["W"]), bias=dev(d["bias"]), alpha=alpha, tables=injected,
                       table_idx=0, out_inv_scale=25.0, out_q=oq2)       # the specialised epilogue
        assert_exact(host(oq2), r["q"], f"{label} gemm int8, specialised epilogue")
        nm.nm_gemm_pwl(dev(d["A"]), dev(d["W"]), bias=dev(d["bias"]), alpha=alpha, tables=built,
                       table_idx=0, out_inv_scale=25.0, out_q=oq2)
        diff = np.abs(host(oq2).astype(int) - r["q"].astype(int))
        assert diff.max() <= 1 and (diff > 0).mean() < 1e-3


@pytest.mark.parametrize("label,flags,e_th,dk_th", ELASTIC)
def test_elastic_tables_encoder_layer(oracle, label, flags, e_th, dk_th):
    """The tiny encoder layer with all four tables built with Algorithm 3 / Algorithm 2."""
    want, got = run_layer(oracle, "tiny", elastic=(flags, e_th, dk_th))
    for k in ("qkv", "scores", "p", "ctx", "ln1", "ffn1", "y_q"):
        assert_exact(got[k], want[k], f"{label} tiny layer {k}")
    for k in ("attn", "ffn2", "y_f32"):
        assert_f32_close(got[k], want[k], f"{label} tiny layer {k}")
    want, got = run_layer(oracle, "tiny", library_tables=True, elastic=(flags, e_th, dk_th))
    diff = np.abs(got["y_q"].astype(int) - want["y_q"].astype(int))
    assert diff.max() <= 1 and (diff > 0).mean() < 2e-3
    assert np.allclose(got["y_f32"], want["y_f32"], rtol=1e-4, atol=1e-5)


def test_encoder_layer_two_level_gelu_table_headline_shape(oracle):
    """The headline layer with merged tables in the two-level form: FFN1 looks its GELU table up in
    two levels inside the large-tile kernel (the other kernels read the expanded form); every stage
    equals the oracle's layer on the same merged tables."""
    want, got = run_layer(oracle, "bert_base_layer", elastic=(nm.NM_TABLE_MERGE | nm.NM_TABLE_COMPACT, 0.0, 0.01))
    for k in ("qkv", "ctx", "ln1", "ffn1", "y_q"):
        assert_exact(got[k], want[k], f"two-level tables, headline layer {k}")
    for k in ("attn", "ffn2", "y_f32"):
        assert_f32_close(got[k], want[k], f"two-level tables, headline layer {k}")


# ---- merged tables looked up in two levels (cell of x, merged segment of the cell) ------------

@pytest.mark.parametrize("name,lo,hi,nprim,dk", [("gelu", -4.0, 4.0, 16, 0.1), ("gelu", -8.0, 8.0, 256, 0.01),
                                                  ("exp", -16.0, 0.0, 128, 0.01), ("rsqrt", 1e-3, 64.0, 256, 0.05)])
@pytest.mark.parametrize("clamp", [0, 1])
def test_two_level_tables_pwl_apply(oracle, name, lo, hi, nprim, dk, clamp):
    """nm_pwl_apply on a merged table kept in two levels (NM_TABLE_COMPACT) against the oracle's
    direct evaluation of the merged table (search over Algorithm 2's start points): outputs exact,
    reported cell exact, the library's cell map equal to the oracle's start points.  First case: the
    paper's worked GELU example (threshold 0.1, primary length 0.5: 8 segments for 16 cells)."""
    mt = oracle.build_table_merged_direct(OID[name], lo, hi, nprim, dk, flags=clamp)
    te, _ = oracle.build_table_merged(OID[name], lo, hi, nprim, dk, flags=clamp)
    flags = nm.NM_TABLE_MERGE | nm.NM_TABLE_COMPACT | clamp
    injected = nm.nm_tables_from_arrays([(name, lo, hi, nprim, flags)], [te.k], [te.b])
    built = nm.nm_build_tables([(name, lo, hi, nprim, flags, 0.0, dk)])
    for tb, exact in ((injected, True), (built, False)):
        cmap, ck, cb = nm.nm_tables_get_compact(tb, 0)
        assert np.array_equal(cmap, mt.cell_to_segment()) and ck.size == mt.nseg
        if exact:
            assert np.array_equal(ck, mt.k) and np.array_equal(cb, mt.b)
        print(f"[two-level] {name} {nprim} cells -> {ck.size} segments: {8 * ck.size + nprim} bytes in LDS "
              f"instead of {8 * nprim}")
    x = np.concatenate([W.sweep_values(lo, hi, 60001, seed=3), np.array([np.nan, np.inf, -np.inf], np.float32)])
    y, q, s, c = oracle.pwl_apply_merged(x, mt, out_inv_scale=21.0)
    for n in (x.size, 7):   # vector path and the scalar tail path
        yq = torch.empty(n, dtype=torch.int8, device=DEV)
        yf = torch.empty(n, dtype=torch.float32, device=DEV)
        ys = torch.empty(n, dtype=torch.int16, device=DEV)
        nm.nm_pwl_apply(dev(x[:n]), 1.0, injected, 0, 21.0, out_q=yq, out_f32=yf, dbg_seg=ys)
        assert_exact(host(ys).view(np.uint16), c[:n], "two-level: primary cell")
        assert_exact(mt.cell_to_segment()[host(ys).view(np.uint16)], s[:n], "two-level: merged segment")
        assert_exact(host(yq), q[:n], "two-level: int8")
        assert_f32_close(host(yf), y[:n], "two-level: fp32")
    yq = torch.empty(x.size, dtype=torch.int8, device=DEV)
    nm.nm_pwl_apply(dev(x), 1.0, built, 0, 21.0, out_q=yq)
    d = np.abs(host(yq).astype(int) - q.astype(int))
    assert d.max() <= 1 and (d > 0).mean() < 1e-3
    # int32 input
    a = np.random.default_rng(8).integers(-40000, 40000, size=30001, dtype=np.int32)
    alpha = float(np.float32((hi - lo) / 60000.0))
    y, q, s, c = oracle.pwl_apply_merged(a, mt, alpha=alpha, out_inv_scale=9.0)
    yq = torch.empty(a.size, dtype=torch.int8, device=DEV)
    nm.nm_pwl_apply(dev(a), alpha, injected, 0, 9.0, out_q=yq)
    assert_exact(host(yq), q, "two-level: int32 input")


@pytest.mark.parametrize("M,N,K", [(256, 384, 256), (70, 50, 96)])
def test_two_level_table_gemm_epilogue(oracle, M, N, K):
    """nm_gemm_pwl with a two-level GELU table (streaming and generic kernels): the same outputs as
    the oracle's GEMM followed by its direct evaluation of the merged table."""
    lo, hi, nprim, dk = -8.0, 8.0, 128, 0.01
    mt = oracle.build_table_merged_direct(OID["gelu"], lo, hi, nprim, dk)
    te, _ = oracle.build_table_merged(OID["gelu"], lo, hi, nprim, dk)
    dt = nm.nm_tables_from_arrays([("gelu", lo, hi, nprim, nm.NM_TABLE_MERGE | nm.NM_TABLE_COMPACT)], [te.k], [te.b])
    d = W.gemm_inputs(M, N, K, seed=M + K + 2, full_range=False)
    alpha = float(np.float32(6.0 / (20 * 20 * np.sqrt(K))))
    pre = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha)["y"]      # fp32 pre-activations
    y, q, s, c = oracle.pwl_apply_merged(pre.ravel(), mt, out_inv_scale=25.0)
    oq = torch.empty((M, N), dtype=torch.int8, device=DEV)
    of = torch.empty((M, N), dtype=torch.float32, device=DEV)
    seg = torch.empty((M, N), dtype=torch.int16, device=DEV)
    nm.nm_gemm_pwl(dev(d["A"]), dev(d["W"]), bias=dev(d["bias"]), alpha=alpha, tables=dt, table_idx=0,
                   out_inv_scale=25.0, out_q=oq, out_f32=of, dbg_seg=seg)
    assert_exact(host(seg).view(np.uint16).ravel(), c, "two-level gemm: primary cell")
    assert_exact(host(oq).ravel(), q, "two-level gemm: int8")
    assert_f32_close(host(of).ravel(), y, "two-level gemm: fp32")
    oq2 = torch.empty_like(oq)
    nm.nm_gemm_pwl(dev(d["A"]), dev(d["W"]), bias=dev(d["bias"]), alpha=alpha, tables=dt, table_idx=0,
                   out_inv_scale=25.0, out_q=oq2)
    assert_exact(host(oq2).ravel(), q, "two-level gemm: int8 only")
    assert len(np.unique(s)) > 5


@pytest.mark.parametrize("M,N,K,nprim,dk", [(4096, 3072, 768, 128, 0.01), (3900, 784, 512, 256, 0.001), (8192, 1024, 512, 1024, 0.002)])
def test_two_level_table_in_the_tile_kernel_sampled(oracle, M, N, K, nprim, dk):
    """int8 output through a two-level GELU table at shapes the large-tile kernel takes (256 x 192,
    128 x 128 with ragged edges, 256 x 128; up to 1024 primary cells): its own epilogue looks the cell
    byte up first and the merged segment's line second.  The oracle computes 64 sampled rows: its GEMM,
    then its direct evaluation of the merged table."""
    lo, hi = -8.0, 8.0
    mt = oracle.build_table_merged_direct(OID["gelu"], lo, hi, nprim, dk)
    te, _ = oracle.build_table_merged(OID["gelu"], lo, hi, nprim, dk)
    assert mt.nseg <= 256
    dt = nm.nm_tables_from_arrays([("gelu", lo, hi, nprim, nm.NM_TABLE_MERGE | nm.NM_TABLE_COMPACT)], [te.k], [te.b])
    d = W.gemm_inputs(M, N, K, seed=M + K + 3, full_range=False)
    alpha = float(np.float32(9.0 / (20 * 20 * np.sqrt(K))))
    rows = np.unique(np.concatenate([np.array([0, 1, 127, 128, 255, 256, M - 129, M - 2, M - 1]),
                                     np.random.default_rng(M).choice(M, 55, replace=False)]))
    pre = oracle.gemm_pwl(np.ascontiguousarray(d["A"][rows]), d["W"], bias=d["bias"], alpha=alpha)["y"]
    y, q, s, c = oracle.pwl_apply_merged(pre.ravel(), mt, out_inv_scale=25.0)
    oq = torch.full((M + 1, N), 77, dtype=torch.int8, device=DEV)
    nm.nm_gemm_pwl(dev(d["A"]), dev(d["W"]), bias=dev(d["bias"]), alpha=alpha, tables=dt, table_idx=0,
                   out_inv_scale=25.0, out_q=oq, M=M)
    got = host(oq)
    assert_exact(got[rows].ravel(), q, f"two-level table, tile kernel, {nprim} cells -> {mt.nseg} segments")
    assert np.all(got[M] == 77)
    assert len(np.unique(s)) > 5


def test_two_level_table_limits():
    """More than 256 merged segments do not fit the byte map; the other entry points use a two-level
    table's expanded form (same results)."""
    with pytest.raises(nm.NmError) as ei:
        nm.nm_build_tables([("exp", -16.0, 0.0, 512, nm.NM_TABLE_MERGE | nm.NM_TABLE_COMPACT, 0.0, 0.0)])
    assert ei.value.status == nm.NM_ERR_UNSUPPORTED
    t = nm.nm_build_tables([("rsqrt", 1e-3, 64.0, 64, nm.NM_TABLE_MERGE | nm.NM_TABLE_COMPACT, 0.0, 0.05),
                            ("rsqrt", 1e-3, 64.0, 64, nm.NM_TABLE_MERGE, 0.0, 0.05)])
    x = torch.randn((33, 200), device=DEV)
    g = torch.ones(200, device=DEV)
    b = torch.zeros(200, device=DEV)
    q0 = torch.empty((33, 200), dtype=torch.int8, device=DEV)
    q1 = torch.empty_like(q0)
    nm.nm_layernorm_pwl(x, g, b, 1e-5, t, 0, 20.0, out_q=q0)
    nm.nm_layernorm_pwl(x, g, b, 1e-5, t, 1, 20.0, out_q=q1)
    assert torch.equal(q0, q1)


# ---- softmax-PWL ------------------------------------------------------------------------------

@pytest.mark.parametrize("rows,cols", [(37, 1), (37, 5), (19, 64), (101, 128), (37, 200), (37, 512),
                                       (9, 777), (5, 1024), (3, 4096), (0, 128)])
@pytest.mark.parametrize("dtype", ["i32", "f32"])
def test_softmax_pwl(oracle, rows, cols, dtype):
    ot, dt = both_tables(oracle, [("exp", -16.0, 0.0, 128), ("recip", 1.0, float(max(64, cols)), 128)])
    a = W.score_rows(rows, cols, seed=rows * 7 + cols)
    alpha = 3e-4
    x = a if dtype == "i32" else (a.astype(np.float32) * np.float32(0.37))
    r = oracle.softmax_pwl(x, alpha, ot[0], ot[1], 127.0) if rows else None
    xd = dev(x)
    oq = torch.empty((rows, cols), dtype=torch.int8, device=DEV)
    of = torch.empty((rows, cols), dtype=torch.float32, device=DEV)
    se = torch.empty((rows, cols), dtype=torch.int16, device=DEV)
    sr = torch.empty((max(rows, 1),), dtype=torch.int16, device=DEV)
    nm.nm_softmax_pwl(xd, alpha, dt, 0, 1, 127.0, out_q=oq, out_f32=of, dbg_seg_exp=se,
                      dbg_seg_recip=sr, rows=rows, cols=cols)
    torch.cuda.synchronize()
    if rows == 0:
        return
    assert_exact(host(se).view(np.uint16), r["seg_exp"], "softmax exp segments")
    assert_exact(host(sr).view(np.uint16)[:rows], r["seg_recip"], "softmax recip segments")
    assert_exact(host(oq), r["q"], "softmax int8")
    assert_f32_close(host(of), r["p"], f"softmax fp32 {rows}x{cols} {dtype}")


def test_softmax_pwl_headline_shape_int8_only(oracle):
    """The launch configuration the benchmark times: 32*12*128 rows of 128, int8 output only."""
    rows, cols = 32 * 12 * 128, 128
    ot, dt = both_tables(oracle, [("exp", -16.0, 0.0, 128), ("recip", 1.0, 128.0, 128)])
    g = np.random.default_rng(5)
    a = np.rint(800 * g.standard_normal((rows, cols))).astype(np.int32)
    alpha = 6.1e-5
    r = oracle.softmax_pwl(a, alpha, ot[0], ot[1], 127.0)
    oq = torch.empty((rows, cols), dtype=torch.int8, device=DEV)
    nm.nm_softmax_pwl(dev(a), alpha, dt, 0, 1, 127.0, out_q=oq)
    assert_exact(host(oq), r["q"], "softmax int8 headline shape")


@pytest.mark.parametrize("rows,cols,dtype", [(98304 + 5, 512, "i32"), (393216 + 3, 128, "i32"), (65536 + 1, 768, "f32")])
def test_softmax_pwl_beyond_cache_sampled_rows(oracle, rows, cols, dtype):
    """Inputs of 192 MB and more take the kernel's streaming variant (several rows per trip); the
    row counts are ragged against every rows-per-trip value.  Rows are independent, so the oracle
    computes a sample of them (the first and last 70 and 1500 random ones) from the same bytes."""
    ot, dt = both_tables(oracle, [("exp", -16.0, 0.0, 128), ("recip", 1.0, float(max(64, cols)), 128)])
    g = torch.Generator(device="cpu").manual_seed(rows + cols)
    if dtype == "i32":
        xd_host = torch.randint(-3000, 3000, (rows, cols), dtype=torch.int32, generator=g)
        alpha = 3e-3
    else:
        xd_host = torch.randn((rows, cols), dtype=torch.float32, generator=g) * 3.0
        alpha = 1.0
    assert xd_host.numel() * 4 >= 192 << 20
    oq = torch.full((rows + 1, cols), 99, dtype=torch.int8, device=DEV)
    sr = torch.empty((rows,), dtype=torch.int16, device=DEV)
    nm.nm_softmax_pwl(xd_host.to(DEV), alpha, dt, 0, 1, 127.0, out_q=oq, dbg_seg_recip=sr, rows=rows, cols=cols)
    torch.cuda.synchronize()
    pick = np.unique(np.concatenate([np.arange(70), np.arange(rows - 70, rows),
                                     np.random.default_rng(1).integers(0, rows, 1500)]))
    r = oracle.softmax_pwl(np.ascontiguousarray(xd_host.numpy()[pick]), alpha, ot[0], ot[1], 127.0)
    got = oq.cpu().numpy()
    assert_exact(got[pick], r["q"], f"softmax int8, sampled rows of {rows}x{cols}")
    assert_exact(sr.cpu().numpy().view(np.uint16)[pick], r["seg_recip"], "softmax recip segments, sampled rows")
    assert np.all(got[rows] == 99)   # nothing past the last row


def test_pwl_apply_beyond_cache_sampled(oracle):
    """2^26 + 3 fp32 values (the size the benchmark times, plus a ragged tail): streaming loads, one
    32 KB span per block; the oracle evaluates a sample of positions and the whole tail."""
    ot, dt = both_tables(oracle, SPECS[:1])
    n = (1 << 26) + 3
    g = torch.Generator(device="cpu").manual_seed(11)
    x = torch.randn((n,), dtype=torch.float32, generator=g) * 3.0
    oq = torch.full((n + 13,), 99, dtype=torch.int8, device=DEV)
    nm.nm_pwl_apply(x.to(DEV), 1.0, dt, 0, 30.0, out_q=oq, n=n)
    torch.cuda.synchronize()
    pick = np.unique(np.concatenate([np.arange(9000), np.arange(n - 9000, n),
                                     np.random.default_rng(2).integers(0, n, 200000)]))
    _, q, _ = oracle.pwl_apply(np.ascontiguousarray(x.numpy()[pick]), ot[0], alpha=1.0, out_inv_scale=30.0)
    got = oq.cpu().numpy()
    assert_exact(got[pick], q, "pwl_apply int8, sampled positions of 2^26 + 3")
    assert np.all(got[n:] == 99)


# ---- LayerNorm-PWL ----------------------------------------------------------------------------

@pytest.mark.parametrize("rows,cols", [(37, 1), (37, 4), (37, 96), (101, 128), (37, 768), (9, 1000),
                                       (37, 1024), (3, 4096), (5, 3000), (0, 768)])
def test_layernorm_pwl(oracle, rows, cols):
    ot, dt = both_tables(oracle, [("rsqrt", 1e-3, 64.0, 128)])
    x = W.float_rows(rows, cols, seed=rows + cols)
    g = np.random.default_rng(cols)
    gamma = (1 + 0.1 * g.standard_normal(cols)).astype(np.float32)
    beta = (0.1 * g.standard_normal(cols)).astype(np.float32)
    oq = torch.empty((rows, cols), dtype=torch.int8, device=DEV)
    of = torch.empty((rows, cols), dtype=torch.float32, device=DEV)
    sg = torch.empty((max(rows, 1),), dtype=torch.int16, device=DEV)
    nm.nm_layernorm_pwl(dev(x), dev(gamma), dev(beta), 1e-5, dt, 0, 31.0, out_q=oq, out_f32=of,
                        dbg_seg=sg, rows=rows, cols=cols)
    torch.cuda.synchronize()
    if rows == 0:
        return
    r = oracle.layernorm_pwl(x, gamma, beta, 1e-5, ot[0], 31.0)
    assert_exact(host(sg).view(np.uint16)[:rows], r["seg"], "layernorm segments")
    assert_exact(host(oq), r["q"], "layernorm int8")
    assert_f32_close(host(of), r["y"], f"layernorm fp32 {rows}x{cols}")


@pytest.mark.parametrize("rows,cols", [(37, 96), (101, 128), (64, 768), (9, 1000), (5, 4096)])
def test_layernorm_pwl2_sqrt_then_reciprocal(oracle, rows, cols):
    """The two-table LayerNorm (square root, then reciprocal): segments of both tables, fp32 and
    int8 outputs against the oracle."""
    ot, dt = both_tables(oracle, [("sqrt", 0.0, 16.0, 128), ("recip", 0.25, 4.0, 64)])
    x = W.float_rows(rows, cols, seed=rows + cols, std=1.4)
    g = np.random.default_rng(cols)
    gamma = (1 + 0.1 * g.standard_normal(cols)).astype(np.float32)
    beta = (0.1 * g.standard_normal(cols)).astype(np.float32)
    r = oracle.layernorm_pwl2(x, gamma, beta, 1e-5, ot[0], ot[1], 31.0)
    oq = torch.empty((rows, cols), dtype=torch.int8, device=DEV)
    of = torch.empty((rows, cols), dtype=torch.float32, device=DEV)
    s1 = torch.empty(rows, dtype=torch.int16, device=DEV)
    s2 = torch.empty(rows, dtype=torch.int16, device=DEV)
    dx, dg, db = dev(x), dev(gamma), dev(beta)
    nm.nm_layernorm_pwl2(dx, dg, db, 1e-5, dt, 0, 1, 31.0, out_q=oq, out_f32=of, dbg_seg_sqrt=s1,
                         dbg_seg_recip=s2)
    assert_exact(host(s1).view(np.uint16), r["seg_sqrt"], "sqrt segments")
    assert_exact(host(s2).view(np.uint16), r["seg_recip"], "reciprocal segments")
    assert_f32_close(host(of), r["y"], f"layernorm2 fp32 {rows}x{cols}")
    assert_exact(host(oq), r["q"], "layernorm2 int8")
    assert len(np.unique(r["seg_sqrt"])) > 2


def test_layernorm_pwl_headline_shape(oracle):
    rows, cols = 4096, 768
    ot, dt = both_tables(oracle, [("rsqrt", 1e-3, 64.0, 128)])
    x = W.float_rows(rows, cols, seed=11, std=1.1)
    g = np.random.default_rng(3)
    gamma = (1 + 0.02 * g.standard_normal(cols)).astype(np.float32)
    beta = (0.02 * g.standard_normal(cols)).astype(np.float32)
    oq = torch.empty((rows, cols), dtype=torch.int8, device=DEV)
    nm.nm_layernorm_pwl(dev(x), dev(gamma), dev(beta), 1e-5, dt, 0, 30.0, out_q=oq)
    r = oracle.layernorm_pwl(x, gamma, beta, 1e-5, ot[0], 30.0)
    assert_exact(host(oq), r["q"], "layernorm int8 headline shape")


# ---- GEMM + epilogue --------------------------------------------------------------------------

GEMM_SHAPES = [(1, 1, 1), (5, 7, 3), (33, 65, 130), (64, 48, 768), (200, 136, 64), (300, 200, 200),
               (256, 384, 128), (129, 257, 80), (128, 64, 16), (7, 300, 1041)]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_accumulators_bit_exact(oracle, M, N, K):
    d = W.gemm_inputs(M, N, K, seed=M * 3 + N * 5 + K)
    r = oracle.gemm_pwl(d["A"], d["W"])
    acc = torch.empty((M, N), dtype=torch.int32, device=DEV)
    nm.nm_gemm_pwl(dev(d["A"]), dev(d["W"]), out_acc=acc)
    assert_exact(host(acc), r["acc"], f"gemm acc {M}x{N}x{K}")


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_full_epilogue(oracle, M, N, K):
    ot, dt = both_tables(oracle, [("gelu", -8.0, 8.0, 128)])
    d = W.gemm_inputs(M, N, K, seed=M + N + K, full_range=False)
    alpha = float(np.float32(6.0 / (20 * 20 * np.sqrt(K))))
    kw = dict(bias=d["bias"], alpha=alpha, resid=d["resid"], resid_scale=0.01, table=ot[0],
              out_inv_scale=25.0)
    r = oracle.gemm_pwl(d["A"], d["W"], **kw)
    oq = torch.empty((M, N), dtype=torch.int8, device=DEV)
    of = torch.empty((M, N), dtype=torch.float32, device=DEV)
    acc = torch.empty((M, N), dtype=torch.int32, device=DEV)
    seg = torch.empty((M, N), dtype=torch.int16, device=DEV)
    nm.nm_gemm_pwl(dev(d["A"]), dev(d["W"]), bias=dev(d["bias"]), alpha=alpha, resid=dev(d["resid"]),
                   resid_scale=0.01, tables=dt, table_idx=0, out_inv_scale=25.0, out_q=oq,
                   out_f32=of, out_acc=acc, dbg_seg=seg)
    assert_exact(host(acc), r["acc"], "gemm acc")
    assert_exact(host(seg).view(np.uint16), r["seg"], "gemm GELU segments")
    assert_exact(host(oq), r["q"], "gemm int8")
    assert_f32_close(host(of), r["y"], f"gemm fp32 {M}x{N}x{K}")
    assert len(np.unique(r["seg"])) > 3 or M * N < 50  # the inputs do exercise the table


@pytest.mark.parametrize("M,N,K", [(33, 65, 130), (256, 384, 128)])
def test_gemm_per_column_scales_no_table(oracle, M, N, K):
    d = W.gemm_inputs(M, N, K, seed=7)
    r = oracle.gemm_pwl(d["A"], d["W"], alpha_vec=d["alpha_vec"] * 1e-3,
                        out_inv_scale_vec=d["out_inv_scale_vec"], bias=d["bias"])
    oq = torch.empty((M, N), dtype=torch.int8, device=DEV)
    of = torch.empty((M, N), dtype=torch.float32, device=DEV)
    nm.nm_gemm_pwl(dev(d["A"]), dev(d["W"]), bias=dev(d["bias"]),
                   alpha_vec=dev((d["alpha_vec"] * 1e-3).astype(np.float32)),
                   out_inv_scale_vec=dev(d["out_inv_scale_vec"]), out_q=oq, out_f32=of)
    assert_exact(host(oq), r["q"], "gemm per-column int8")
    assert_f32_close(host(of), r["y"], "gemm per-column fp32")


@pytest.mark.parametrize("flags", [0, 1])
@pytest.mark.parametrize("M,N,K", [(256, 384, 128), (128, 1536, 256), (100, 130, 64)])
def test_gemm_int8_only_table_out_of_range(oracle, M, N, K, flags):
    """int8-only output (the specialised table epilogue) with pre-activations far outside the
    table range, with and without the input-clamp flag."""
    ot, dt = both_tables(oracle, [("gelu", -2.0, 2.0, 32)], flags=flags)
    d = W.gemm_inputs(M, N, K, seed=3 + M, full_range=False)
    alpha = float(np.float32(40.0 / (20 * 20 * np.sqrt(K))))
    r = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha, table=ot[0], out_inv_scale=9.0)
    assert (r["seg"] == 0).mean() > 0.05 and (r["seg"] == 31).mean() > 0.05
    oq = torch.empty((M, N), dtype=torch.int8, device=DEV)
    nm.nm_gemm_pwl(dev(d["A"]), dev(d["W"]), bias=dev(d["bias"]), alpha=alpha, tables=dt, table_idx=0,
                   out_inv_scale=9.0, out_q=oq)
    assert_exact(host(oq), r["q"], f"gemm int8-only, table flags {flags}")


@pytest.mark.parametrize("M,N,K,what", [
    (6400, 64, 256, "narrow 256x64 tile"), (12800, 1024, 128, "two-stage 128x128 tile, several per CU"),
    (12800, 1024, 512, "three-stage 128x128 tile, several per CU"), (640, 256, 1024, "64x128 split-k tile"),
    (4099, 200, 384, "ragged edges on the streaming tiles"), (130, 136, 65536, "largest K")])
def test_gemm_every_streaming_tile_configuration(oracle, M, N, K, what):
    """Shapes that reach each tile configuration of the streaming kernel (chosen by the host from
    M, N, K), full comparison of the int8 output with table, and of fp32 output with residual."""
    ot, dt = both_tables(oracle, [("gelu", -8.0, 8.0, 128)])
    d = W.gemm_inputs(M, N, K, seed=K + N, full_range=False)
    alpha = float(np.float32(6.0 / (20 * 20 * np.sqrt(K))))
    r = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha, table=ot[0], out_inv_scale=25.0)
    dA, dW, db, dr = dev(d["A"]), dev(d["W"]), dev(d["bias"]), dev(d["resid"])
    oq = torch.empty((M, N), dtype=torch.int8, device=DEV)
    nm.nm_gemm_pwl(dA, dW, bias=db, alpha=alpha, tables=dt, table_idx=0, out_inv_scale=25.0, out_q=oq)
    assert_exact(host(oq), r["q"], f"int8 + table: {what}")
    r2 = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha, resid=d["resid"], resid_scale=0.02)
    of = torch.empty((M, N), dtype=torch.float32, device=DEV)
    nm.nm_gemm_pwl(dA, dW, bias=db, alpha=alpha, resid=dr, resid_scale=0.02, out_f32=of)
    assert_f32_close(host(of), r2["y"], f"fp32 + residual: {what}")
    r3 = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha, resid=d["resid"], resid_scale=0.02,
                         table=ot[0], out_inv_scale=25.0)
    nm.nm_gemm_pwl(dA, dW, bias=db, alpha=alpha, resid=dr, resid_scale=0.02, tables=dt, table_idx=0,
                   out_inv_scale=25.0, out_q=oq)
    assert_exact(host(oq), r3["q"], f"int8 + residual + table: {what}")


@pytest.mark.parametrize("M,N,K,what", [
    (3900, 2992, 384, "256x192 tiles, two stages, ragged edges"), (8192, 1024, 512, "256x128 tiles"),
    (8192, 768, 512, "128x192 tiles"), (4096, 768, 512, "128x128 tiles"),
    (4000, 720, 640, "128x128 tiles, ragged edges"), (4096, 3072, 768, "256x192 tiles, one per CU")])
def test_gemm_tile_kernel_configurations(oracle, M, N, K, what):
    """Shapes that reach each configuration of the large-tile kernel (aligned operands, K a multiple
    of 128, scalar alpha): int8 output with and without the table, fp32 output with the residual."""
    ot, dt = both_tables(oracle, [("gelu", -8.0, 8.0, 128)])
    d = W.gemm_inputs(M, N, K, seed=K + N + 1, full_range=False)
    alpha = float(np.float32(6.0 / (20 * 20 * np.sqrt(K))))
    dA, dW, db, dr = dev(d["A"]), dev(d["W"]), dev(d["bias"]), dev(d["resid"])
    oq = torch.full((M, N), 77, dtype=torch.int8, device=DEV)
    r = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha, table=ot[0], out_inv_scale=25.0)
    nm.nm_gemm_pwl(dA, dW, bias=db, alpha=alpha, tables=dt, table_idx=0, out_inv_scale=25.0, out_q=oq)
    assert_exact(host(oq), r["q"], f"int8 + table: {what}")
    assert len(np.unique(r["seg"])) > 8
    r1 = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha, out_inv_scale=40.0)
    nm.nm_gemm_pwl(dA, dW, bias=db, alpha=alpha, out_inv_scale=40.0, out_q=oq)
    assert_exact(host(oq), r1["q"], f"int8: {what}")
    nm.nm_gemm_pwl(dA, dW, alpha=alpha, out_inv_scale=40.0, out_q=oq)      # no bias vector
    r1b = oracle.gemm_pwl(d["A"], d["W"], alpha=alpha, out_inv_scale=40.0)
    assert_exact(host(oq), r1b["q"], f"int8, no bias: {what}")
    r2 = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha, resid=d["resid"], resid_scale=0.02)
    of = torch.full((M, N), -3.0, dtype=torch.float32, device=DEV)
    nm.nm_gemm_pwl(dA, dW, bias=db, alpha=alpha, resid=dr, resid_scale=0.02, out_f32=of)
    assert_f32_close(host(of), r2["y"], f"fp32 + residual: {what}")


def test_gemm_extreme_operands(oracle):
    """All-(-127) x all-(+127) at the largest K of the workloads: |acc| = K * 127^2 > 2^24."""
    M, N, K = 40, 72, 3072
    A = np.full((M, K), -127, np.int8)
    Wm = np.full((N, K), 127, np.int8)
    r = oracle.gemm_pwl(A, Wm, alpha=1e-6)
    acc = torch.empty((M, N), dtype=torch.int32, device=DEV)
    of = torch.empty((M, N), dtype=torch.float32, device=DEV)
    nm.nm_gemm_pwl(dev(A), dev(Wm), alpha=1e-6, out_acc=acc, out_f32=of)
    assert_exact(host(acc), r["acc"], "extreme acc")
    assert_f32_close(host(of), r["y"], "extreme fp32")


def test_gemm_headline_ffn1_sampled(oracle):
    """FFN1 of the headline configuration (4096 x 3072 x 768) with the GELU table, in the launch
    configuration the benchmark times; 64 full output rows are checked against the oracle."""
    M, N, K = 4096, 3072, 768
    ot, dt = both_tables(oracle, [("gelu", -8.0, 8.0, 128)])
    d = W.gemm_inputs(M, N, K, seed=1, full_range=False)
    alpha = float(np.float32(1.5e-3))
    oq = torch.empty((M, N), dtype=torch.int8, device=DEV)
    nm.nm_gemm_pwl(dev(d["A"]), dev(d["W"]), bias=dev(d["bias"]), alpha=alpha, tables=dt, table_idx=0,
                   out_inv_scale=20.0, out_q=oq)
    rows = np.random.default_rng(0).choice(M, 64, replace=False)
    r = oracle.gemm_pwl(d["A"][rows], d["W"], bias=d["bias"], alpha=alpha, table=ot[0], out_inv_scale=20.0)
    assert_exact(host(oq)[rows], r["q"], "FFN1 sampled rows")


@pytest.mark.parametrize("M,N,K,split,what", [
    (8192, 3072, 768, 0, "two rounds of tiles"), (8192, 2304, 768, 768, "QKV: one scale per column third, 1.5 rounds"),
    (16384, 4096, 1024, 0, "5.5 rounds, last column tile partly outside"),
    (7977, 3000 + 8, 768, 0, "ragged rows and columns"), (768, 8 * 192 * 16 + 16, 1024, 0, "three tile rows, a tile count that is no multiple of 8")])
def test_gemm_more_tiles_than_compute_units_sampled(oracle, M, N, K, split, what):
    """The QKV / FFN1 shapes of the 512-token workloads (several rounds of 256 x 192 tiles over the
    256 compute units; XCD-aware tile order with and without a tile count that divides by 8): int8
    output with the table, and without it (with one inverse scale per column third where given).  The
    oracle computes 96 sampled rows, among them the first and last of the matrix and rows around tile
    edges."""
    ot, dt = both_tables(oracle, [("gelu", -8.0, 8.0, 128)])
    d = W.gemm_inputs(M, N, K, seed=M + N + K, full_range=False)
    alpha = float(np.float32(6.0 / (20 * 20 * np.sqrt(K))))
    dA, dW, db = dev(d["A"]), dev(d["W"]), dev(d["bias"])
    g = np.random.default_rng(M)
    edge = [r for r in (0, 1, 31, 32, 63, 64, 255, 256, 257, 511, 512, M - 257, M - 256, M - 65, M - 2, M - 1) if 0 <= r < M]
    rows = np.unique(np.concatenate([np.array(edge), g.choice(M, 96 - len(edge), replace=False)]))
    A_s = np.ascontiguousarray(d["A"][rows])
    oq = torch.full((M + 1, N), 77, dtype=torch.int8, device=DEV)
    nm.nm_gemm_pwl(dA, dW, bias=db, alpha=alpha, tables=dt, table_idx=0, out_inv_scale=25.0, out_q=oq, M=M)
    r = oracle.gemm_pwl(A_s, d["W"], bias=d["bias"], alpha=alpha, table=ot[0], out_inv_scale=25.0)
    got = host(oq)
    assert_exact(got[rows], r["q"], f"int8 + table: {what}")
    assert np.all(got[M] == 77)
    if split:
        inv3 = (40.0, 23.0, 31.0)
        nm.nm_gemm_pwl(dA, dW, bias=db, alpha=alpha, split_cols=split, out_inv_scale3=inv3, out_q=oq, M=M)
        want = np.concatenate([oracle.gemm_pwl(A_s, d["W"][t * split:(t + 1) * split], bias=d["bias"][t * split:(t + 1) * split],
                                               alpha=alpha, out_inv_scale=inv3[t])["q"] for t in range(3)], axis=1)
    else:
        nm.nm_gemm_pwl(dA, dW, bias=db, alpha=alpha, out_inv_scale=40.0, out_q=oq, M=M)
        want = oracle.gemm_pwl(A_s, d["W"], bias=d["bias"], alpha=alpha, out_inv_scale=40.0)["q"]
    got = host(oq)
    assert_exact(got[rows], want, f"int8: {what}")
    assert np.all(got[M] == 77)


@pytest.mark.parametrize("lo,hi", [(-8.0, 8.0), (-1.0, 3.0), (-6.0, 2.5)])
def test_two_segment_table_is_decided_by_one_compare_exactly(oracle, lo, hi):
    """A table of two segments (ReLU in the CNN) is evaluated in the matrix product's epilogue with a
    compare against the smallest value of segment 1 instead of index and gather.  With zero operands the
    pre-activation of column n is bias[n] exactly, so the bias vector sweeps the neighbourhood of the
    break point float by float (and zeros, denormals, infinities, NaN); a huge output scale makes the
    int8 code tell a tiny negative from zero.  Every code equals the oracle's, which indexes the table."""
    ot, dt = both_tables(oracle, [("relu", lo, hi, 2)])
    mid = np.float32((lo + hi) / 2)
    around = [mid]
    for _ in range(300):
        around.append(np.nextafter(around[-1], np.float32(np.inf), dtype=np.float32))
    down = [mid]
    for _ in range(300):
        down.append(np.nextafter(down[-1], np.float32(-np.inf), dtype=np.float32))
    g = np.random.default_rng(3)
    special = np.array([0.0, -0.0, 1e-45, -1e-45, 1e-38, -1e-38, np.inf, -np.inf, np.nan, lo, hi, 3e38, -3e38], np.float32)
    # the index arithmetic rounds (x - lo) to the spacing of floats near (hi - lo) / 2: values within a few
    # of those spacings of the break point are where a compare against the break point itself would
    # disagree with the index, so they are swept densely
    ulp_at_half = np.float32(hi - lo) * np.float32(2.0 ** -24)
    near = (mid + ulp_at_half * np.linspace(-4.0, 4.0, 3001)).astype(np.float32)
    vals = np.concatenate([np.array(around + down, np.float32), special, near,
                           (mid + g.standard_normal(400) * 1e-6).astype(np.float32)])
    N = (vals.size + 127) // 128 * 128
    bias = np.zeros(N, np.float32)
    bias[:vals.size] = vals
    M, K = 256, 64
    A = np.zeros((M, K), np.int8)
    Wm = np.zeros((N, K), np.int8)
    for inv in (1e9, 3.0):
        r = oracle.gemm_pwl(A[:2], Wm, bias=bias, alpha=1.0, table=ot[0], out_inv_scale=inv)
        oq = torch.empty((M, N), dtype=torch.int8, device=DEV)
        nm.nm_gemm_pwl(dev(A), dev(Wm), bias=dev(bias), alpha=1.0, tables=dt, table_idx=0, out_inv_scale=inv, out_q=oq)
        got = host(oq)
        assert_exact(got[:2], r["q"], f"two-segment table [{lo}, {hi}], scale {inv}")
        assert np.all(got == got[0])
    assert len(np.unique(r["seg"])) == 2
    # the sweep does contain values left of the break point that the index puts into segment 1
    seg_of = dict(zip(bias.tolist(), r["seg"][0].tolist()))
    assert any(v < float(mid) and s == 1 for v, s in seg_of.items() if v == v)


# ---- attention products -----------------------------------------------------------------------

@pytest.mark.parametrize("B,S,H,heads", [(1, 64, 128, 2), (3, 40, 96, 3), (2, 128, 768, 12), (1, 200, 64, 1),
                                         (2, 33, 40, 5)])
def test_attention_scores_and_context(oracle, B, S, H, heads):
    g = np.random.default_rng(B + S + H)
    d = H // heads
    qkv = g.integers(-127, 128, size=(B * S, 3 * H), dtype=np.int8)
    q4 = qkv[:, :H].reshape(B, S, heads, d).astype(np.int64)
    k4 = qkv[:, H:2 * H].reshape(B, S, heads, d).astype(np.int64)
    v4 = qkv[:, 2 * H:].reshape(B, S, heads, d).astype(np.int64)
    want = np.einsum("bihc,bjhc->bhij", q4, k4)   # the oracle layer's scores equal this (CPU pin)
    sc = torch.empty((B, heads, S, S), dtype=torch.int32, device=DEV)
    nm.nm_attn_scores(dev(qkv), B, S, H, heads, sc)
    assert_exact(host(sc).astype(np.int64), want, "scores")
    p = g.integers(0, 128, size=(B, heads, S, S), dtype=np.int8)
    cacc = np.einsum("bhij,bjhc->bihc", p.astype(np.int64), v4).reshape(B * S, H)
    alpha, inv = float(np.float32(1.0 / (127 * S))), float(np.float32(3.0))
    v = (cacc.astype(np.float32) * np.float32(alpha)).astype(np.float32)
    want_ctx = np.array([oracle.requant(x, inv) for x in v.ravel()[:4096]])
    ctx = torch.empty((B * S, H), dtype=torch.int8, device=DEV)
    nm.nm_attn_context(dev(p), dev(qkv), B, S, H, heads, alpha, inv, ctx)
    assert np.abs(cacc).max() < 2 ** 24
    assert_exact(host(ctx).ravel()[:4096], want_ctx, "context (first 4096)")
    full = np.clip(np.rint((v * np.float32(inv)).astype(np.float32)), -127, 127).astype(np.int8)
    assert_exact(host(ctx), full, "context")


@pytest.mark.parametrize("B,S,heads", [(1, 64, 2), (2, 128, 12), (1, 200, 1), (2, 33, 1), (1, 256, 2), (3, 7, 2),
                                        (1, 100, 3), (1, 512, 2), (1, 300, 1), (2, 449, 1), (1, 384, 1)])
def test_fused_attention_matches_oracle_stages(oracle, B, S, heads):
    """nm_attention_pwl against scores (int64 einsum), the oracle's softmax-PWL and the oracle's
    requantisation of P V: scores, probabilities and context all bit-exact."""
    H = 64 * heads
    ot, dt = both_tables(oracle, [("exp", -16.0, 0.0, 128), ("recip", 1.0, float(max(64, S)), 128)])
    g = np.random.default_rng(B * 1000 + S)
    qkv = np.clip(np.rint(18 * g.standard_normal((B * S, 3 * H))), -127, 127).astype(np.int8)
    q4 = qkv[:, :H].reshape(B, S, heads, 64).astype(np.int64)
    k4 = qkv[:, H:2 * H].reshape(B, S, heads, 64).astype(np.int64)
    v4 = qkv[:, 2 * H:].reshape(B, S, heads, 64).astype(np.int64)
    scores = np.einsum("bihc,bjhc->bhij", q4, k4)
    alpha_s, inv_p = float(np.float32(1.2e-3)), float(np.float32(127.0))
    sm = oracle.softmax_pwl(scores.reshape(-1, S).astype(np.int32), alpha_s, ot[0], ot[1], inv_p)
    P = sm["q"].reshape(B, heads, S, S)
    cacc = np.einsum("bhij,bjhc->bihc", P.astype(np.int64), v4).reshape(B * S, H)
    assert np.abs(cacc).max() < 2 ** 24
    alpha_c, inv_c = float(np.float32(2.0e-3)), float(np.float32(1.7))
    cv = (cacc.astype(np.float32) * np.float32(alpha_c)).astype(np.float32)
    want_ctx = np.clip(np.rint((cv * np.float32(inv_c)).astype(np.float32)), -127, 127).astype(np.int8)
    ctx = torch.empty((B * S, H), dtype=torch.int8, device=DEV)
    sc = torch.empty((B, heads, S, S), dtype=torch.int32, device=DEV)
    pp = torch.empty((B, heads, S, S), dtype=torch.int8, device=DEV)
    nm.nm_attention_pwl(dev(qkv), B, S, H, heads, alpha_s, dt, 0, 1, inv_p, alpha_c, inv_c, ctx, sc, pp)
    assert_exact(host(sc).astype(np.int64), scores, "fused scores")
    assert_exact(host(pp), P, "fused probabilities")
    assert_exact(host(ctx), want_ctx, "fused context")
    assert len(np.unique(sm["seg_exp"])) > 4  # the exp table is exercised
    # without the optional outputs the context is the same
    ctx2 = torch.empty_like(ctx)
    nm.nm_attention_pwl(dev(qkv), B, S, H, heads, alpha_s, dt, 0, 1, inv_p, alpha_c, inv_c, ctx2)
    assert_exact(host(ctx2), want_ctx, "fused context, no taps")


@pytest.mark.parametrize("S", [128, 200])
def test_fused_attention_clamp_flag_exp_table(oracle, S):
    """Exp table with the input-clamp flag and scores far below the table range."""
    B, heads, H = 2, 2, 128
    ot, dt = both_tables(oracle, [("exp", -4.0, 0.0, 32), ("recip", 1.0, float(S), 64)], flags=1)
    g = np.random.default_rng(S)
    qkv = np.clip(np.rint(30 * g.standard_normal((B * S, 3 * H))), -127, 127).astype(np.int8)
    q4 = qkv[:, :H].reshape(B, S, heads, 64).astype(np.int64)
    k4 = qkv[:, H:2 * H].reshape(B, S, heads, 64).astype(np.int64)
    v4 = qkv[:, 2 * H:].reshape(B, S, heads, 64).astype(np.int64)
    scores = np.einsum("bihc,bjhc->bhij", q4, k4)
    alpha_s, inv_p = float(np.float32(1.5e-3)), float(np.float32(127.0))
    sm = oracle.softmax_pwl(scores.reshape(-1, S).astype(np.int32), alpha_s, ot[0], ot[1], inv_p)
    assert (sm["seg_exp"] == 0).mean() > 0.2
    P = sm["q"].reshape(B, heads, S, S)
    cacc = np.einsum("bhij,bjhc->bihc", P.astype(np.int64), v4).reshape(B * S, H)
    alpha_c, inv_c = float(np.float32(2.0e-3)), float(np.float32(1.7))
    cv = (cacc.astype(np.float32) * np.float32(alpha_c)).astype(np.float32)
    want_ctx = np.clip(np.rint((cv * np.float32(inv_c)).astype(np.float32)), -127, 127).astype(np.int8)
    ctx = torch.empty((B * S, H), dtype=torch.int8, device=DEV)
    pp = torch.empty((B, heads, S, S), dtype=torch.int8, device=DEV)
    nm.nm_attention_pwl(dev(qkv), B, S, H, heads, alpha_s, dt, 0, 1, inv_p, alpha_c, inv_c, ctx, None, pp)
    assert_exact(host(pp), P, "fused probabilities, clamped exp input")
    assert_exact(host(ctx), want_ctx, "fused context, clamped exp input")


def test_fused_attention_unsupported_shapes():
    dt = nm.nm_build_tables([("exp", -16.0, 0.0, 64), ("recip", 1.0, 64.0, 64)])
    x = torch.zeros((8 * 96 * 3,), dtype=torch.int8, device=DEV)
    for (B, S, H, heads) in [(1, 8, 96, 3), (1, 513, 64, 1)]:
        with pytest.raises(nm.NmError) as ei:
            nm.nm_attention_pwl(x, B, S, H, heads, 1.0, dt, 0, 1, 1.0, 1.0, 1.0, x)
        assert ei.value.status == nm.NM_ERR_UNSUPPORTED


# ---- encoder layer ----------------------------------------------------------------------------

def run_layer(oracle, name, library_tables=False, seed=0, elastic=None):
    cfg = W.config(name)
    p = W.layer_params(name, seed)
    specs = [W.table_ranges(cfg)[n] for n in ("gelu", "exp", "recip", "rsqrt")]
    if elastic is None:
        ot, dt = both_tables(oracle, specs)
        if library_tables:
            dt = nm.nm_build_tables(specs)
    else:
        ot, dt, dt_lib = elastic_tables(oracle, specs, *elastic)
        if library_tables:
            dt = dt_lib
    tb = dict(zip(("gelu", "exp", "recip", "rsqrt"), ot))
    want = oracle.encoder_layer(p, tb, p["x"])
    B, S, H, nh, F = (cfg[k] for k in ("B", "S", "H", "heads", "F"))
    M = B * S
    devw = {n: dev(p[n]) for n in nm.LAYER_PTRS}
    desc = nm.make_layer_desc(p, devw, dt)
    ws = torch.empty(nm.nm_encoder_layer_workspace(desc), dtype=torch.uint8, device=DEV)
    taps = dict(qkv=torch.empty((M, 3 * H), dtype=torch.int8, device=DEV),
                scores=torch.empty((B, nh, S, S), dtype=torch.int32, device=DEV),
                p=torch.empty((B, nh, S, S), dtype=torch.int8, device=DEV),
                ctx=torch.empty((M, H), dtype=torch.int8, device=DEV),
                attn=torch.empty((M, H), dtype=torch.float32, device=DEV),
                ln1=torch.empty((M, H), dtype=torch.int8, device=DEV),
                ffn1=torch.empty((M, F), dtype=torch.int8, device=DEV),
                ffn2=torch.empty((M, H), dtype=torch.float32, device=DEV))
    yq = torch.empty((M, H), dtype=torch.int8, device=DEV)
    yf = torch.empty((M, H), dtype=torch.float32, device=DEV)
    nm.nm_encoder_layer(desc, dev(p["x"]), yq, yf, ws, taps=taps)
    got = {k: host(v) for k, v in taps.items()}
    got["y_q"], got["y_f32"] = host(yq), host(yf)
    # a second run without taps (intermediates in the workspace) must give the same output
    yq2 = torch.empty_like(yq)
    nm.nm_encoder_layer(desc, dev(p["x"]), yq2, None, ws)
    assert_exact(host(yq2), got["y_q"], "layer output with workspace intermediates")
    return want, got


@pytest.mark.parametrize("name", ["tiny", "ragged", "long_seq", "bert_base_layer"])
def test_encoder_layer_all_stages(oracle, name):
    want, got = run_layer(oracle, name)
    for k in ("qkv", "scores", "p", "ctx", "ln1", "ffn1", "y_q"):
        assert_exact(got[k], want[k], f"{name} layer {k}")
    for k in ("attn", "ffn2", "y_f32"):
        assert_f32_close(got[k], want[k], f"{name} layer {k}")


@pytest.mark.parametrize("name", ["bert_base_s512", "bert_large_s512"])
def test_encoder_layer_s512_full_size(oracle, name):
    """The 512-token layers of the 12- and 24-layer workloads at full size (fused attention with
    wrapped row-sum accumulators): every stage exact."""
    want, got = run_layer(oracle, name)
    for k in ("qkv", "scores", "p", "ctx", "ln1", "ffn1", "y_q"):
        assert_exact(got[k], want[k], f"{name} layer {k}")
    for k in ("attn", "ffn2", "y_f32"):
        assert_f32_close(got[k], want[k], f"{name} layer {k}")


@pytest.mark.parametrize("name,n_layers", [("tiny", 3), ("ragged", 2), ("bert_base_layer", 2)])
def test_encoder_stack(oracle, name, n_layers):
    """nm_encoder_stack against the oracle's layers applied one after the other."""
    cfg = W.config(name)
    ps = W.stack_params(name, n_layers)
    specs = [W.table_ranges(cfg)[n] for n in ("gelu", "exp", "recip", "rsqrt")]
    ot, dt = both_tables(oracle, specs)
    want = oracle.encoder_stack(ps, dict(zip(("gelu", "exp", "recip", "rsqrt"), ot)), ps[0]["x"])
    keep, descs = [], []
    for p in ps:
        devw = {n: dev(p[n]) for n in nm.LAYER_PTRS}
        keep.append(devw)
        descs.append(nm.make_layer_desc(p, devw, dt))
    M, H = cfg["B"] * cfg["S"], cfg["H"]
    ws = torch.empty(nm.nm_encoder_stack_workspace(descs), dtype=torch.uint8, device=DEV)
    yq = torch.empty((M, H), dtype=torch.int8, device=DEV)
    yf = torch.empty((M, H), dtype=torch.float32, device=DEV)
    nm.nm_encoder_stack(descs, dev(ps[0]["x"]), yq, yf, ws)
    assert_exact(host(yq), want["y_q"], f"{name} x{n_layers} stack output")
    assert_f32_close(host(yf), want["y_f32"], f"{name} x{n_layers} stack fp32 output")
    # fp32 output only
    yf2 = torch.empty_like(yf)
    nm.nm_encoder_stack(descs, dev(ps[0]["x"]), None, yf2, ws)
    assert_f32_close(host(yf2), want["y_f32"], "stack, fp32 output only")
    with pytest.raises(nm.NmError) as ei:
        nm.nm_encoder_stack(descs, dev(ps[0]["x"]), yq, None, ws, ws_bytes=ws.numel() - 1)
    assert ei.value.status == nm.NM_ERR_WORKSPACE


@pytest.mark.parametrize("name,n_layers,batch", [("bert_base_s512", 12, None), ("bert_large_s512", 24, 8)])
def test_encoder_stack_full_depth(oracle, name, n_layers, batch):
    """The 12-layer and the 24-layer workloads at their full depth, every layer with weights and
    calibrated scales of its own: int8 output exact after all requantisations.  The 12-layer stack
    runs its full batch; the 24-layer one 8 of its 32 sequences (the oracle's share of the time)."""
    cfg = W.config(name)
    ps = W.stack_params(name, n_layers)
    B = cfg["B"] if batch is None else batch
    x = ps[0]["x"][: B * cfg["S"]]
    for p in ps:
        p["B"] = B
    specs = [W.table_ranges(cfg)[n] for n in ("gelu", "exp", "recip", "rsqrt")]
    ot, dt = both_tables(oracle, specs)
    want = oracle.encoder_stack(ps, dict(zip(("gelu", "exp", "recip", "rsqrt"), ot)), x)
    keep, descs = [], []
    for p in ps:
        devw = {n: dev(p[n]) for n in nm.LAYER_PTRS}
        keep.append(devw)
        descs.append(nm.make_layer_desc(p, devw, dt))
    M, H = B * cfg["S"], cfg["H"]
    ws = torch.empty(nm.nm_encoder_stack_workspace(descs), dtype=torch.uint8, device=DEV)
    yq = torch.empty((M, H), dtype=torch.int8, device=DEV)
    yf = torch.empty((M, H), dtype=torch.float32, device=DEV)
    nm.nm_encoder_stack(descs, dev(x), yq, yf, ws)
    assert_exact(host(yq), want["y_q"], f"{name} x{n_layers} stack output")
    assert_f32_close(host(yf), want["y_f32"], f"{name} x{n_layers} stack fp32 output")
    assert len(np.unique(want["y_q"])) > 100  # the stack's output is not degenerate


def run_layer_folded(oracle, cfg, p, flags):
    """The layer without taps of the fp32 tensors (so that the LayerNorms may run inside the matrix
    products' kernels); returns the oracle's and the library's ln1 / y_q / y_f32."""
    specs = [W.table_ranges(cfg)[n] for n in ("gelu", "exp", "recip", "rsqrt")]
    ot, dt = both_tables(oracle, specs)
    want = oracle.encoder_layer(p, dict(zip(("gelu", "exp", "recip", "rsqrt"), ot)), p["x"])
    M, H = cfg["B"] * cfg["S"], cfg["H"]
    devw = {n: dev(p[n]) for n in nm.LAYER_PTRS}
    desc = nm.make_layer_desc(p, devw, dt, flags=flags)
    ws = torch.empty(nm.nm_encoder_layer_workspace(desc), dtype=torch.uint8, device=DEV)
    taps = dict(ln1=torch.empty((M, H), dtype=torch.int8, device=DEV))
    yq = torch.full((M, H), 99, dtype=torch.int8, device=DEV)
    yf = torch.full((M, H), float("nan"), dtype=torch.float32, device=DEV)
    nm.nm_encoder_layer(desc, dev(p["x"]), yq, yf, ws, taps=taps)
    got = dict(ln1=host(taps["ln1"]), y_q=host(yq), y_f32=host(yf))
    yq2 = torch.full((M, H), 99, dtype=torch.int8, device=DEV)
    nm.nm_encoder_layer(desc, dev(p["x"]), yq2, None, ws)      # int8 output only
    assert_exact(host(yq2), got["y_q"], "folded LayerNorm, int8 output only")
    return want, got


@pytest.mark.parametrize("name", ["bert_base_s512", "bert_large_s512"])
def test_encoder_layer_layernorm_folded_into_gemm(oracle, name):
    """NM_LAYER_FOLD_LAYERNORM: out-projection + LayerNorm and FFN2 + LayerNorm as one kernel each
    (H = 768 and H = 1024, full-size layers): same int8 and fp32 results as the oracle."""
    cfg = W.config(name)
    want, got = run_layer_folded(oracle, cfg, W.layer_params(name, 0), nm.NM_LAYER_FOLD_LAYERNORM)
    assert_exact(got["ln1"], want["ln1"], f"{name} folded: ln1")
    assert_exact(got["y_q"], want["y_q"], f"{name} folded: y_q")
    assert_f32_close(got["y_f32"], want["y_f32"], f"{name} folded: y_f32")


@pytest.mark.parametrize("B,S,H,heads,F", [(3, 50, 768, 12, 1024), (1, 70, 1024, 16, 512)])
def test_encoder_layer_layernorm_folded_ragged_rows(oracle, B, S, H, heads, F):
    """The folded kernels on row counts that are not a multiple of their 64-row blocks."""
    cfg = dict(B=B, S=S, H=H, heads=heads, F=F, nseg=64)
    base = "bert_base_layer" if H == 768 else "bert_large_s512"
    p = W.with_scales(W.layer_tensors(cfg, 3), W.stored_scales(base, 0))
    want, got = run_layer_folded(oracle, cfg, p, nm.NM_LAYER_FOLD_LAYERNORM)
    assert_exact(got["ln1"], want["ln1"], "folded, ragged rows: ln1")
    assert_exact(got["y_q"], want["y_q"], "folded, ragged rows: y_q")
    assert_f32_close(got["y_f32"], want["y_f32"], "folded, ragged rows: y_f32")
    # the flag that forbids folding gives the same results through the two-kernel path
    want2, got2 = run_layer_folded(oracle, cfg, p, nm.NM_LAYER_NO_FOLD_LAYERNORM)
    assert_exact(got2["y_q"], got["y_q"], "two-kernel path")


def test_encoder_layer_with_library_built_tables(oracle):
    """The product path builds its own tables (host code of the library).  They may differ from
    the oracle's in the last bit, so int8 outputs are compared to within one code."""
    want, got = run_layer(oracle, "tiny", library_tables=True)
    diff = np.abs(got["y_q"].astype(int) - want["y_q"].astype(int))
    assert diff.max() <= 1 and (diff > 0).mean() < 1e-3
    assert np.allclose(got["y_f32"], want["y_f32"], rtol=1e-4, atol=1e-5)


def test_workspace_errors():
    cfg = W.config("tiny")
    p = W.layer_params("tiny", 0)
    specs = [W.table_ranges(cfg)[n] for n in ("gelu", "exp", "recip", "rsqrt")]
    dt = nm.nm_build_tables(specs)
    devw = {n: dev(p[n]) for n in nm.LAYER_PTRS}
    desc = nm.make_layer_desc(p, devw, dt)
    need = nm.nm_encoder_layer_workspace(desc)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    yq = torch.empty((64, 128), dtype=torch.int8, device=DEV)
    with pytest.raises(nm.NmError) as ei:
        nm.nm_encoder_layer(desc, dev(p["x"]), yq, None, ws, ws_bytes=need - 1)
    assert ei.value.status == nm.NM_ERR_WORKSPACE
    with pytest.raises(nm.NmError) as ei:
        nm.nm_encoder_layer(desc, dev(p["x"]), yq, None, ws[1:], ws_bytes=need)
    assert ei.value.status == nm.NM_ERR_WORKSPACE
    d2, k, b, inv_w = nm.nm_tables_get(dt, 1)
    assert d2.nseg == specs[1][3] and k.shape == (specs[1][3],) and nm.nm_tables_count(dt) == 4


def test_gemm_misaligned_pointers(oracle):
    """Operands and outputs that start one byte / one element off an aligned address: the generic
    kernel with scalar accesses must give the same result as the aligned fast path."""
    M, N, K = 70, 132, 192
    d = W.gemm_inputs(M, N, K, seed=5, full_range=False)
    ot, dt = both_tables(oracle, [("gelu", -8.0, 8.0, 64)])
    alpha = float(np.float32(6.0 / (20 * 20 * np.sqrt(K))))
    r = oracle.gemm_pwl(d["A"], d["W"], bias=d["bias"], alpha=alpha, resid=d["resid"], resid_scale=0.02,
                        table=ot[0], out_inv_scale=25.0)

    def off(a, dtype):
        raw = torch.zeros(a.size + 8, dtype=dtype, device=DEV)
        raw[1:1 + a.size] = dev(a).view(-1)
        return raw, raw[1:1 + a.size].view(*a.shape)

    keepA, dA = off(d["A"], torch.int8)
    keepW, dW = off(d["W"], torch.int8)
    keepb, db = off(d["bias"], torch.float32)
    keepr, dr = off(d["resid"], torch.int8)
    rawq = torch.zeros(M * N + 8, dtype=torch.int8, device=DEV)
    rawf = torch.zeros(M * N + 8, dtype=torch.float32, device=DEV)
    oq, of = rawq[3:3 + M * N].view(M, N), rawf[1:1 + M * N].view(M, N)
    nm.nm_gemm_pwl(dA, dW, bias=db, alpha=alpha, resid=dr, resid_scale=0.02, tables=dt, table_idx=0,
                   out_inv_scale=25.0, out_q=oq, out_f32=of)
    assert_exact(host(oq), r["q"], "misaligned gemm int8")
    assert_f32_close(host(of), r["y"], "misaligned gemm fp32")
    assert int(host(rawq)[:3].any()) == 0 and int(host(rawq)[3 + M * N:].any()) == 0  # nothing written outside
