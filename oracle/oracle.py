"""ctypes access to the CPU oracle ``nm_oracle.c`` (test infrastructure only).

Every function here only marshals numpy arrays into the C oracle; the arithmetic lives in the C
file, next to the citations of the paper passages it follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nm_oracle.c")
_LIB = os.path.join(_HERE, "libnm_oracle.so")

F_GELU, F_EXP, F_RECIP, F_RSQRT, F_RELU, F_SQRT, F_IDENTITY = range(7)
FLAG_CLAMP_INPUT = 1
FLAG_BIAS_CORRECT = 2
DT_I32, DT_F32 = 0, 1

FN = C.CFUNCTYPE(C.c_double, C.c_double)


class CTable(C.Structure):
    _fields_ = [("lo", C.c_float), ("hi", C.c_float), ("inv_w", C.c_float), ("nseg", C.c_int32),
                ("flags", C.c_int32), ("k", C.c_void_p), ("b", C.c_void_p)]


class CGemm(C.Structure):
    _fields_ = [("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32), ("A", C.c_void_p),
                ("W", C.c_void_p), ("bias", C.c_void_p), ("alpha_vec", C.c_void_p),
                ("alpha", C.c_float), ("resid", C.c_void_p), ("resid_scale", C.c_float),
                ("table", C.POINTER(CTable)), ("out_inv_scale", C.c_float),
                ("out_inv_scale_vec", C.c_void_p), ("out_q", C.c_void_p), ("out_f32", C.c_void_p),
                ("out_acc", C.c_void_p), ("dbg_seg", C.c_void_p)]


class CConv(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "H", "W", "Cin", "Cout", "kh", "kw", "stride", "pad")] + [
        ("x", C.c_void_p), ("w", C.c_void_p), ("bias", C.c_void_p), ("alpha_vec", C.c_void_p),
        ("alpha", C.c_float), ("resid", C.c_void_p), ("resid_scale", C.c_float),
        ("table", C.POINTER(CTable)), ("out_inv_scale", C.c_float), ("out_q", C.c_void_p),
        ("out_f32", C.c_void_p), ("out_acc", C.c_void_p)]


_LAYER_FLOATS = ["alpha_qkv", "inv_s_q", "inv_s_k", "inv_s_v", "alpha_scores", "inv_s_p",
                 "alpha_ctx", "inv_s_ctx", "alpha_o", "resid1_scale", "inv_s_ln1", "alpha_1",
                 "inv_s_ffn1", "alpha_2", "resid2_scale", "inv_s_out"]


class CLayer(C.Structure):
    _fields_ = ([("B", C.c_int32), ("S", C.c_int32), ("H", C.c_int32), ("heads", C.c_int32),
                 ("F", C.c_int32)] +
                [(n, C.c_void_p) for n in ("Wqkv", "bqkv", "Wo", "bo", "W1", "b1", "W2", "b2",
                                           "gamma1", "beta1", "gamma2", "beta2")] +
                [("eps1", C.c_float), ("eps2", C.c_float)] +
                [(n, C.c_float) for n in _LAYER_FLOATS] +
                [(n, C.POINTER(CTable)) for n in ("t_gelu", "t_exp", "t_recip", "t_rsqrt")])


class CTaps(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("qkv", "scores", "p", "ctx", "attn", "ln1", "ffn1",
                                          "ffn2")]


_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (contraction off, OpenMP over rows).  Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra",
               "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> C.CDLL:
    global _lib
    with _lock:
        if _lib is None:
            L = C.CDLL(build())
            L.nmo_eval_fn.restype = C.c_double
            L.nmo_eval_fn.argtypes = [C.c_int32, C.c_double]
            L.nmo_table_build.argtypes = [C.c_int32, C.c_float, C.c_float, C.c_int32, C.c_int32,
                                          C.c_double, C.c_void_p, C.c_void_p, C.c_void_p]
            L.nmo_table_build_fn.argtypes = [FN, FN, C.c_float, C.c_float, C.c_int32, C.c_int32,
                                             C.c_double, C.c_void_p, C.c_void_p, C.c_void_p]
            L.nmo_size_optimize.argtypes = [FN, C.c_double, C.c_double, C.c_double, C.c_double,
                                            C.c_void_p, C.c_int32]
            L.nmo_size_optimize_builtin.argtypes = [C.c_int32, C.c_double, C.c_double, C.c_double,
                                                    C.c_double, C.c_void_p, C.c_int32]
            L.nmo_table_build_merged.argtypes = [C.c_int32, C.c_float, C.c_float, C.c_int32,
                                                 C.c_double, C.c_int32, C.c_double, C.c_void_p,
                                                 C.c_void_p, C.c_void_p, C.c_void_p]
            L.nmo_segidx.argtypes = [C.c_float, C.POINTER(CTable)]
            L.nmo_pwl_eval.restype = C.c_float
            L.nmo_pwl_eval.argtypes = [C.c_float, C.POINTER(CTable)]
            L.nmo_requant.restype = C.c_int8
            L.nmo_requant.argtypes = [C.c_float, C.c_float]
            L.nmo_pwl_apply.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_int64,
                                        C.POINTER(CTable), C.c_float, C.c_void_p, C.c_void_p,
                                        C.c_void_p]
            L.nmo_canonical_sum.restype = C.c_float
            L.nmo_canonical_sum.argtypes = [C.c_void_p, C.c_int32]
            L.nmo_canonical_sumsq.restype = C.c_float
            L.nmo_canonical_sumsq.argtypes = [C.c_void_p, C.c_int32]
            L.nmo_softmax_pwl.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_int64, C.c_int32,
                                          C.POINTER(CTable), C.POINTER(CTable), C.c_float,
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
            L.nmo_layernorm_pwl.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float,
                                            C.c_int64, C.c_int32, C.POINTER(CTable), C.c_float,
                                            C.c_void_p, C.c_void_p, C.c_void_p]
            L.nmo_layernorm_pwl2.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float,
                                             C.c_int64, C.c_int32, C.POINTER(CTable), C.POINTER(CTable),
                                             C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
            L.nmo_gemm_pwl.argtypes = [C.POINTER(CGemm)]
            L.nmo_conv2d_pwl.argtypes = [C.POINTER(CConv)]
            L.nmo_maxpool_i8.argtypes = [C.c_void_p] + [C.c_int32] * 7 + [C.c_void_p]
            L.nmo_avgpool_i8.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                         C.c_float, C.c_void_p, C.c_void_p]
            L.nmo_encoder_layer.argtypes = [C.POINTER(CLayer), C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.POINTER(CTaps)]
            L.nmo_encoder_layer_exact.argtypes = [C.POINTER(CLayer), C.c_void_p, C.c_int32,
                                                  C.c_void_p, C.c_void_p]
            _lib = L
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with status {rc}")


def _p(a):
    return None if a is None else a.ctypes.data


def _arr(a, dtype):
    if a is None:
        return None
    return np.ascontiguousarray(a, dtype=dtype)


class Table:
    """One uniform PWL table (k, b per segment) owned by numpy arrays."""

    def __init__(self, lo, hi, nseg, k, b, inv_w, flags=0, func=None):
        self.lo = np.float32(lo)
        self.hi = np.float32(hi)
        self.nseg = int(nseg)
        self.k = np.ascontiguousarray(k, dtype=np.float32)
        self.b = np.ascontiguousarray(b, dtype=np.float32)
        self.inv_w = np.float32(inv_w)
        self.flags = int(flags)
        self.func = func
        self.c = CTable(float(self.lo), float(self.hi), float(self.inv_w), self.nseg,
                        self.flags & FLAG_CLAMP_INPUT, self.k.ctypes.data, self.b.ctypes.data)

    def ref(self):
        return C.byref(self.c)


def build_table(func: int, lo: float, hi: float, nseg: int, flags: int = 0,
                e_th: float = 0.0) -> Table:
    k = np.empty(nseg, np.float32)
    b = np.empty(nseg, np.float32)
    inv_w = np.empty(1, np.float32)
    _check(lib().nmo_table_build(func, lo, hi, nseg, flags, e_th, _p(k), _p(b), _p(inv_w)),
           "table_build")
    return Table(lo, hi, nseg, k, b, inv_w[0], flags, func)


def build_table_fn(f, lo: float, hi: float, nseg: int, F=None, flags: int = 0,
                   e_th: float = 0.0) -> Table:
    """Table of an arbitrary Python function f (and, optionally, its antiderivative F)."""
    k = np.empty(nseg, np.float32)
    b = np.empty(nseg, np.float32)
    inv_w = np.empty(1, np.float32)
    cf = FN(f)
    cF = FN(F) if F is not None else C.cast(None, FN)
    _check(lib().nmo_table_build_fn(cf, cF, lo, hi, nseg, flags, e_th, _p(k), _p(b), _p(inv_w)),
           "table_build_fn")
    return Table(lo, hi, nseg, k, b, inv_w[0], flags)


def build_table_merged(func: int, lo: float, hi: float, nprimary: int, dk_th: float,
                       flags: int = 0, e_th: float = 0.0):
    k = np.empty(nprimary, np.float32)
    b = np.empty(nprimary, np.float32)
    inv_w = np.empty(1, np.float32)
    nm = np.zeros(1, np.int32)
    _check(lib().nmo_table_build_merged(func, lo, hi, nprimary, dk_th, flags, e_th, _p(k), _p(b),
                                        _p(inv_w), _p(nm)), "table_build_merged")
    return Table(lo, hi, nprimary, k, b, inv_w[0], flags, func), int(nm[0])


class MergedTable:
    """A merged table in its own form: start cells (multiples of the primary length from lo) and one
    line per merged segment."""

    def __init__(self, lo, hi, nprimary, start_cell, k, b, inv_w, flags=0):
        self.lo, self.hi, self.nprimary = float(lo), float(hi), int(nprimary)
        self.start_cell = np.ascontiguousarray(start_cell, np.int32)
        self.k = np.ascontiguousarray(k, np.float32)
        self.b = np.ascontiguousarray(b, np.float32)
        self.inv_w, self.flags = np.float32(inv_w), int(flags)

    @property
    def nseg(self):
        return int(self.k.size)

    def cell_to_segment(self):
        """Merged segment of every primary cell."""
        return (np.searchsorted(self.start_cell, np.arange(self.nprimary), side="right") - 1).astype(np.uint8)

    def ref(self):
        class _S(C.Structure):
            _fields_ = [("lo", C.c_float), ("hi", C.c_float), ("inv_w", C.c_float), ("nprimary", C.c_int32),
                        ("flags", C.c_int32), ("nseg", C.c_int32), ("start_cell", C.c_void_p),
                        ("k", C.c_void_p), ("b", C.c_void_p)]
        self._struct = _S(self.lo, self.hi, float(self.inv_w), self.nprimary, self.flags & FLAG_CLAMP_INPUT, self.nseg,
                          self.start_cell.ctypes.data, self.k.ctypes.data, self.b.ctypes.data)
        return C.byref(self._struct)


def build_table_merged_direct(func: int, lo: float, hi: float, nprimary: int, dk_th: float,
                              flags: int = 0, e_th: float = 0.0) -> MergedTable:
    """Algorithm 2 + Algorithm 3 without expansion: start cells and one line per merged segment."""
    start = np.zeros(nprimary, np.int32)
    k = np.zeros(nprimary, np.float32)
    b = np.zeros(nprimary, np.float32)
    inv_w = np.zeros(1, np.float32)
    n = np.zeros(1, np.int32)
    fn = lib().nmo_table_build_merged_direct
    fn.argtypes = [C.c_int32, C.c_float, C.c_float, C.c_int32, C.c_double, C.c_int32, C.c_double,
                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    _check(fn(func, lo, hi, nprimary, dk_th, flags, e_th, _p(start), _p(k), _p(b), _p(inv_w), _p(n)),
           "table_build_merged_direct")
    m = int(n[0])
    return MergedTable(lo, hi, nprimary, start[:m].copy(), k[:m].copy(), b[:m].copy(), inv_w[0], flags)


def pwl_apply_merged(x, t: MergedTable, alpha: float = 1.0, out_inv_scale: float = 1.0):
    """Direct evaluation of a merged table.  Returns (y, q, merged segment, primary cell)."""
    x = np.ascontiguousarray(x)
    dt = DT_I32 if x.dtype == np.int32 else DT_F32
    if dt == DT_F32:
        x = x.astype(np.float32)
    n = x.size
    y = np.empty(n, np.float32)
    q = np.empty(n, np.int8)
    s = np.empty(n, np.uint16)
    c = np.empty(n, np.uint16)
    fn = lib().nmo_pwl_apply_merged
    fn.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_int64, C.c_void_p, C.c_float, C.c_void_p,
                   C.c_void_p, C.c_void_p, C.c_void_p]
    _check(fn(_p(x), dt, alpha, n, t.ref(), out_inv_scale, _p(q), _p(y), _p(s), _p(c)), "pwl_apply_merged")
    return y, q, s, c


def size_optimize(func_or_callable, r_min, r_max, dlx, dk_th):
    cap = int(round((r_max - r_min) / dlx)) + 1
    xs = np.empty(cap, np.float64)
    if callable(func_or_callable):
        n = lib().nmo_size_optimize(FN(func_or_callable), r_min, r_max, dlx, dk_th, _p(xs), cap)
    else:
        n = lib().nmo_size_optimize_builtin(func_or_callable, r_min, r_max, dlx, dk_th, _p(xs),
                                            cap)
    if n < 0:
        raise RuntimeError(f"oracle size_optimize failed with status {n}")
    return xs[:n].copy()


def eval_fn(func: int, x: float) -> float:
    return lib().nmo_eval_fn(func, x)


def segidx(x: float, t: Table) -> int:
    return lib().nmo_segidx(float(np.float32(x)), t.ref())


def pwl_eval(x: float, t: Table) -> np.float32:
    return np.float32(lib().nmo_pwl_eval(float(np.float32(x)), t.ref()))


def requant(v: float, inv_scale: float) -> int:
    return int(lib().nmo_requant(float(np.float32(v)), float(np.float32(inv_scale))))


def canonical_sum(x) -> np.float32:
    x = _arr(x, np.float32)
    return np.float32(lib().nmo_canonical_sum(_p(x), x.size))


def canonical_sumsq(x) -> np.float32:
    x = _arr(x, np.float32)
    return np.float32(lib().nmo_canonical_sumsq(_p(x), x.size))


def pwl_apply(x, t: Table, alpha=1.0, out_inv_scale=1.0):
    """Returns (y fp32, q int8, seg uint16) for a flat int32 or fp32 array."""
    x = np.ascontiguousarray(x)
    dt = DT_I32 if x.dtype == np.int32 else DT_F32
    if dt == DT_F32:
        x = x.astype(np.float32, copy=False)
    y = np.empty(x.shape, np.float32)
    q = np.empty(x.shape, np.int8)
    s = np.empty(x.shape, np.uint16)
    _check(lib().nmo_pwl_apply(_p(x), dt, alpha, x.size, t.ref(), out_inv_scale, _p(q), _p(y),
                               _p(s)), "pwl_apply")
    return y, q, s


def softmax_pwl(x, alpha, t_exp: Table, t_recip: Table, out_inv_scale):
    """x: [rows, cols] int32 or fp32.  Returns dict(p, q, seg_exp, seg_recip)."""
    x = np.ascontiguousarray(x)
    dt = DT_I32 if x.dtype == np.int32 else DT_F32
    if dt == DT_F32:
        x = x.astype(np.float32, copy=False)
    rows, cols = x.shape
    p = np.empty((rows, cols), np.float32)
    q = np.empty((rows, cols), np.int8)
    se = np.empty((rows, cols), np.uint16)
    sr = np.empty(rows, np.uint16)
    _check(lib().nmo_softmax_pwl(_p(x), dt, alpha, rows, cols, t_exp.ref(), t_recip.ref(),
                                 out_inv_scale, _p(q), _p(p), _p(se), _p(sr)), "softmax_pwl")
    return dict(p=p, q=q, seg_exp=se, seg_recip=sr)


def layernorm_pwl(x, gamma, beta, eps, t_rsqrt: Table, out_inv_scale):
    x = _arr(x, np.float32)
    gamma = _arr(gamma, np.float32)
    beta = _arr(beta, np.float32)
    rows, cols = x.shape
    y = np.empty((rows, cols), np.float32)
    q = np.empty((rows, cols), np.int8)
    s = np.empty(rows, np.uint16)
    _check(lib().nmo_layernorm_pwl(_p(x), _p(gamma), _p(beta), eps, rows, cols, t_rsqrt.ref(),
                                   out_inv_scale, _p(q), _p(y), _p(s)), "layernorm_pwl")
    return dict(y=y, q=q, seg=s)


def layernorm_pwl2(x, gamma, beta, eps, t_sqrt: Table, t_recip: Table, out_inv_scale):
    """LayerNorm with a square-root table followed by a reciprocal table."""
    x = _arr(x, np.float32)
    gamma = _arr(gamma, np.float32)
    beta = _arr(beta, np.float32)
    rows, cols = x.shape
    y = np.empty((rows, cols), np.float32)
    q = np.empty((rows, cols), np.int8)
    s1 = np.empty(rows, np.uint16)
    s2 = np.empty(rows, np.uint16)
    _check(lib().nmo_layernorm_pwl2(_p(x), _p(gamma), _p(beta), eps, rows, cols, t_sqrt.ref(), t_recip.ref(),
                                    out_inv_scale, _p(q), _p(y), _p(s1), _p(s2)), "layernorm_pwl2")
    return dict(y=y, q=q, seg_sqrt=s1, seg_recip=s2)


def gemm_pwl(A, W, bias=None, alpha=1.0, alpha_vec=None, resid=None, resid_scale=0.0,
             table: Table | None = None, out_inv_scale=1.0, out_inv_scale_vec=None):
    """A [M,K] int8, W [N,K] int8.  Returns dict(acc, y, q, seg)."""
    A = _arr(A, np.int8)
    W = _arr(W, np.int8)
    M, K = A.shape
    N = W.shape[0]
    assert W.shape[1] == K
    bias = _arr(bias, np.float32)
    alpha_vec = _arr(alpha_vec, np.float32)
    resid = _arr(resid, np.int8)
    osv = _arr(out_inv_scale_vec, np.float32)
    acc = np.empty((M, N), np.int32)
    y = np.empty((M, N), np.float32)
    q = np.empty((M, N), np.int8)
    seg = np.zeros((M, N), np.uint16)
    g = CGemm(M, N, K, _p(A), _p(W), _p(bias), _p(alpha_vec), alpha, _p(resid), resid_scale,
              C.pointer(table.c) if table is not None else None, out_inv_scale, _p(osv), _p(q), _p(y),
              _p(acc), _p(seg))
    _check(lib().nmo_gemm_pwl(C.byref(g)), "gemm_pwl")
    return dict(acc=acc, y=y, q=q, seg=seg)


def conv_out_hw(H, W, kh, kw, stride, pad):
    return (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1


def conv2d_pwl(x, w, stride=1, pad=0, bias=None, alpha=1.0, alpha_vec=None, resid=None,
               resid_scale=0.0, table: Table | None = None, out_inv_scale=1.0, want_acc=True):
    """x [B,H,W,Cin] int8, w [Cout,kh,kw,Cin] int8.  Returns dict(acc, y, q), each [B,Ho,Wo,Cout]."""
    x = _arr(x, np.int8)
    w = _arr(w, np.int8)
    B, H, W, Cin = x.shape
    Cout, kh, kw, _ = w.shape
    assert w.shape[3] == Cin
    Ho, Wo = conv_out_hw(H, W, kh, kw, stride, pad)
    bias = _arr(bias, np.float32)
    alpha_vec = _arr(alpha_vec, np.float32)
    resid = _arr(resid, np.int8)
    acc = np.empty((B, Ho, Wo, Cout), np.int32) if want_acc else None
    y = np.empty((B, Ho, Wo, Cout), np.float32)
    q = np.empty((B, Ho, Wo, Cout), np.int8)
    g = CConv(B, H, W, Cin, Cout, kh, kw, stride, pad, _p(x), _p(w), _p(bias), _p(alpha_vec), alpha,
              _p(resid), resid_scale, C.pointer(table.c) if table is not None else None,
              out_inv_scale, _p(q), _p(y), _p(acc))
    _check(lib().nmo_conv2d_pwl(C.byref(g)), "conv2d_pwl")
    return dict(acc=acc, y=y, q=q)


def maxpool_i8(x, k=3, stride=2, pad=1):
    x = _arr(x, np.int8)
    B, H, W, Cc = x.shape
    Ho, Wo = conv_out_hw(H, W, k, k, stride, pad)
    y = np.empty((B, Ho, Wo, Cc), np.int8)
    _check(lib().nmo_maxpool_i8(_p(x), B, H, W, Cc, k, stride, pad, _p(y)), "maxpool_i8")
    return y


def avgpool_i8(x, alpha, out_inv_scale):
    """x [B, HW, C] int8 -> dict(q [B,C] int8, y [B,C] fp32)."""
    x = _arr(x, np.int8)
    B, HW, Cc = x.shape
    q = np.empty((B, Cc), np.int8)
    y = np.empty((B, Cc), np.float32)
    _check(lib().nmo_avgpool_i8(_p(x), B, HW, Cc, C.c_float(alpha), C.c_float(out_inv_scale), _p(q), _p(y)),
           "avgpool_i8")
    return dict(q=q, y=y)


def relu_table() -> Table:
    """max(x, 0) as a PWL table: two chord segments on a symmetric range are exact (k = {0, 1})."""
    return build_table(F_RELU, -8.0, 8.0, 2)


def resnet_forward(p: dict, x=None, calibrate: bool = False, keep: bool = False):
    """The residual CNN of the workload generator, operation by operation (convolutions with the
    folded batch-norm scale / bias, ReLU as a PWL table, exact int8 max pooling, linear average
    pooling, classifier as a matrix product).  ``calibrate``: instead of using p's activation
    scales, set each tensor's scale to absmax / 127 of its fp32 values as the network runs
    (Section 3.2 step 1: ranges come from running the model) and return them.
    Returns dict(logits fp32 [B, classes], tensors {name: int8} if keep, scales if calibrate)."""
    relu = relu_table()
    act = dict(x=p["s_x"]) if calibrate else p["act_scales"]
    cur = {"x": _arr(p["x"] if x is None else x, np.int8)}
    out = {}
    for op in p["graph"]:
        n = op["name"]
        src = cur[op["src"]]
        if op["op"] == "conv":
            resid = cur[op["resid"]] if op["resid"] else None
            if calibrate:
                av = (act[op["src"]] * p["s_w"][n] * p["gain"][n]).astype(np.float32)
                rs = float(np.float32(act[op["resid"]])) if op["resid"] else 0.0
            else:
                av, rs = p["alpha_vec"][n], p["resid_scale"][n]
            kw = dict(stride=op["stride"], pad=op["pad"], bias=p["bias"][n], alpha_vec=av, resid=resid,
                      resid_scale=rs, table=relu if op["relu"] else None, want_acc=False)
            if calibrate:
                y = conv2d_pwl(src, p["w"][n], out_inv_scale=1.0, **kw)["y"]
                act[op["dst"]] = float(np.abs(y).max()) / 127.0
                inv = float(np.float32(1.0 / act[op["dst"]]))
            else:
                inv = p["inv_s"][n]
            cur[op["dst"]] = conv2d_pwl(src, p["w"][n], out_inv_scale=inv, **kw)["q"]
        elif op["op"] == "maxpool":
            cur[op["dst"]] = maxpool_i8(src, op["k"], op["stride"], op["pad"])
            if calibrate:
                act[op["dst"]] = act[op["src"]]
        elif op["op"] == "avgpool":
            B = src.shape[0]
            flat = src.reshape(B, -1, op["C"])
            if calibrate:
                alpha = float(np.float32(act[op["src"]] / (op["H"] * op["H"])))
                y = avgpool_i8(flat, alpha, 1.0)["y"]
                act[op["dst"]] = float(np.abs(y).max()) / 127.0
                inv = float(np.float32(1.0 / act[op["dst"]]))
            else:
                alpha, inv = p["alpha"][n], p["inv_s"][n]
            cur[op["dst"]] = avgpool_i8(flat, alpha, inv)["q"]
        elif op["op"] == "fc":
            alpha = float(np.float32(act[op["src"]] * p["s_w"][n])) if calibrate else p["alpha"][n]
            out["logits"] = gemm_pwl(src, p["w"][n], bias=p["bias"][n], alpha=alpha)["y"]
        if not keep and op["op"] != "fc":  # drop tensors nothing reads any more
            live = {o["src"] for o in p["graph"][p["graph"].index(op) + 1:]} | \
                   {o.get("resid") for o in p["graph"][p["graph"].index(op) + 1:]}
            for k in [k for k in cur if k not in live]:
                del cur[k]
    if keep:
        out["tensors"] = cur
    if calibrate:
        out["scales"] = act
    return out


def _make_layer(p: dict, tables: dict):
    """p: the layer parameter dict produced by the workload generator (numpy arrays + floats).
    Returns (CLayer, keepalive list)."""
    keep = []

    def ptr(name, dtype):
        a = _arr(p[name], dtype)
        keep.append(a)
        return a.ctypes.data

    L = CLayer()
    L.B, L.S, L.H, L.heads, L.F = (int(p[k]) for k in ("B", "S", "H", "heads", "F"))
    for n in ("Wqkv", "Wo", "W1", "W2"):
        setattr(L, n, ptr(n, np.int8))
    for n in ("bqkv", "bo", "b1", "b2", "gamma1", "beta1", "gamma2", "beta2"):
        setattr(L, n, ptr(n, np.float32))
    L.eps1 = float(p["eps1"])
    L.eps2 = float(p["eps2"])
    for n in _LAYER_FLOATS:
        setattr(L, n, float(np.float32(p[n])))
    for n in ("gelu", "exp", "recip", "rsqrt"):
        t = tables[n]
        keep.append(t)
        setattr(L, "t_" + n, C.pointer(t.c))
    return L, keep


def encoder_layer(p: dict, tables: dict, x, want_taps: bool = True):
    """PWL int8 encoder layer.  Returns dict with y_q, y_f32 and (optionally) every intermediate."""
    L, keep = _make_layer(p, tables)
    x = _arr(x, np.int8)
    B, S, H, nh, F = L.B, L.S, L.H, L.heads, L.F
    M = B * S
    out = dict(y_q=np.empty((M, H), np.int8), y_f32=np.empty((M, H), np.float32))
    taps = CTaps()
    if want_taps:
        out.update(qkv=np.empty((M, 3 * H), np.int8), scores=np.empty((B, nh, S, S), np.int32),
                   p=np.empty((B, nh, S, S), np.int8), ctx=np.empty((M, H), np.int8),
                   attn=np.empty((M, H), np.float32), ln1=np.empty((M, H), np.int8),
                   ffn1=np.empty((M, F), np.int8), ffn2=np.empty((M, H), np.float32))
        for n in ("qkv", "scores", "p", "ctx", "attn", "ln1", "ffn1", "ffn2"):
            setattr(taps, n, out[n].ctypes.data)
    _check(lib().nmo_encoder_layer(C.byref(L), _p(x), _p(out["y_q"]), _p(out["y_f32"]),
                                   C.byref(taps)), "encoder_layer")
    del keep
    return out


def encoder_stack(params: list, tables: dict, x):
    """Layers applied one after the other: layer l reads the int8 output of layer l-1 (the paper's
    Section 4 models are stacks of identical encoder layers).  Returns the last layer's outputs."""
    out = None
    for p in params:
        out = encoder_layer(p, tables, x, want_taps=False)
        x = out["y_q"]
    return out


ABSMAX_NAMES = ("x", "q", "k", "v", "p", "ctx", "ln1", "ffn1", "out", "gelu_in_min", "gelu_in_max",
                "softmax_den_max", "var_eps_max")


def encoder_layer_exact(p: dict, tables: dict, x, quantise: bool):
    """binary64 true-function layer.  Returns (y [M,H] float64, dict of observed ranges)."""
    L, keep = _make_layer(p, tables)
    x = _arr(x, np.int8)
    M = L.B * L.S
    y = np.empty((M, L.H), np.float64)
    am = np.zeros(13, np.float64)
    _check(lib().nmo_encoder_layer_exact(C.byref(L), _p(x), 1 if quantise else 0, _p(y), _p(am)),
           "encoder_layer_exact")
    del keep
    return y, dict(zip(ABSMAX_NAMES, am.tolist()))
