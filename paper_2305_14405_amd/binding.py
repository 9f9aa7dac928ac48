"""Thin ctypes binding of the C ABI in ``include/nm.h``: argument marshalling only.

Functions carry the names of the C entry points.  Tensors are ``torch`` device tensors (PyTorch is
used for device memory and streams only); every step of the computation runs in the HIP library.
There is no fallback: if ``libnm_hip.so`` is missing the import of the library fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libnm_hip.so")

NM_OK = 0
NM_ERR_INVALID_ARG, NM_ERR_UNSUPPORTED, NM_ERR_ALLOC, NM_ERR_HIP, NM_ERR_WORKSPACE = -1, -2, -3, -4, -5
FUNC = {"gelu": 0, "exp": 1, "recip": 2, "rsqrt": 3, "relu": 4, "sqrt": 5, "identity": 6}
NM_TABLE_CLAMP_INPUT, NM_TABLE_BIAS_CORRECT, NM_TABLE_MERGE, NM_TABLE_COMPACT = 1, 2, 4, 8
NM_DT_I32, NM_DT_F32 = 0, 1

# every symbol include/nm.h declares
EXPORTS = ("nm_last_error", "nm_version", "nm_table_build_host", "nm_build_tables",
           "nm_tables_from_arrays", "nm_tables_count", "nm_tables_get", "nm_tables_get_compact", "nm_tables_destroy",
           "nm_gemm_pwl", "nm_softmax_pwl", "nm_layernorm_pwl", "nm_layernorm_pwl2", "nm_pwl_apply", "nm_attn_scores",
           "nm_attn_context", "nm_attention_pwl", "nm_encoder_layer_workspace", "nm_encoder_layer",
           "nm_encoder_layer_noalloc",
           "nm_encoder_stack_workspace", "nm_encoder_stack", "nm_conv2d_workspace", "nm_conv2d_pwl",
           "nm_maxpool_i8", "nm_avgpool_i8", "nm_cnn_workspace", "nm_cnn_run")
NM_OP_CONV, NM_OP_MAXPOOL, NM_OP_AVGPOOL, NM_OP_GEMM = 0, 1, 2, 3
NM_LAYER_FOLD_LAYERNORM, NM_LAYER_NO_FOLD_LAYERNORM = 1, 2
NM_NOALLOC_MAX_WORKSPACE = 64 << 20  # bytes of the buffer built into the library (nm_encoder_layer_noalloc)


class NmError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"nm status {status}: {message}")
        self.status = status


class TableDesc(C.Structure):
    _fields_ = [("func", C.c_int32), ("lo", C.c_float), ("hi", C.c_float), ("nseg", C.c_int32),
                ("flags", C.c_int32), ("e_th", C.c_float), ("dk_th", C.c_float)]


class GemmDesc(C.Structure):
    _fields_ = [("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32), ("A", C.c_void_p),
                ("W", C.c_void_p), ("bias", C.c_void_p), ("alpha_vec", C.c_void_p),
                ("alpha", C.c_float), ("resid", C.c_void_p), ("resid_scale", C.c_float),
                ("tables", C.c_void_p), ("table_idx", C.c_int32), ("out_inv_scale", C.c_float),
                ("out_inv_scale_vec", C.c_void_p), ("out_q", C.c_void_p), ("out_f32", C.c_void_p),
                ("out_acc", C.c_void_p), ("dbg_seg", C.c_void_p), ("split_cols", C.c_int32),
                ("out_inv_scale3", C.c_float * 3)]


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "H", "W", "Cin", "Cout", "kh", "kw", "stride", "pad")] + [
        ("x", C.c_void_p), ("w", C.c_void_p), ("bias", C.c_void_p), ("alpha_vec", C.c_void_p),
        ("alpha", C.c_float), ("resid", C.c_void_p), ("resid_scale", C.c_float),
        ("tables", C.c_void_p), ("table_idx", C.c_int32), ("out_inv_scale", C.c_float),
        ("out_q", C.c_void_p), ("out_f32", C.c_void_p), ("dbg_acc", C.c_void_p)]


class CnnOp(C.Structure):
    _fields_ = [("kind", C.c_int32), ("conv", ConvDesc), ("gemm", GemmDesc), ("x", C.c_void_p),
                ("y", C.c_void_p), ("y_f32", C.c_void_p)] + \
               [(n, C.c_int32) for n in ("B", "H", "W", "C", "k", "stride", "pad")] + \
               [("alpha", C.c_float), ("out_inv_scale", C.c_float)]


LAYER_FLOATS = ("alpha_qkv", "inv_s_q", "inv_s_k", "inv_s_v", "alpha_scores", "inv_s_p",
                "alpha_ctx", "inv_s_ctx", "alpha_o", "resid1_scale", "inv_s_ln1", "alpha_1",
                "inv_s_ffn1", "alpha_2", "resid2_scale", "inv_s_out")
LAYER_PTRS = ("Wqkv", "bqkv", "Wo", "bo", "W1", "b1", "W2", "b2", "gamma1", "beta1", "gamma2",
              "beta2")
TAP_NAMES = ("qkv", "scores", "p", "ctx", "attn", "ln1", "ffn1", "ffn2")


class LayerDesc(C.Structure):
    _fields_ = ([(n, C.c_int32) for n in ("B", "S", "H", "heads", "F")] +
                [(n, C.c_void_p) for n in LAYER_PTRS] +
                [("eps1", C.c_float), ("eps2", C.c_float)] +
                [(n, C.c_float) for n in LAYER_FLOATS] +
                [("tables", C.c_void_p)] +
                [(n, C.c_int32) for n in ("gelu_idx", "exp_idx", "recip_idx", "rsqrt_idx", "flags")])


class LayerTaps(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in TAP_NAMES]


_lib = None


def load(preload_torch: bool = True) -> C.CDLL:
    """Load libnm_hip.so.  torch is imported first so that the process uses one HIP runtime."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with "
                          "`python -m paper_2305_14405_amd.build` (there is no CPU fallback)")
    # torch bundles its own HIP runtime; it must be in the process before this library is, so that
    # both resolve to the same runtime (device pointers and streams are shared between them)
    del preload_torch
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = C.CDLL(LIB_PATH)
    L.nm_last_error.restype = C.c_char_p
    L.nm_table_build_host.argtypes = [C.POINTER(TableDesc), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p]
    L.nm_build_tables.argtypes = [C.POINTER(TableDesc), C.c_int32, C.c_void_p,
                                  C.POINTER(C.c_void_p)]
    L.nm_tables_from_arrays.argtypes = [C.POINTER(TableDesc), C.c_int32, C.POINTER(C.c_void_p),
                                        C.POINTER(C.c_void_p), C.c_void_p, C.POINTER(C.c_void_p)]
    L.nm_tables_count.argtypes = [C.c_void_p]
    L.nm_tables_get.argtypes = [C.c_void_p, C.c_int32, C.POINTER(TableDesc), C.c_void_p,
                                C.c_void_p, C.c_void_p]
    L.nm_tables_get_compact.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.nm_tables_destroy.argtypes = [C.c_void_p]
    L.nm_tables_destroy.restype = None
    L.nm_gemm_pwl.argtypes = [C.POINTER(GemmDesc), C.c_void_p]
    L.nm_softmax_pwl.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_int64, C.c_int32,
                                 C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.nm_layernorm_pwl.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_int64,
                                   C.c_int32, C.c_void_p, C.c_int32, C.c_float, C.c_void_p,
                                   C.c_void_p, C.c_void_p, C.c_void_p]
    L.nm_layernorm_pwl2.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_int64,
                                    C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.nm_pwl_apply.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_int64, C.c_void_p, C.c_int32,
                               C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.nm_attn_scores.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                 C.c_void_p, C.c_void_p]
    L.nm_attn_context.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                  C.c_int32, C.c_float, C.c_float, C.c_void_p, C.c_void_p]
    L.nm_attention_pwl.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                   C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_float, C.c_float,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.nm_encoder_layer_workspace.argtypes = [C.POINTER(LayerDesc), C.POINTER(C.c_size_t)]
    L.nm_encoder_layer.argtypes = [C.POINTER(LayerDesc), C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_size_t, C.POINTER(LayerTaps), C.c_void_p]
    L.nm_encoder_layer_noalloc.argtypes = [C.POINTER(LayerDesc), C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_void_p]
    L.nm_conv2d_workspace.argtypes = [C.POINTER(ConvDesc), C.POINTER(C.c_size_t)]
    L.nm_conv2d_pwl.argtypes = [C.POINTER(ConvDesc), C.c_void_p, C.c_size_t, C.c_void_p]
    L.nm_maxpool_i8.argtypes = [C.c_void_p] + [C.c_int32] * 7 + [C.c_void_p, C.c_void_p]
    L.nm_avgpool_i8.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_float,
                                C.c_void_p, C.c_void_p, C.c_void_p]
    L.nm_cnn_workspace.argtypes = [C.POINTER(CnnOp), C.c_int32, C.POINTER(C.c_size_t)]
    L.nm_cnn_run.argtypes = [C.POINTER(CnnOp), C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
    L.nm_encoder_stack_workspace.argtypes = [C.POINTER(LayerDesc), C.c_int32, C.POINTER(C.c_size_t)]
    L.nm_encoder_stack.argtypes = [C.POINTER(LayerDesc), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_size_t, C.c_void_p]
    _lib = L
    return L


def _check(rc):
    if rc != NM_OK:
        raise NmError(rc, load().nm_last_error().decode())


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / None."""
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        assert t.is_contiguous(), "tensors passed to the C ABI must be contiguous"
        return t.data_ptr()
    return t.ctypes.data


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def nm_last_error() -> str:
    return load().nm_last_error().decode()


def nm_version() -> int:
    return load().nm_version()


def _desc(spec) -> TableDesc:
    """spec: (func name or id, lo, hi, nseg[, flags[, e_th[, dk_th]]])."""
    func, lo, hi, nseg, *rest = spec
    flags = rest[0] if len(rest) > 0 else 0
    e_th = rest[1] if len(rest) > 1 else 0.0
    dk_th = rest[2] if len(rest) > 2 else 0.0
    fid = FUNC[func] if isinstance(func, str) else int(func)
    return TableDesc(fid, lo, hi, nseg, flags, e_th, dk_th)


def nm_table_build_host(spec):
    """Host-only table construction.  Returns (k, b, inv_w, n_distinct) as numpy values."""
    import numpy as np
    d = _desc(spec)
    n = max(int(d.nseg), 1)
    k = np.zeros(n, np.float32)
    b = np.zeros(n, np.float32)
    inv_w = np.zeros(1, np.float32)
    nd = np.zeros(1, np.int32)
    _check(load(preload_torch=False).nm_table_build_host(C.byref(d), k.ctypes.data, b.ctypes.data,
                                                         inv_w.ctypes.data, nd.ctypes.data))
    return k, b, inv_w[0], int(nd[0])


class Tables:
    """Owner of an nm_tables object."""

    def __init__(self, handle, n):
        self.handle = handle
        self.n = n

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.nm_tables_destroy(self.handle)
            self.handle = None


def nm_build_tables(specs, stream=None) -> Tables:
    arr = (TableDesc * len(specs))(*[_desc(s) for s in specs])
    out = C.c_void_p()
    _check(load().nm_build_tables(arr, len(specs), _stream(stream), C.byref(out)))
    return Tables(out.value, len(specs))


def nm_tables_from_arrays(specs, ks, bs, stream=None) -> Tables:
    import numpy as np
    arr = (TableDesc * len(specs))(*[_desc(s) for s in specs])
    ks = [np.ascontiguousarray(k, np.float32) for k in ks]
    bs = [np.ascontiguousarray(b, np.float32) for b in bs]
    kp = (C.c_void_p * len(specs))(*[k.ctypes.data for k in ks])
    bp = (C.c_void_p * len(specs))(*[b.ctypes.data for b in bs])
    out = C.c_void_p()
    _check(load().nm_tables_from_arrays(arr, len(specs), kp, bp, _stream(stream), C.byref(out)))
    return Tables(out.value, len(specs))


def nm_tables_count(t: Tables) -> int:
    return load().nm_tables_count(t.handle if t else None)


def nm_tables_get(t: Tables, idx: int):
    import numpy as np
    d = TableDesc()
    _check(load().nm_tables_get(t.handle, idx, C.byref(d), None, None, None))
    k = np.zeros(d.nseg, np.float32)
    b = np.zeros(d.nseg, np.float32)
    inv_w = np.zeros(1, np.float32)
    _check(load().nm_tables_get(t.handle, idx, None, k.ctypes.data, b.ctypes.data,
                                inv_w.ctypes.data))
    return d, k, b, inv_w[0]


def nm_tables_get_compact(t: Tables, idx: int):
    """Two-level form of a table built with NM_TABLE_COMPACT: (cell_to_segment uint8 [nseg], k, b)."""
    import numpy as np
    d = TableDesc()
    _check(load().nm_tables_get(t.handle, idx, C.byref(d), None, None, None))
    n = C.c_int32()
    _check(load().nm_tables_get_compact(t.handle, idx, C.byref(n), None, None, None))
    cmap = np.zeros(d.nseg, np.uint8)
    k = np.zeros(n.value, np.float32)
    b = np.zeros(n.value, np.float32)
    _check(load().nm_tables_get_compact(t.handle, idx, None, cmap.ctypes.data, k.ctypes.data, b.ctypes.data))
    return cmap, k, b


def nm_gemm_pwl(A, W, *, bias=None, alpha=1.0, alpha_vec=None, resid=None, resid_scale=0.0,
                tables: Tables | None = None, table_idx=-1, out_inv_scale=1.0,
                out_inv_scale_vec=None, out_q=None, out_f32=None, out_acc=None, dbg_seg=None,
                stream=None, M=None, N=None, K=None, split_cols=0, out_inv_scale3=None):
    d = GemmDesc()
    d.M = A.shape[0] if M is None else M
    d.K = A.shape[1] if K is None else K
    d.N = W.shape[0] if N is None else N
    d.A, d.W, d.bias, d.alpha_vec = _ptr(A), _ptr(W), _ptr(bias), _ptr(alpha_vec)
    d.alpha = alpha
    d.resid, d.resid_scale = _ptr(resid), resid_scale
    d.tables = tables.handle if tables is not None else None
    d.table_idx = table_idx
    d.out_inv_scale = out_inv_scale
    d.out_inv_scale_vec = _ptr(out_inv_scale_vec)
    d.out_q, d.out_f32, d.out_acc, d.dbg_seg = _ptr(out_q), _ptr(out_f32), _ptr(out_acc), _ptr(dbg_seg)
    d.split_cols = split_cols
    if out_inv_scale3 is not None:
        d.out_inv_scale3 = (C.c_float * 3)(*[float(v) for v in out_inv_scale3])
    _check(load().nm_gemm_pwl(C.byref(d), _stream(stream)))


def nm_softmax_pwl(x, alpha, tables: Tables, exp_idx, recip_idx, out_inv_scale, *, out_q=None,
                   out_f32=None, dbg_seg_exp=None, dbg_seg_recip=None, stream=None, rows=None,
                   cols=None):
    import torch
    dt = NM_DT_I32 if x.dtype == torch.int32 else NM_DT_F32
    rows = x.shape[0] if rows is None else rows
    cols = x.shape[1] if cols is None else cols
    _check(load().nm_softmax_pwl(_ptr(x), dt, alpha, rows, cols, tables.handle, exp_idx, recip_idx,
                                 out_inv_scale, _ptr(out_q), _ptr(out_f32), _ptr(dbg_seg_exp),
                                 _ptr(dbg_seg_recip), _stream(stream)))


def nm_layernorm_pwl(x, gamma, beta, eps, tables: Tables, rsqrt_idx, out_inv_scale, *, out_q=None,
                     out_f32=None, dbg_seg=None, stream=None, rows=None, cols=None):
    rows = x.shape[0] if rows is None else rows
    cols = x.shape[1] if cols is None else cols
    _check(load().nm_layernorm_pwl(_ptr(x), _ptr(gamma), _ptr(beta), eps, rows, cols,
                                   tables.handle, rsqrt_idx, out_inv_scale, _ptr(out_q),
                                   _ptr(out_f32), _ptr(dbg_seg), _stream(stream)))


def nm_layernorm_pwl2(x, gamma, beta, eps, tables: Tables, sqrt_idx, recip_idx, out_inv_scale, *,
                      out_q=None, out_f32=None, dbg_seg_sqrt=None, dbg_seg_recip=None, stream=None):
    rows, cols = x.shape
    _check(load().nm_layernorm_pwl2(_ptr(x), _ptr(gamma), _ptr(beta), eps, rows, cols, tables.handle,
                                    sqrt_idx, recip_idx, out_inv_scale, _ptr(out_q), _ptr(out_f32),
                                    _ptr(dbg_seg_sqrt), _ptr(dbg_seg_recip), _stream(stream)))


def nm_pwl_apply(x, alpha, tables: Tables, idx, out_inv_scale, *, out_q=None, out_f32=None,
                 dbg_seg=None, stream=None, n=None):
    import torch
    dt = NM_DT_I32 if x.dtype == torch.int32 else NM_DT_F32
    n = x.numel() if n is None else n
    _check(load().nm_pwl_apply(_ptr(x), dt, alpha, n, tables.handle, idx, out_inv_scale,
                               _ptr(out_q), _ptr(out_f32), _ptr(dbg_seg), _stream(stream)))


def nm_attn_scores(qkv, B, S, H, heads, scores, stream=None):
    _check(load().nm_attn_scores(_ptr(qkv), B, S, H, heads, _ptr(scores), _stream(stream)))


def nm_attn_context(p, qkv, B, S, H, heads, alpha, out_inv_scale, ctx, stream=None):
    _check(load().nm_attn_context(_ptr(p), _ptr(qkv), B, S, H, heads, alpha, out_inv_scale,
                                  _ptr(ctx), _stream(stream)))


def nm_attention_pwl(qkv, B, S, H, heads, alpha_scores, tables: Tables, exp_idx, recip_idx, inv_s_p,
                     alpha_ctx, inv_s_ctx, ctx, scores_out=None, p_out=None, stream=None):
    _check(load().nm_attention_pwl(_ptr(qkv), B, S, H, heads, alpha_scores, tables.handle, exp_idx,
                                   recip_idx, inv_s_p, alpha_ctx, inv_s_ctx, _ptr(ctx),
                                   _ptr(scores_out), _ptr(p_out), _stream(stream)))


def make_layer_desc(params: dict, dev: dict, tables: Tables, idx=(0, 1, 2, 3), flags=0) -> LayerDesc:
    """params: numbers (dims, eps, fp32 multipliers); dev: device tensors of the weights."""
    d = LayerDesc()
    for n in ("B", "S", "H", "heads", "F"):
        setattr(d, n, int(params[n]))
    for n in LAYER_PTRS:
        setattr(d, n, _ptr(dev[n]))
    d.eps1, d.eps2 = float(params["eps1"]), float(params["eps2"])
    for n in LAYER_FLOATS:
        setattr(d, n, float(params[n]))
    d.tables = tables.handle
    d.gelu_idx, d.exp_idx, d.recip_idx, d.rsqrt_idx = idx
    d.flags = flags
    return d


def nm_encoder_layer_workspace(desc: LayerDesc) -> int:
    n = C.c_size_t()
    _check(load().nm_encoder_layer_workspace(C.byref(desc), C.byref(n)))
    return n.value


def nm_encoder_layer(desc: LayerDesc, x, y_q, y_f32, ws, taps: dict | None = None, stream=None,
                     ws_bytes=None):
    ct = None
    if taps:
        ct = LayerTaps()
        for n in TAP_NAMES:
            setattr(ct, n, _ptr(taps.get(n)))
    nbytes = ws.numel() * ws.element_size() if ws_bytes is None else ws_bytes
    _check(load().nm_encoder_layer(C.byref(desc), _ptr(x), _ptr(y_q), _ptr(y_f32), _ptr(ws), nbytes,
                                   C.byref(ct) if ct is not None else None, _stream(stream)))


def nm_encoder_layer_noalloc(desc: LayerDesc, x, y_q, y_f32, stream=None):
    _check(load().nm_encoder_layer_noalloc(C.byref(desc), _ptr(x), _ptr(y_q), _ptr(y_f32), _stream(stream)))


def _desc_array(descs):
    arr = (LayerDesc * len(descs))()
    for i, d in enumerate(descs):
        C.memmove(C.byref(arr, i * C.sizeof(LayerDesc)), C.byref(d), C.sizeof(LayerDesc))
    return arr


def nm_encoder_stack_workspace(descs) -> int:
    n = C.c_size_t()
    _check(load().nm_encoder_stack_workspace(_desc_array(descs), len(descs), C.byref(n)))
    return n.value


def nm_encoder_stack(descs, x, y_q, y_f32, ws, stream=None, ws_bytes=None):
    nbytes = ws.numel() * ws.element_size() if ws_bytes is None else ws_bytes
    _check(load().nm_encoder_stack(_desc_array(descs), len(descs), _ptr(x), _ptr(y_q), _ptr(y_f32),
                                   _ptr(ws), nbytes, _stream(stream)))


def make_conv_desc(x, w, stride=1, pad=0, *, bias=None, alpha=1.0, alpha_vec=None, resid=None,
                   resid_scale=0.0, tables: Tables | None = None, table_idx=-1, out_inv_scale=1.0,
                   out_q=None, out_f32=None, dbg_acc=None) -> ConvDesc:
    """x [B,H,W,Cin] int8 device tensor, w [Cout,kh,kw,Cin] int8 device tensor."""
    d = ConvDesc()
    d.B, d.H, d.W, d.Cin = (int(v) for v in x.shape)
    d.Cout, d.kh, d.kw = int(w.shape[0]), int(w.shape[1]), int(w.shape[2])
    d.stride, d.pad = stride, pad
    d.x, d.w, d.bias, d.alpha_vec = _ptr(x), _ptr(w), _ptr(bias), _ptr(alpha_vec)
    d.alpha = alpha
    d.resid, d.resid_scale = _ptr(resid), resid_scale
    d.tables = tables.handle if tables is not None else None
    d.table_idx = table_idx
    d.out_inv_scale = out_inv_scale
    d.out_q, d.out_f32, d.dbg_acc = _ptr(out_q), _ptr(out_f32), _ptr(dbg_acc)
    return d


def nm_conv2d_workspace(desc: ConvDesc) -> int:
    n = C.c_size_t()
    _check(load().nm_conv2d_workspace(C.byref(desc), C.byref(n)))
    return n.value


def nm_conv2d_pwl(desc: ConvDesc, ws=None, stream=None, ws_bytes=None):
    nbytes = 0 if ws is None else (ws.numel() * ws.element_size() if ws_bytes is None else ws_bytes)
    _check(load().nm_conv2d_pwl(C.byref(desc), _ptr(ws), nbytes, _stream(stream)))


def nm_maxpool_i8(x, y, k=3, stride=2, pad=1, stream=None):
    B, H, W, Cc = (int(v) for v in x.shape)
    _check(load().nm_maxpool_i8(_ptr(x), B, H, W, Cc, k, stride, pad, _ptr(y), _stream(stream)))


def nm_avgpool_i8(x, alpha, out_inv_scale, *, out_q=None, out_f32=None, stream=None):
    """x [B, HW, C] int8 device tensor."""
    B, HW, Cc = (int(v) for v in x.shape)
    _check(load().nm_avgpool_i8(_ptr(x), B, HW, Cc, alpha, out_inv_scale, _ptr(out_q), _ptr(out_f32),
                                _stream(stream)))


def make_gemm_desc(A, W, *, bias=None, alpha=1.0, alpha_vec=None, resid=None, resid_scale=0.0,
                   tables: Tables | None = None, table_idx=-1, out_inv_scale=1.0, out_q=None, out_f32=None) -> GemmDesc:
    d = GemmDesc()
    d.M, d.K, d.N = int(A.shape[0]), int(A.shape[1]), int(W.shape[0])
    d.A, d.W, d.bias, d.alpha_vec = _ptr(A), _ptr(W), _ptr(bias), _ptr(alpha_vec)
    d.alpha = alpha
    d.resid, d.resid_scale = _ptr(resid), resid_scale
    d.tables = tables.handle if tables is not None else None
    d.table_idx = table_idx
    d.out_inv_scale = out_inv_scale
    d.out_q, d.out_f32 = _ptr(out_q), _ptr(out_f32)
    return d


def cnn_op_conv(desc: ConvDesc) -> CnnOp:
    o = CnnOp()
    o.kind, o.conv = NM_OP_CONV, desc
    return o


def cnn_op_gemm(desc: GemmDesc) -> CnnOp:
    o = CnnOp()
    o.kind, o.gemm = NM_OP_GEMM, desc
    return o


def cnn_op_maxpool(x, y, k=3, stride=2, pad=1) -> CnnOp:
    o = CnnOp()
    o.kind, o.x, o.y = NM_OP_MAXPOOL, _ptr(x), _ptr(y)
    o.B, o.H, o.W, o.C = (int(v) for v in x.shape)
    o.k, o.stride, o.pad = k, stride, pad
    return o


def cnn_op_avgpool(x, alpha, out_inv_scale, out_q=None, out_f32=None) -> CnnOp:
    """x [B, HW, C]."""
    o = CnnOp()
    o.kind, o.x, o.y, o.y_f32 = NM_OP_AVGPOOL, _ptr(x), _ptr(out_q), _ptr(out_f32)
    o.B, o.H, o.C = (int(v) for v in x.shape)
    o.alpha, o.out_inv_scale = alpha, out_inv_scale
    return o


def _op_array(ops):
    arr = (CnnOp * len(ops))()
    for i, o in enumerate(ops):
        C.memmove(C.byref(arr, i * C.sizeof(CnnOp)), C.byref(o), C.sizeof(CnnOp))
    return arr


def nm_cnn_workspace(ops) -> int:
    n = C.c_size_t()
    _check(load().nm_cnn_workspace(_op_array(ops), len(ops), C.byref(n)))
    return n.value


def nm_cnn_run(ops, ws=None, stream=None, ws_bytes=None, op_array=None):
    """ops: list of CnnOp (or pass a prebuilt ctypes array as op_array to skip the copy)."""
    arr = op_array if op_array is not None else _op_array(ops)
    nbytes = 0 if ws is None else (ws.numel() * ws.element_size() if ws_bytes is None else ws_bytes)
    _check(load().nm_cnn_run(arr, len(arr), _ptr(ws), nbytes, _stream(stream)))
