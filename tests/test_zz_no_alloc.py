"""The entry point that allocates nothing (nm_encoder_layer_noalloc) against the entry point it is a
variant of (nm_encoder_layer with a caller-owned workspace): int8 output bit-exact, fp32 output
within 1e-5 relative, on two calls in a row, the second with a smaller input that leaves the first
call's data in most of the built-in buffer."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2305_14405_amd import binding as nm
import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _layer(name):
    cfg = W.config(name)
    p = W.layer_params(name, 0)
    specs = [W.table_ranges(cfg)[n] for n in ("gelu", "exp", "recip", "rsqrt")]
    tables = nm.nm_build_tables(specs)
    devw = {n: torch.from_numpy(np.ascontiguousarray(p[n])).to(DEV) for n in nm.LAYER_PTRS}
    desc = nm.make_layer_desc(p, devw, tables)
    x = torch.from_numpy(p["x"]).to(DEV)
    M, H = cfg["B"] * cfg["S"], cfg["H"]
    return desc, x, M, H, (tables, devw)


def _both(name):
    desc, x, M, H, keep = _layer(name)
    ws = torch.empty(nm.nm_encoder_layer_workspace(desc), dtype=torch.uint8, device=DEV)
    want_q = torch.empty((M, H), dtype=torch.int8, device=DEV)
    want_f = torch.empty((M, H), dtype=torch.float32, device=DEV)
    nm.nm_encoder_layer(desc, x, want_q, want_f, ws)
    got_q = torch.full((M, H), 99, dtype=torch.int8, device=DEV)
    got_f = torch.full((M, H), float("nan"), dtype=torch.float32, device=DEV)
    nm.nm_encoder_layer_noalloc(desc, x, got_q, got_f)
    torch.cuda.synchronize()
    wq, gq = want_q.cpu().numpy(), got_q.cpu().numpy()
    wf, gf = want_f.cpu().numpy(), got_f.cpu().numpy()
    assert np.array_equal(gq, wq), f"{name}: {int((gq != wq).sum())} int8 codes differ"
    assert np.all(np.abs(gf - wf) <= 1e-5 * np.abs(wf)), f"{name}: fp32 output differs"
    return ws.numel()


def test_noalloc_matches_workspace_entry_point_twice():
    big = _both("bert_base_layer")   # fills most of the built-in buffer
    small = _both("tiny")            # second call, smaller input, same buffer
    assert small < big <= nm.NM_NOALLOC_MAX_WORKSPACE
    _both("ragged")                  # shapes that take the generic kernels


def test_noalloc_rejects_shapes_beyond_the_buffer():
    desc, x, M, H, keep = _layer("bert_base_s512")
    assert nm.nm_encoder_layer_workspace(desc) > nm.NM_NOALLOC_MAX_WORKSPACE
    y = torch.empty((M, H), dtype=torch.int8, device=DEV)
    with pytest.raises(nm.NmError) as ei:
        nm.nm_encoder_layer_noalloc(desc, x, y, None)
    assert ei.value.status == nm.NM_ERR_WORKSPACE
    assert "built-in buffer" in str(ei.value)
