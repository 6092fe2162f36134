"""Glue shared by the GPU tests, the smoke check and the benchmark: uploads of generated inputs and
numpy re-statements of the documented index maps.  No kernel arithmetic lives here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2605_08568_amd as pa
import synth_inputs as si


def upload_layer(lay: si.Layer, device="cuda") -> pa.Layer:
    """Row-major device copy of a generated layer."""
    if lay.dtype == "bf16":
        Vt = pa.bf16_from_bits(lay.Vt_store, device); Ut = pa.bf16_from_bits(lay.Ut_store, device)
    else:
        Vt = torch.from_numpy(lay.Vt_store).to(device); Ut = torch.from_numpy(lay.Ut_store).to(device)
    return pa.Layer(Vt, Ut, lay.n, lay.m, lay.R, lay.G, pa.PARSE_ROWMAJOR)


def upload_tokens(X: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    return pa.bf16_from_bits(X, device) if dtype == "bf16" else torch.from_numpy(X).to(device)


def i32(a, device="cuda") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)


def mfma16_v(Vt: np.ndarray) -> np.ndarray:
    """The operand-order index map of the header for the right factor, restated with numpy axes:
    (r, i) -> [rb][kb][q][j][e] with r = 32 rb + j, i = 16 kb + 8 q + e."""
    R, n = Vt.shape
    return np.ascontiguousarray(Vt.reshape(R // 32, 32, n // 16, 2, 8).transpose(0, 2, 3, 1, 4)).reshape(R, n)


def mfma16_u(Ut: np.ndarray) -> np.ndarray:
    """(r, c) -> [kb][cb][q][j][e] with r = 16 kb + 8 q + e, c = 32 cb + j."""
    R, m = Ut.shape
    return np.ascontiguousarray(Ut.reshape(R // 16, 2, 8, m // 32, 32).transpose(0, 3, 1, 4, 2)).reshape(R, m)


def oracle_factors(lay: si.Layer):
    """(U0, sigma, V) for the oracle: exact generator factors for fp32 layers; for bf16 layers the rounded
    stored values with sigma already inside the left factor."""
    if lay.dtype == "bf16":
        Vt, Ut = lay.stored_values()
        return Ut.T.copy(), np.ones(lay.R), Vt
    return lay.U0, lay.sigma, lay.V


# ---- guard bands: every output and workspace of a checked call sits between two canaries of 4 KiB -----------------
CANARY = 4096
_CANARY_BYTE = 0xA5


def guarded_bytes(nbytes: int, device="cuda"):
    """(whole buffer, the nbytes in the middle); both ends hold the canary byte."""
    nbytes = max(int(nbytes), 256)
    buf = torch.full((nbytes + 2 * CANARY,), _CANARY_BYTE, dtype=torch.uint8, device=device)
    return buf, buf[CANARY:CANARY + nbytes]


def guarded_like(rows: int, cols: int, dtype, device="cuda"):
    """(whole buffer, a [rows][cols] tensor of `dtype` in its middle)."""
    esz = torch.empty((), dtype=dtype).element_size()
    buf, mid = guarded_bytes(rows * cols * esz, device)
    return buf, mid[:rows * cols * esz].view(dtype).view(rows, cols)


def check_guards(buf: torch.Tensor, what: str):
    torch.cuda.synchronize()
    n = buf.numel() - 2 * CANARY
    assert bool(torch.all(buf[:CANARY] == _CANARY_BYTE)), f"{what}: stores below the buffer"
    assert bool(torch.all(buf[CANARY + n:] == _CANARY_BYTE)), f"{what}: stores beyond the buffer"


def forward_guarded(mode, layer, patterns, X, tok_offsets, pattern_id, Y=None, workspace=None, no_workspace=False):
    """pa.lowrank_forward with Y and the workspace (exactly the queried size) between canaries, checked after the call."""
    if Y is not None or workspace is not None:
        return pa.lowrank_forward(mode, layer, patterns, X, tok_offsets, pattern_id, Y, workspace, no_workspace)
    rows = X.shape[0]
    ybuf, Yt = guarded_like(rows, layer.m, X.dtype, X.device)
    wbuf, ws = None, None
    if not no_workspace:
        need = pa.lowrank_workspace_bytes(mode, layer, rows, patterns.k, pattern_id.numel(), patterns.n_patterns)
        wbuf, ws = guarded_bytes(need, X.device)
    pa.lowrank_forward(mode, layer, patterns, X, tok_offsets, pattern_id, Yt, ws, no_workspace)
    check_guards(ybuf, "Y")
    if wbuf is not None:
        check_guards(wbuf, "workspace")
    return Yt


def decode_multi_guarded(layers, patterns, X, pattern_id):
    rows = X.shape[0]
    ys = [guarded_like(rows, l.m, X.dtype, X.device) for l in layers]
    wbuf, ws = guarded_bytes(pa.lowrank_decode_multi_workspace_bytes(layers), X.device)
    pa.lowrank_decode_multi(layers, patterns, X, pattern_id, [v for _, v in ys], ws)
    for i, (b, _) in enumerate(ys):
        check_guards(b, f"Y[{i}]")
    check_guards(wbuf, "workspace")
    return [v for _, v in ys]


def prefill_multi_guarded(layers, patterns, X, tok_offsets, pattern_id):
    rows = X.shape[0]
    ys = [guarded_like(rows, l.m, X.dtype, X.device) for l in layers]
    import ctypes as C
    from paper_2605_08568_amd import binding as _b
    nl = len(layers)
    larr = (_b._Layer * nl)(*[l.c() for l in layers])
    parr = (_b._Patterns * nl)(*[p.c() for p in patterns])
    wbuf, ws = guarded_bytes(int(pa.lib().parse_lowrank_prefill_multi_workspace_bytes(larr, parr, nl, rows)), X.device)
    pa.lowrank_prefill_multi(layers, patterns, X, tok_offsets, pattern_id, [v for _, v in ys], ws)
    for i, (b, _) in enumerate(ys):
        check_guards(b, f"Y[{i}]")
    check_guards(wbuf, "workspace")
    return [v for _, v in ys]
