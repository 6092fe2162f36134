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
