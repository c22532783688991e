"""Shared plumbing of the GPU parity tests: move a seeded workload to the GPU, run the
library through its C ABI, compute the oracle, and measure the error the way the
tolerances are stated."""
from __future__ import annotations

import numpy as np

import bcr_inputs as gen
from oracle import bcr_oracle as orc

# max error relative to the scale of the sum (S = sum of |terms|) and to max|Y|:
# 1e-5 for fp32, 2e-3 for fp16 / bf16 inputs with fp32 accumulation
TOL = {gen.F32: 1e-5, gen.F16: 2e-3, gen.BF16: 2e-3}


def torch_dev():
    import torch
    return torch, torch.device("cuda:0")


def to_device(a: np.ndarray, dtype: str):
    """Storage-typed NumPy array -> torch tensor on the GPU (same bits)."""
    torch, dev = torch_dev()
    if dtype == gen.BF16:
        return torch.from_numpy(a.view(np.int16).copy()).to(dev).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def pack_workload(g, W, dtype, mask, **kw):
    return g.pack(W, dtype, mask.BR, mask.BC, mask.row_ptr, mask.row_idx, mask.col_ptr, mask.col_idx, **kw)


def oracle_product(W, X, dtype, mask, rows=None, cols=None):
    return orc.bcr_product(gen.storage_to_f64(W, dtype), gen.storage_to_f64(X, dtype), mask, rows=rows, cols=cols)


def errors(Y: np.ndarray, Yref: np.ndarray, S: np.ndarray):
    """(max |Y - Yref| / S over entries with S > 0,  max |Y - Yref| / max |Yref|,
    exact-zero check where S == 0)."""
    Y = np.asarray(Y, dtype=np.float64)
    diff = np.abs(Y - Yref)
    pos = S > 0
    e_scale = float((diff[pos] / S[pos]).max()) if pos.any() else 0.0
    denom = float(np.abs(Yref).max())
    e_max = float(diff.max() / denom) if denom > 0 else float(diff.max())
    zeros_ok = bool((Y[~pos] == 0).all())
    return e_scale, e_max, zeros_ok


def assert_close(Y, Yref, S, dtype, what=""):
    assert np.isfinite(np.asarray(Y)).all(), f"{what}: non-finite output (unwritten or corrupt)"
    e_scale, e_max, zeros_ok = errors(Y, Yref, S)
    tol = TOL[dtype]
    assert zeros_ok, f"{what}: an output with no surviving term is not exactly zero"
    assert e_scale <= tol, f"{what}: max |err| / sum|terms| = {e_scale:.3e} > {tol}"
    assert e_max <= tol, f"{what}: max |err| / max|Y| = {e_max:.3e} > {tol}"
    return e_scale, e_max


def run_spmm(g, A, X_np, dtype, M, N, ldx=None, ldy=None, **tune):
    """Run grim_bcr_spmm on a K x N host matrix; returns Y (M x N float32, host).  Y is
    prefilled with NaN so that an unwritten entry is caught."""
    torch, dev = torch_dev()
    K = X_np.shape[0]
    ldx = N if ldx is None else ldx
    ldy = N if ldy is None else ldy
    Xp = np.zeros((K, ldx), dtype=X_np.dtype)
    Xp[:, :N] = X_np
    Xd = to_device(Xp, dtype)
    Yd = torch.full((M, ldy), float("nan"), dtype=torch.float32, device=dev)
    g.spmm(A, Xd, N, ldx, Yd, ldy, torch.cuda.current_stream(), **tune)
    torch.cuda.synchronize()
    Y = Yd.cpu().numpy()
    if ldy > N:
        assert np.isnan(Y[:, N:]).all(), "wrote outside the N columns of Y"
    return Y[:, :N].copy()


def run_spmv(g, A, x_np, dtype, M, batch, ldx=None, ldy=None):
    torch, dev = torch_dev()
    K = x_np.shape[0]
    ldx = batch if ldx is None else ldx
    ldy = batch if ldy is None else ldy
    xp = np.zeros((K, ldx), dtype=x_np.dtype)
    xp[:, :batch] = x_np
    xd = to_device(xp, dtype)
    yd = torch.full((M, ldy), float("nan"), dtype=torch.float32, device=dev)
    g.spmv(A, xd, batch, ldx, yd, ldy, torch.cuda.current_stream())
    torch.cuda.synchronize()
    y = yd.cpu().numpy()
    if ldy > batch:
        assert np.isnan(y[:, batch:]).all()
    return y[:, :batch].copy()
