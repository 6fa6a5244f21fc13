"""Helpers shared by the GPU parity tests: drive the HIP library through its
binding and bring results back as numpy arrays; compare grids and codes with the
oracle under the acceptance rules of the tests."""
from __future__ import annotations

import numpy as np
import torch

import paper_2407_10032_amd as lq

DEV = "cuda"


def to_dev(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV, dtype=dtype)


params_for = lq.params_for
grid_shape = lq.grid_shape


def gpu_hessian(x_chunks, c):
    """Accumulate H over an iterable of [n x c] fp32 numpy chunks."""
    H = torch.zeros((c, c), dtype=torch.float32, device=DEV)
    ws = None
    for xc in x_chunks:
        X = to_dev(xc)
        need = lq.lq_workspace_bytes(lq.LQ_CALL_HESSIAN, 0, c, X.shape[0])
        if ws is None or ws.numel() < need:
            ws = lq.alloc_workspace(need)
        lq.lq_hessian_accumulate(H, X, ws)
    torch.cuda.synchronize()
    return H


def gpu_cholesky(H, damp):
    c = H.shape[0]
    U = torch.empty((c, c), dtype=torch.float32, device=DEV)
    d = torch.empty(c, dtype=torch.float32, device=DEV)
    info = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    ws = lq.alloc_workspace(lq.lq_workspace_bytes(lq.LQ_CALL_CHOLESKY, 0, c))
    lq.lq_cholesky_inv(H, damp, U, d, info, ws)
    torch.cuda.synchronize()
    return U, d, int(info.item())


def gpu_fit_grid(W, d, P, init=None):
    r, c = W.shape
    grid = torch.empty(grid_shape(P, r, c), dtype=torch.float32, device=DEV)
    ws = lq.alloc_workspace(lq.lq_workspace_bytes(lq.LQ_CALL_FIT_GRID, r, c, 0, P))
    if init is None:
        lq.lq_fit_grid(W, d, P, grid, ws)
    else:
        lq.lq_fit_grid_from(W, d, P, init, grid, ws)
    torch.cuda.synchronize()
    return grid


def gpu_quantize(W, U, grid, P, want_loss=True):
    """Returns (W_hat, codes, row_loss); W is copied first (the call works in place)."""
    r, c = W.shape
    Wq = W.clone()
    codes = torch.empty((r, c), dtype=torch.uint8, device=DEV)
    row_loss = torch.empty(r, dtype=torch.float32, device=DEV) if want_loss else None
    ws = lq.alloc_workspace(lq.lq_workspace_bytes(lq.LQ_CALL_QUANTIZE, r, c, 0, P))
    lq.lq_quantize_layer(Wq, U, grid, P, codes, row_loss, ws)
    torch.cuda.synchronize()
    return Wq, codes, row_loss


def gpu_layer_pass(W_np, x_chunks, P):
    """All four calls on the device; returns a dict of numpy results."""
    c = W_np.shape[1]
    H = gpu_hessian(x_chunks, c)
    U, d, info = gpu_cholesky(H, P.damp)
    W = to_dev(W_np)
    grid = gpu_fit_grid(W, d, P)
    Wq, codes, row_loss = gpu_quantize(W, U, grid, P)
    return dict(H=H.cpu().numpy(), U=U.cpu().numpy(), d=d.cpu().numpy(), info=info,
                grid=grid.cpu().numpy(), W_hat=Wq.cpu().numpy(), codes=codes.cpu().numpy(),
                row_loss=row_loss.cpu().numpy())


# ------------------------------------------------------------------ comparisons
def nu_grid_match(G_gpu, G_ref, rtol=1e-4):
    """Per row: every centroid within rtol * max|g| of the oracle's."""
    scale = np.abs(G_ref).max(axis=1, keepdims=True)
    return np.all(np.abs(G_gpu - G_ref) <= rtol * scale, axis=1)


def aff_grid_match(SZ_gpu, SZ_ref, rtol=1e-4):
    """Per group: S within rtol relative and the same integer zero-point."""
    s_ok = np.abs(SZ_gpu[..., 0] - SZ_ref[..., 0]) <= rtol * np.abs(SZ_ref[..., 0])
    z_ok = SZ_gpu[..., 1] == SZ_ref[..., 1]
    return s_ok & z_ok


def code_agreement(codes_gpu, codes_ref):
    return float(np.mean(codes_gpu.astype(np.int64) == codes_ref.astype(np.int64)))


def compare_rows_strict(mode, bits, W_rows, d, U64, grid_g, codes_g, grid_ref, codes_ref, p=4.0,
                        group_size=0, B=128, say=print):
    """Grid and code check of EVERY sampled row against the float64 oracle.

    A row whose grid equals the oracle's (1e-4 relative; affine: every group's S within 1e-4
    and the same integer Z) has its codes compared with the oracle's codes.  A row whose grid
    differs must carry an equally good grid -- Eq. 5 objective of the row within 1e-3 of the
    oracle's (non-uniform), Eq. 7 objective of every differing group within 1e-5 (affine), both
    evaluated in float64 -- and its codes are compared with the oracle's column loop run from
    the DEVICE's grid for that row (rows are independent problems, Eq. 1).  Asserts the
    objective rule; returns (share of rows / groups with the oracle's grid, pooled code
    agreement over all rows, number of rows re-run from the device's grid).
    """
    from oracle import leanquant_oracle as orc

    W64 = np.asarray(W_rows, dtype=np.float64)
    om = orc.importance(d, p)
    gg = np.asarray(grid_g, dtype=np.float64)
    if mode == "nu":
        row_ok = nu_grid_match(gg, grid_ref)
        share = float(row_ok.mean())
        if (~row_ok).any():
            og = orc.eq5_objective(W64[~row_ok], om, gg[~row_ok])
            orf = orc.eq5_objective(W64[~row_ok], om, np.asarray(grid_ref)[~row_ok])
            say(f"    {int((~row_ok).sum())} rows with another grid: Eq. 5 objective ratios {np.array2string(og / orf, precision=6)}")
            assert np.all(og <= orf * (1 + 1e-3)), (og / orf)
    else:
        g = group_size if group_size else W64.shape[1]
        m = aff_grid_match(gg, grid_ref)
        row_ok = m.all(axis=1)
        share = float(m.mean())
        worst = 0.0
        for k, gi in zip(*np.nonzero(~m)):
            sl = slice(gi * g, (gi + 1) * g)
            og = orc.eq7_objective(W64[k, sl], om[sl], float(gg[k, gi, 0]), float(gg[k, gi, 1]), bits)
            orf = orc.eq7_objective(W64[k, sl], om[sl], float(grid_ref[k, gi, 0]), float(grid_ref[k, gi, 1]), bits)
            worst = max(worst, og / orf - 1.0)
            assert og <= orf * (1 + 1e-5), (k, gi, og, orf)
        if (~m).any():
            say(f"    {int((~m).sum())} groups with another (S, Z): worst Eq. 7 objective excess {worst:.2e}")
    ref_codes = np.array(codes_ref, dtype=np.int64, copy=True)
    redo = np.nonzero(~row_ok)[0]
    if redo.size:
        _, c2, _ = orc.quantize_layer(W64[redo], U64, gg[redo], mode, bits, group_size=group_size, B=B)
        ref_codes[redo] = c2
    agree = code_agreement(np.asarray(codes_g), ref_codes)
    return share, agree, int(redo.size)
