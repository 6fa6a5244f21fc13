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
