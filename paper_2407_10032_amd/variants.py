"""Summed loss of a quantized layer under the grid-fit variants the paper ablates.

    python -m paper_2407_10032_amd.variants [--config c1] [--rows 0] [--tokens 0]

For one seeded synthetic layer: H, U and d are computed once (Algorithm 1 lines 3-4); then,
for every bit width, the outlier-preservation strength p of Eq. 5 in {0, 2, 3, 4} and the
two initialisations (Eq. 6 and k-means++), and for affine grids the search of Eq. 7 against
the plain min-max grid, the grids are learned and the column loop run, and
the layer's loss  sum_k 1/2 (w_k - w_hat_k) H_d (w_k - w_hat_k)^T  (the sum the loop's scaled
errors add up to) is printed relative to the p = 4 / Eq. 6 setting of the paper.  Everything
runs on the GPU through the C ABI; the uniform numbers of the k-means++ draws come from a
seeded numpy generator.  The perplexity columns of the paper's tables need models and data
that are not here; this is the layer-level quantity those tables move with.
"""
from __future__ import annotations

import argparse

import numpy as np
import torch

import lq_synth

from . import binding as lq


def _ws(which, r, c, n, P):
    return lq.alloc_workspace(lq.lq_workspace_bytes(which, r, c, n, P))


def layer_loss(W, U, d, P, init):
    """init: None (Eq. 6) or a device tensor [r x 2^b] of uniforms for k-means++ seeding."""
    r, c = W.shape
    K = 1 << P.bits
    ws = _ws(lq.LQ_CALL_FIT_GRID, r, c, 0, P)
    if P.mode == lq.LQ_GRID_AFFINE:
        g = P.group_size if P.group_size > 0 else c
        grid = torch.empty((r, c // g, 2), dtype=torch.float32, device="cuda")
    else:
        grid = torch.empty((r, K), dtype=torch.float32, device="cuda")
    if P.mode == lq.LQ_GRID_AFFINE:
        lq.lq_fit_grid(W, d, P, grid, ws)
    elif init is None:
        lq.lq_fit_grid(W, d, P, grid, ws)
    else:
        seed = torch.empty((r, K), dtype=torch.float32, device="cuda")
        lq.lq_kmeanspp_seed(W, d, P, init, seed, ws)
        lq.lq_fit_grid_from(W, d, P, seed, grid, ws)
    Wq = W.clone()
    codes = torch.empty((r, c), dtype=torch.uint8, device="cuda")
    row_loss = torch.empty(r, dtype=torch.float32, device="cuda")
    lq.lq_quantize_layer(Wq, U, grid, P, codes, row_loss, _ws(lq.LQ_CALL_QUANTIZE, r, c, 0, P))
    torch.cuda.synchronize()
    return float(row_loss.double().sum().item())


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", default="c1")
    ap.add_argument("--rows", type=int, default=0, help="use only the first ROWS rows of W")
    ap.add_argument("--tokens", type=int, default=0, help="override the token count")
    args = ap.parse_args()
    lq.load()
    cfg = lq_synth.CONFIGS[args.config]
    if args.tokens:
        cfg = cfg.scaled(n_tokens=args.tokens)
    c = cfg.c
    H = torch.zeros((c, c), dtype=torch.float32, device="cuda")
    ws = None
    for xc in lq_synth.activation_chunks(cfg):
        X = torch.from_numpy(np.ascontiguousarray(xc, dtype=np.float32)).cuda()
        need = lq.lq_workspace_bytes(lq.LQ_CALL_HESSIAN, 0, c, X.shape[0], None)
        if ws is None or ws.numel() < need:
            ws = lq.alloc_workspace(need)
        lq.lq_hessian_accumulate(H, X, ws)
    U = torch.empty((c, c), dtype=torch.float32, device="cuda")
    d = torch.empty(c, dtype=torch.float32, device="cuda")
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    lq.lq_cholesky_inv(H, cfg.damp, U, d, info, _ws(lq.LQ_CALL_CHOLESKY, 0, c, 0, None))
    assert int(info.item()) == 0
    Wn = lq_synth.weights(cfg)
    if args.rows:
        Wn = Wn[:args.rows]
    W = torch.from_numpy(np.ascontiguousarray(Wn, dtype=np.float32)).cuda()
    r = W.shape[0]
    print("layer %s: W %d x %d, %d tokens, damp %.2f, B = %d" % (cfg.name, r, c, cfg.n_tokens, cfg.damp, cfg.block))
    print("%-5s %-6s %-10s %14s %10s" % ("bits", "p", "init", "sum of loss", "vs paper"))
    for bits in (4, 3, 2):
        u = torch.from_numpy(np.random.default_rng(9000 + bits).random((r, 1 << bits))).cuda()
        base = None
        rows = []
        for p in (4.0, 3.0, 2.0, 0.0):
            for name, init in (("Eq. 6", None), ("k-means++", u)):
                P = lq.lq_params_default(bits=bits, mode=lq.LQ_GRID_NONUNIFORM, block=cfg.block,
                                         damp=cfg.damp, p=p, T=cfg.T)
                loss = layer_loss(W, U, d, P, init)
                if base is None:
                    base = loss
                rows.append((bits, p, name, loss, loss / base))
        for b, p, name, loss, rel in rows:
            print("%-5d %-6g %-10s %14.6e %10.4f" % (b, p, name, loss, rel))
    # affine grids: the search of Eq. 7 against the plain min-max grid (no shrinking, t = 0,
    # the grid of the GPTQ baseline), with and without the loss-error-aware weights
    print("%-5s %-6s %-6s %-10s %14s %10s" % ("bits", "group", "p", "grid", "sum of loss", "vs paper"))
    for bits, group in ((4, 128), (3, 128), (2, 64)):
        if c % group:
            continue
        base = None
        for p, t_override, name in ((4.0, -1, "Eq. 7"), (0.0, -1, "Eq. 7"), (4.0, 0, "min-max")):
            P = lq.lq_params_default(bits=bits, mode=lq.LQ_GRID_AFFINE, group_size=group, block=cfg.block,
                                     damp=cfg.damp, p=p, T=cfg.T, t_override=t_override)
            loss = layer_loss(W, U, d, P, None)
            if base is None:
                base = loss
            print("%-5d %-6d %-6g %-10s %14.6e %10.4f" % (bits, group, p, name, loss, loss / base))


if __name__ == "__main__":
    main()
