"""Float64 CPU oracle for LeanQuant's per-layer quantization pass.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
pass computes, written from the paper (arXiv 2407.10032) and used solely to
check the HIP library: only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it.  It shares no code with the HIP
path and never takes an input or an expected value from it.

Everything is numpy float64 (the paper states no precision); fp32 inputs are
upcast on entry.  Steps follow Algorithm 1 in the paper's order and notation:
W is r x c (rows = output channels), X is held tokens-by-channels (N x c, the
transpose of the paper's c x N), b = bit width, B = block size, df = dampening
factor, p = outlier-preservation strength.

Readings of points the paper leaves open (each also listed in the design
document):
  * "Cholesky" in Algorithm 1 line 4 is the UPPER factor U with
    (H + lambda I)^-1 = U^T U, because lines 16-19 use rows U[j, j:] of it.
  * diag(H^-1) in Eq. 5 / Eq. 7 is the diagonal of the true damped inverse
    (Section 3.1 speaks of the inverse Hessian's diagonal), not of its factor.
  * Lloyd's algorithm runs to an assignment fixed point, at most max_iter
    (default 100) updates; an empty cluster keeps its centroid; a tie between
    two grid points goes to the lower one.            -- parity unpinned: the
    paper fixes neither the cap nor the empty-cluster rule.
  * Eq. 8's t is floored to an integer; candidates are t_min, t_max in
    {0..t} inclusive; rounding is round-half-to-even; Z is not clipped;
    a constant group gets S = 1, Z = 0.
  * Importance weights are used as omega_i = (d_i / min d)^-p; the common
    factor changes no argmin.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# Step 1-2: Hessian, dampening, inverse, Cholesky   (Algorithm 1, lines 3-4)
# --------------------------------------------------------------------------
def hessian(X, H=None):
    """H (+)= 2 X^T X for X given as N x c (Section 2.2: H = 2 X X^T with X c x N)."""
    X = np.asarray(X, dtype=F64)
    G = 2.0 * (X.T @ X)
    return G if H is None else H + G


def dampen(H, df):
    """H + df * avg(diag H) * I   (Algorithm 1 line 4; Section 2.2, 'mild dampening')."""
    H = np.asarray(H, dtype=F64)
    lam = df * np.mean(np.diag(H))
    return H + lam * np.eye(H.shape[0])


def cholesky_inv(H, df):
    """Return (U, d): U upper with (H_d)^-1 = U^T U, d = diag((H_d)^-1).

    Literal three-step route of Algorithm 1 line 4: dampen, invert, factor.
    """
    Hd = dampen(H, df)
    Hinv = np.linalg.inv(Hd)
    Hinv = 0.5 * (Hinv + Hinv.T)
    L = np.linalg.cholesky(Hinv)          # lower, Hinv = L L^T
    U = np.ascontiguousarray(L.T)         # upper, Hinv = U^T U
    return U, np.diag(Hinv).copy()


# --------------------------------------------------------------------------
# Quantizers   (Section 2.1)
# --------------------------------------------------------------------------
def quant_nu_index(w, G):
    """Index of the nearest point of the ascending grid G (last axis); ties -> lower index.

    w: (..., n), G: (..., K) with matching leading axes.
    """
    w = np.asarray(w, dtype=F64)
    G = np.asarray(G, dtype=F64)
    dist = np.abs(w[..., :, None] - G[..., None, :])
    return np.argmin(dist, axis=-1)       # first minimum = lowest index


def quant_nu(w, G):
    idx = quant_nu_index(w, G)
    return np.take_along_axis(np.asarray(G, dtype=F64), idx, axis=-1), idx


def quant_aff_int(w, S, Z, bits):
    """w_int = clip(round(w / S) + Z, 0, 2^b - 1)   (Section 2.1, affine grid)."""
    return np.clip(np.rint(np.asarray(w, dtype=F64) / S) + Z, 0.0, float(2 ** bits - 1))


def quant_aff(w, S, Z, bits):
    """(w_int - Z) * S and the integer code."""
    wi = quant_aff_int(w, S, Z, bits)
    return (wi - Z) * S, wi


def minmax_affine(w, bits):
    """Min-max asymmetric S and Z of one weight group (Section 2.1)."""
    w = np.asarray(w, dtype=F64)
    lo, hi = w.min(), w.max()
    if hi == lo:
        return 1.0, 0.0
    S = (hi - lo) / (2 ** bits - 1)
    return S, -np.rint(lo / S)


# --------------------------------------------------------------------------
# Step 3: loss-error-aware grids
# --------------------------------------------------------------------------
def importance(d, p):
    """omega_i = (d_i / min d)^-p, proportional to (H^-1_ii)^-p of Eq. 5 / Eq. 7."""
    d = np.asarray(d, dtype=F64)
    return (d / d.min()) ** (-float(p))


def uniform_init(w, bits):
    """Eq. 6: 2^b evenly spaced points from min(w) to max(w), last axis = row."""
    w = np.asarray(w, dtype=F64)
    K = 2 ** bits
    lo = w.min(axis=-1, keepdims=True)
    hi = w.max(axis=-1, keepdims=True)
    return lo + (hi - lo) / (K - 1) * np.arange(K, dtype=F64)


def eq5_objective(w, omega, G):
    """sum_i omega_i |quant_nu(w_i, G) - w_i|^2 per row (Eq. 5)."""
    q, _ = quant_nu(w, G)
    return np.sum(omega * (q - np.asarray(w, dtype=F64)) ** 2, axis=-1)


def lloyd_step(w, omega, G):
    """One assignment + centroid update of weighted 1-D k-means; returns (G_new, idx)."""
    K = G.shape[-1]
    idx = quant_nu_index(w, G)
    Gn = G.copy()
    for m in range(K):
        sel = (idx == m)
        den = np.sum(np.where(sel, omega, 0.0), axis=-1)
        num = np.sum(np.where(sel, omega * w, 0.0), axis=-1)
        ok = den > 0.0
        Gn[..., m] = np.where(ok, num / np.where(ok, den, 1.0), G[..., m])
    return Gn, idx


def fit_grid_nu(W, d, bits, p, max_iter=100, init=None, history=None):
    """Non-uniform grid per row: weighted k-means on the row's weights (Eq. 5),
    started from the uniformly spaced grid (Eq. 6), Lloyd's algorithm to an
    assignment fixed point or max_iter updates.  Returns G [r x 2^b] ascending.

    history (optional list) receives the per-row Eq. 5 objective before each update.
    """
    W = np.atleast_2d(np.asarray(W, dtype=F64))
    omega = importance(d, p)[None, :]
    G = uniform_init(W, bits) if init is None else np.array(init, dtype=F64, copy=True)
    prev = None
    done = np.zeros(W.shape[0], dtype=bool)
    for _ in range(max_iter):
        Gn, idx = lloyd_step(W, omega, G)
        if history is not None:
            history.append(eq5_objective(W, omega, G))
        if prev is not None:
            done |= np.all(idx == prev, axis=-1)
        # a row whose assignment did not change has stopped: its grid is kept
        G = np.where(done[:, None], G, Gn)
        prev = idx
        if done.all():
            break
    return G


def kmeanspp_init(W, d, bits, p, u):
    """Weighted k-means++ seeding, the initialisation the paper's appendix table on grid
    point initialisation compares Eq. 6 against (Arthur & Vassilvitskii's D^2 sampling with
    the importance weights of Eq. 5 as point masses).

    u [r x 2^b] are uniform numbers in [0, 1) supplied by the caller (one per centre), so
    that the procedure is a function of its inputs.  Centre 0 of a row is drawn with
    probability proportional to omega_i, centre m with probability proportional to
    omega_i * min_j (w_i - g_j)^2; a draw takes the first index whose cumulative mass
    reaches u * total.  If every remaining mass is zero the first column is taken.  Returns
    the centres of every row in ascending order.
    """
    W = np.atleast_2d(np.asarray(W, dtype=F64))
    omega = importance(d, p)
    r, c = W.shape
    K = 1 << bits
    u = np.asarray(u, dtype=F64).reshape(r, K)
    G = np.empty((r, K), dtype=F64)
    for k in range(r):
        w = W[k]
        dist2 = np.full(c, np.inf)
        for m in range(K):
            mass = omega if m == 0 else omega * dist2
            cum = np.cumsum(mass)
            total = cum[-1]
            i = 0 if not (total > 0.0) else int(min(np.searchsorted(cum, u[k, m] * total, side="left"), c - 1))
            if total > 0.0:
                while mass[i] == 0.0 and i + 1 < c:      # u = 0 or flat steps: a point with mass
                    i += 1
            G[k, m] = w[i]
            dist2 = np.minimum(dist2, (w - w[i]) ** 2)
    return np.sort(G, axis=1)


def shrink_steps(bits, T):
    """Eq. 8: t = 0.2T / 0.3T / 0.4T for b = 4 / 3 / 2, floored to an integer."""
    frac = {4: 0.2, 3: 0.3, 2: 0.4}[bits]
    return int(np.floor(frac * T + 1e-9))


def fit_group_aff(w, omega, bits, T, t):
    """Enumerative search of Eq. 7 on one group; returns (S, Z, loss, t_min, t_max).

    Candidates in the order t_min = 0..t (outer), t_max = 0..t (inner); the
    first smallest loss wins.
    """
    w = np.asarray(w, dtype=F64)
    omega = np.asarray(omega, dtype=F64)
    lo0, hi0 = w.min(), w.max()
    R = hi0 - lo0
    if R == 0.0:
        return 1.0, 0.0, eq7_objective(w, omega, 1.0, 0.0, bits), 0, 0
    qmax = float(2 ** bits - 1)
    tmax = np.arange(t + 1, dtype=F64)
    best = (np.inf, 0, 0, 1.0, 0.0)
    for tmin in range(t + 1):
        lo = lo0 + tmin * R / T
        hi = hi0 - tmax * R / T                      # (t+1,)
        S = (hi - lo) / qmax
        Z = -np.rint(lo / S)
        wi = np.clip(np.rint(w[None, :] / S[:, None]) + Z[:, None], 0.0, qmax)
        q = (wi - Z[:, None]) * S[:, None]
        loss = np.sum(omega[None, :] * (q - w[None, :]) ** 2, axis=1)
        k = int(np.argmin(loss))                     # first minimum
        if loss[k] < best[0]:
            best = (float(loss[k]), tmin, k, float(S[k]), float(Z[k]))
    return best[3], best[4], best[0], best[1], best[2]


def fit_grid_aff(W, d, bits, p, group_size=0, T=2048, t=None):
    """Affine grid per (row, group): returns SZ [r x n_groups x 2] = (S, Z)   (Eq. 7)."""
    W = np.atleast_2d(np.asarray(W, dtype=F64))
    r, c = W.shape
    g = c if group_size in (0, None) else int(group_size)
    if c % g:
        raise ValueError("group size must divide the number of columns")
    if t is None:
        t = shrink_steps(bits, T)
    omega = importance(d, p)
    SZ = np.empty((r, c // g, 2), dtype=F64)
    for k in range(r):
        for gi in range(c // g):
            sl = slice(gi * g, (gi + 1) * g)
            S, Z, _, _, _ = fit_group_aff(W[k, sl], omega[sl], bits, T, t)
            SZ[k, gi, 0] = S
            SZ[k, gi, 1] = Z
    return SZ


def eq7_objective(w, omega, S, Z, bits):
    q, _ = quant_aff(w, S, Z, bits)
    return float(np.sum(np.asarray(omega, dtype=F64) * (q - np.asarray(w, dtype=F64)) ** 2))


# --------------------------------------------------------------------------
# Step 4: blocked quantize-and-propagate loop   (Algorithm 1, lines 10-21)
# --------------------------------------------------------------------------
def quantize_layer(W, U, grid, mode, bits, group_size=0, B=128):
    """Run the column loop with H^-1 := U (upper Cholesky factor).

    grid: nu -> G [r x 2^b]; aff -> SZ [r x n_groups x 2].
    Returns (W_hat [r x c], codes [r x c] int, row_loss [r] = 1/2 sum_j E_kj^2,
    the summed loss error of Eq. 3 per row).
    """
    W = np.array(W, dtype=F64, copy=True)
    U = np.asarray(U, dtype=F64)
    r, c = W.shape
    What = np.zeros((r, c), dtype=F64)
    codes = np.zeros((r, c), dtype=np.int64)
    row_loss = np.zeros(r, dtype=F64)
    g = c if group_size in (0, None) else int(group_size)
    for i in range(0, c, B):
        nb = min(B, c - i)
        E = np.zeros((r, nb), dtype=F64)
        for j in range(i, i + nb):
            wj = W[:, j]
            if mode == "nu":
                q, code = quant_nu(wj[:, None], grid)
                q, code = q[:, 0], code[:, 0]
            elif mode == "aff":
                S = grid[:, j // g, 0]
                Z = grid[:, j // g, 1]
                q, code = quant_aff(wj, S, Z, bits)
            else:
                raise ValueError(mode)
            What[:, j] = q
            codes[:, j] = code
            e = (wj - q) / U[j, j]
            E[:, j - i] = e
            W[:, j:i + nb] -= np.outer(e, U[j, j:i + nb])
        W[:, i + nb:] -= E @ U[i:i + nb, i + nb:]
        row_loss += 0.5 * np.sum(E * E, axis=1)
    return What, codes, row_loss


def layer_loss(W, What, H):
    """tr((W - W_hat) H (W - W_hat)^T) = ||W X - W_hat X||_F^2 * 2 (Eq. 1 with H = 2 X X^T)."""
    D = np.asarray(W, dtype=F64) - np.asarray(What, dtype=F64)
    return float(np.sum((D @ np.asarray(H, dtype=F64)) * D))


# --------------------------------------------------------------------------
# The whole pass   (Algorithm 1)
# --------------------------------------------------------------------------
def leanquant_layer(W, H, mode, bits, df=0.01, p=4.0, B=128, group_size=0, T=2048, t=None,
                    max_iter=100):
    """Algorithm 1 from an accumulated H: returns dict with U, d, grid, W_hat, codes, row_loss."""
    U, d = cholesky_inv(H, df)
    if mode == "nu":
        grid = fit_grid_nu(W, d, bits, p, max_iter=max_iter)
    else:
        grid = fit_grid_aff(W, d, bits, p, group_size=group_size, T=T, t=t)
    What, codes, row_loss = quantize_layer(W, U, grid, mode, bits, group_size=group_size, B=B)
    return dict(U=U, d=d, grid=grid, W_hat=What, codes=codes, row_loss=row_loss)


# --------------------------------------------------------------------------
# Exhaustive per-column OBS in fixed order (Eq. 3 and Eq. 9): an independent
# statement of the loop used to pin quantize_layer on tiny layers.
# --------------------------------------------------------------------------
def obs_fixed_order(W, Hd, quant_col):
    """Quantize columns 0..c-1 in order with the explicit inverse Hessian.

    quant_col(j, w_col) -> quantized column.  After each column the remaining
    weights move by -delta_j (Eq. 3) and the inverse Hessian loses row and
    column j (Eq. 9).  Returns (W_hat, sum over columns of eps_j per row).
    """
    W = np.array(W, dtype=F64, copy=True)
    Hinv = np.linalg.inv(np.asarray(Hd, dtype=F64))
    r, c = W.shape
    What = np.zeros_like(W)
    eps = np.zeros(r, dtype=F64)
    for j in range(c):
        q = quant_col(j, W[:, j])
        What[:, j] = q
        err = q - W[:, j]                                   # quant(w_j) - w_j
        eps += 0.5 * err ** 2 / Hinv[j, j]
        W += np.outer(err / Hinv[j, j], Hinv[:, j])         # w <- w + delta_j
        Hinv = Hinv - np.outer(Hinv[:, j], Hinv[j, :]) / Hinv[j, j]
        Hinv[j, :] = 0.0
        Hinv[:, j] = 0.0
        Hinv[j, j] = 1.0                                    # placeholder, never used again
    return What, eps


# --------------------------------------------------------------------------
# LeanQuant-Exact (Algorithm 2 of the appendix): greedy order, explicit inverse
# --------------------------------------------------------------------------
def exact_row(w, Hinv, quant):
    """Algorithm 2's loop for one row.

    w [c]; Hinv [c x c] the inverse Hessian the row starts from; quant(w_vec) ->
    (quantized values, codes) on the row's fixed grid.  In each of the c steps the
    not yet quantized weight with the smallest loss error (quant(w_i) - w_i)^2 /
    (2 Hinv_ii) (Eq. 3) is quantized (ties: lowest index), the other weights move by
    -Hinv[:, i] / Hinv_ii (w_i - w_hat_i), and row and column i leave the inverse
    (Eq. 9).  Returns (w_hat, codes, order, eps) with eps the summed loss error.
    """
    w = np.array(w, dtype=F64, copy=True)
    Hinv = np.array(Hinv, dtype=F64, copy=True)
    c = w.size
    w_hat = np.zeros(c, dtype=F64)
    codes = np.zeros(c, dtype=np.int64)
    live = np.ones(c, dtype=bool)
    order = []
    eps = 0.0
    for _ in range(c):
        q, code = quant(w)
        score = np.where(live, (q - w) ** 2 / (2.0 * np.where(live, np.diag(Hinv), 1.0)), np.inf)
        i = int(np.argmin(score))                     # first minimum = lowest index
        order.append(i)
        eps += score[i]
        w_hat[i] = q[i]
        codes[i] = code[i]
        hii = Hinv[i, i]
        col = Hinv[:, i].copy()
        w = w - col / hii * (w[i] - q[i])
        Hinv = Hinv - np.outer(col, Hinv[i, :]) / hii
        Hinv[i, :] = 0.0
        Hinv[:, i] = 0.0
        live[i] = False
        w[i] = q[i]
    return w_hat, codes, np.array(order), eps


def leanquant_exact(W, H, mode, bits, df=0.01, p=4.0, T=2048, t=None, max_iter=100):
    """Algorithm 2 for every row of W from an accumulated H.

    Readings: the inverse is the damped one, as in Algorithm 1 (Algorithm 2 writes
    (2 X X^T)^-1; Section 2.2's dampening is what keeps it invertible); the grid is
    learned once from the original row (lines 3-7 precede the loop); the affine grid is
    one (S, Z) per row.  Returns dict with grid, W_hat, codes, order, eps.
    """
    W = np.atleast_2d(np.asarray(W, dtype=F64))
    Hinv = np.linalg.inv(dampen(H, df))
    d = np.diag(Hinv).copy()
    r, c = W.shape
    if mode == "nu":
        grid = fit_grid_nu(W, d, bits, p, max_iter=max_iter)
    else:
        grid = fit_grid_aff(W, d, bits, p, group_size=0, T=T, t=t)
    What = np.zeros((r, c))
    codes = np.zeros((r, c), dtype=np.int64)
    order = np.zeros((r, c), dtype=np.int64)
    eps = np.zeros(r)
    for k in range(r):
        if mode == "nu":
            quant = lambda v, G=grid[k]: quant_nu(v, G)
        else:
            S, Z = grid[k, 0, 0], grid[k, 0, 1]
            quant = lambda v, S=S, Z=Z: quant_aff(v, S, Z, bits)
        What[k], codes[k], order[k], eps[k] = exact_row(W[k], Hinv, quant)
    return dict(grid=grid, W_hat=What, codes=codes, order=order, eps=eps, Hinv=Hinv, d=d)
