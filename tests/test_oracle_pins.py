"""Pins that tie the float64 oracle to what the paper and the mathematics fix.

None of these re-type the oracle's own formula: each checks it against a
closed form, a library routine, a brute-force enumeration written separately,
an invariant, or a value the paper prints.  CPU only.
"""
import itertools
import os

import numpy as np
import pytest
import scipy.linalg
from scipy.cluster.vq import kmeans2

from oracle import leanquant_oracle as orc

RNG = np.random.default_rng


def _spd_case(c, n, seed, outliers=2):
    g = RNG(seed)
    X = g.standard_normal((n, c))
    for ch in g.choice(c, size=min(outliers, c), replace=False):
        X[:, ch] *= 7.0
    return X


# ------------------------------------------------------------------ step 1
def test_hessian_is_twice_gram_by_explicit_loops():
    """Section 2.2: H = 2 X X^T (X is c x N).  Triple loop over its definition."""
    g = RNG(1)
    N, c = 7, 4
    X = g.standard_normal((N, c))
    H = orc.hessian(X)
    ref = np.zeros((c, c))
    for a in range(c):
        for b in range(c):
            for t in range(N):
                ref[a, b] += 2.0 * X[t, a] * X[t, b]
    assert H.shape == (c, c)
    np.testing.assert_allclose(H, ref, rtol=1e-13, atol=1e-13)
    # accumulation over token chunks gives the same matrix
    H2 = orc.hessian(X[4:], orc.hessian(X[:4]))
    np.testing.assert_allclose(H2, ref, rtol=1e-13, atol=1e-13)


def test_hessian_layer_loss_identity():
    """Eq. 1: ||W X - W_hat X||_F^2 = 1/2 tr(D H D^T) with X c x N, H = 2 X X^T."""
    g = RNG(2)
    N, c, r = 50, 6, 3
    X = g.standard_normal((N, c))
    W = g.standard_normal((r, c))
    Wh = W + 0.1 * g.standard_normal((r, c))
    lhs = np.linalg.norm(W @ X.T - Wh @ X.T) ** 2
    assert orc.layer_loss(W, Wh, orc.hessian(X)) == pytest.approx(2.0 * lhs, rel=1e-12)


# ------------------------------------------------------------------ step 2
def test_dampening_closed_form():
    """Algorithm 1 line 4: lambda = df * avg(diag H)."""
    H = np.diag([1.0, 2.0, 3.0, 10.0])
    Hd = orc.dampen(H, 0.01)
    np.testing.assert_allclose(np.diag(Hd), np.array([1, 2, 3, 10]) + 0.01 * 4.0)
    assert np.count_nonzero(Hd - np.diag(np.diag(Hd))) == 0


def test_cholesky_inv_diagonal_closed_form():
    h = np.array([4.0, 1.0, 0.25, 9.0])
    U, d = orc.cholesky_inv(np.diag(h), 0.5)
    lam = 0.5 * h.mean()
    np.testing.assert_allclose(U, np.diag(1.0 / np.sqrt(h + lam)), atol=1e-15)
    np.testing.assert_allclose(d, 1.0 / (h + lam), rtol=1e-14)


def test_cholesky_inv_against_lapack_and_identities():
    X = _spd_case(24, 200, 3)
    H = orc.hessian(X)
    U, d = orc.cholesky_inv(H, 0.01)
    Hd = H + 0.01 * np.trace(H) / 24 * np.eye(24)
    # upper triangular with positive diagonal, U^T U H_d = I
    assert np.allclose(U, np.triu(U))
    assert np.all(np.diag(U) > 0)
    np.testing.assert_allclose(U.T @ U @ Hd, np.eye(24), atol=1e-9)
    # LAPACK on the explicit inverse (scipy), upper factor
    ref = scipy.linalg.cholesky(scipy.linalg.inv(Hd), lower=False)
    np.testing.assert_allclose(U, ref, rtol=1e-8, atol=1e-12)
    # d is the true inverse diagonal = column sums of squares of U
    np.testing.assert_allclose(d, np.diag(scipy.linalg.inv(Hd)), rtol=1e-9)
    np.testing.assert_allclose(d, np.sum(U * U, axis=0), rtol=1e-9)
    # one-factorization route: H_d = R R^T with R upper  =>  U = R^-1
    J = np.eye(24)[::-1]
    Lr = np.linalg.cholesky(J @ Hd @ J)
    R = J @ Lr @ J
    assert np.allclose(R, np.triu(R))
    np.testing.assert_allclose(np.linalg.inv(R), U, rtol=1e-8, atol=1e-12)
    # a lower factor would NOT satisfy this: guards a transposed result
    assert not np.allclose(U @ U.T @ Hd, np.eye(24), atol=1e-6)


# ------------------------------------------------------------------ quantizers
def _golden(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        out[k] = [float(x) for x in v]
    return out


def test_paper_toy_grid(repo_root):
    """Appendix 'Quantization Grid': a 2-bit grid {-1, -0.33, 0.33, 1} sends 0.25 to 0.33,
    and evenly spaced points over [-1, 1] are exactly that grid (Eq. 6)."""
    gold = _golden(os.path.join(repo_root, "tests", "golden", "toy_grid_b2.txt"))
    bits = int(gold["bits"][0])
    w = np.array([[gold["wmin"][0], gold["weight"][0], gold["wmax"][0]]])
    G = orc.uniform_init(w, bits)
    np.testing.assert_allclose(G[0], gold["grid"], atol=0.005)
    qn, idx = orc.quant_nu(np.array([gold["weight"]]), np.array([gold["grid"]]))
    assert qn[0, 0] == gold["quantized"][0] and idx[0, 0] == 2
    qn, idx = orc.quant_nu(np.array([gold["weight"]]), G)
    assert qn[0, 0] == pytest.approx(gold["quantized"][0], abs=0.005) and idx[0, 0] == 2


def test_minmax_affine_grid_closed_form():
    """Section 2.1: when min(w)/S is an integer the affine grid is the 2^b evenly
    spaced points from min(w) to max(w); every point maps to itself."""
    for bits, lo, hi in ((2, -1.0, 2.0), (3, -3.5, 0.0), (4, 0.0, 7.5)):
        w = np.array([lo, 0.3 * lo + 0.7 * hi, hi])
        S, Z = orc.minmax_affine(w, bits)
        assert S == pytest.approx((hi - lo) / (2 ** bits - 1), rel=1e-15)
        grid = np.linspace(lo, hi, 2 ** bits)
        q, code = orc.quant_aff(grid, S, Z, bits)
        np.testing.assert_allclose(q, grid, atol=1e-14)
        np.testing.assert_array_equal(code, np.arange(2 ** bits))
        # everything lands on a grid point, out-of-range values on the end points
        q2, _ = orc.quant_aff(np.linspace(lo - 1, hi + 1, 501), S, Z, bits)
        assert np.all(np.min(np.abs(q2[:, None] - grid[None, :]), axis=1) < 1e-13)
    # The appendix's [-1, 1] example has min/S = -1.5: with the integer zero-point of
    # Section 2.1 the grid is shifted by half a step; the formula is followed, not the prose.
    S, Z = orc.minmax_affine(np.array([-1.0, 1.0]), 2)
    assert Z == 2.0
    np.testing.assert_allclose(orc.quant_aff(np.array([-9.0, 9.0]), S, Z, 2)[0], [-4 / 3, 2 / 3])


def test_quant_nu_is_nearest_point_bruteforce_and_ties_low():
    g = RNG(5)
    G = np.sort(g.standard_normal((3, 8)), axis=1)
    w = g.standard_normal((3, 50))
    q, idx = orc.quant_nu(w, G)
    for k in range(3):
        for i in range(50):
            best = min(range(8), key=lambda m: (abs(G[k, m] - w[k, i]), m))
            assert idx[k, i] == best and q[k, i] == G[k, best]
    qt, it = orc.quant_nu(np.array([[0.5]]), np.array([[0.0, 1.0]]))
    assert it[0, 0] == 0 and qt[0, 0] == 0.0


def test_quant_aff_rounding_and_clip():
    # round-half-to-even, then zero-point, then clip to [0, 2^b - 1]
    q, wi = orc.quant_aff(np.array([0.5, 1.5, 2.5, -7.0, 100.0]), 1.0, 2.0, 3)
    np.testing.assert_array_equal(wi, [2, 4, 4, 0, 7])
    np.testing.assert_array_equal(q, [0, 2, 2, -2, 5])


# ------------------------------------------------------------------ step 3, non-uniform
def _plain_lloyd(points, init, iters):
    """Unweighted Lloyd written separately (lists, no numpy broadcasting)."""
    cent = list(init)
    for _ in range(iters):
        sums = [0.0] * len(cent)
        cnts = [0] * len(cent)
        for x in points:
            m = min(range(len(cent)), key=lambda k: (abs(cent[k] - x), k))
            sums[m] += x
            cnts[m] += 1
        new = [sums[k] / cnts[k] if cnts[k] else cent[k] for k in range(len(cent))]
        if new == cent:
            break
        cent = new
    return cent


def test_p0_reduces_to_plain_kmeans():
    """p = 0 makes every importance weight 1 (Section 3.2.1): plain Lloyd, any H."""
    g = RNG(6)
    W = g.standard_normal((4, 200)) * 0.02
    d = np.exp(g.standard_normal(200))                 # arbitrary inverse diagonal
    G = orc.fit_grid_nu(W, d, 3, 0.0, max_iter=500)
    for k in range(4):
        init = orc.uniform_init(W[k:k + 1], 3)[0]
        ref = _plain_lloyd(list(W[k]), list(init), 500)
        np.testing.assert_allclose(G[k], ref, rtol=1e-11, atol=1e-15)
    # library cross-check where no cluster empties (kmeans2 handles those differently)
    Wd = np.sort(g.uniform(-1, 1, (1, 400)))
    Gd = orc.fit_grid_nu(Wd, np.ones(400), 2, 0.0, max_iter=500)
    cent, _ = kmeans2(Wd[0][:, None], orc.uniform_init(Wd, 2)[0][:, None], iter=500, minit="matrix")
    np.testing.assert_allclose(Gd[0], cent[:, 0], rtol=1e-9)


def test_identity_hessian_p0_is_plain_kmeans_end_to_end():
    """H = I, p = 0: the non-uniform grid is plain per-row k-means of W."""
    g = RNG(7)
    W = g.standard_normal((3, 64))
    out = orc.leanquant_layer(W, np.eye(64), "nu", 2, df=0.01, p=0.0, B=16)
    for k in range(3):
        ref = _plain_lloyd(list(W[k]), list(orc.uniform_init(W[k:k + 1], 2)[0]), 1000)
        np.testing.assert_allclose(out["grid"][k], ref, rtol=1e-11)


def test_weighted_kmeans_equals_point_replication():
    """Integer importance weights m_i == the point repeated m_i times, unweighted."""
    g = RNG(8)
    c = 60
    w = g.standard_normal(c)
    m = g.integers(1, 6, c)
    # importance() gives (d/min d)^-p; choose d so that omega = m exactly for p = 1
    d = (1.0 / m) * 1.0
    om = orc.importance(d, 1.0)
    scale = om[0] / m[0]
    np.testing.assert_allclose(om, m * scale, rtol=1e-14)
    init = orc.uniform_init(w[None, :], 3)
    G = orc.fit_grid_nu(w[None, :], d, 3, 1.0, max_iter=300)
    rep = np.repeat(w, m)
    ref = _plain_lloyd(list(rep), list(init[0]), 300)
    np.testing.assert_allclose(G[0], ref, rtol=1e-10, atol=1e-14)


def test_lloyd_monotone_sorted_bounded():
    """Eq. 5 objective never increases; centroids stay ascending and inside [min, max]."""
    g = RNG(9)
    W = g.standard_normal((6, 300)) * 0.02
    W[g.random((6, 300)) < 0.02] *= 12.0
    d = np.exp(2.0 * g.standard_normal(300))
    hist = []
    G = orc.fit_grid_nu(W, d, 4, 4.0, max_iter=60, history=hist)
    H = np.array(hist)                      # iterations x rows
    assert np.all(np.diff(H, axis=0) <= 1e-12 * np.abs(H[:-1]) + 1e-300)
    assert np.all(np.diff(G, axis=1) >= 0)
    assert np.all(G.min(1) >= W.min(1) - 1e-15) and np.all(G.max(1) <= W.max(1) + 1e-15)
    om = orc.importance(d, 4.0)
    assert np.all(orc.eq5_objective(W, om, G) <= orc.eq5_objective(W, om, orc.uniform_init(W, 4)))


def test_fixed_point_is_idempotent_and_cap_counts_updates():
    g = RNG(10)
    W = g.standard_normal((2, 120))
    d = np.ones(120)
    G = orc.fit_grid_nu(W, d, 2, 2.0, max_iter=500)
    G2, _ = orc.lloyd_step(W, orc.importance(d, 2.0)[None, :], G)
    np.testing.assert_array_equal(G, G2)
    # max_iter = 1 is exactly one update of the uniform grid
    G1 = orc.fit_grid_nu(W, d, 2, 2.0, max_iter=1)
    ref, _ = orc.lloyd_step(W, orc.importance(d, 2.0)[None, :], orc.uniform_init(W, 2))
    np.testing.assert_array_equal(G1, ref)


def test_empty_cluster_keeps_its_point():
    w = np.array([[0.0, 0.01, 0.02, 10.0]])
    G = orc.fit_grid_nu(w, np.ones(4), 2, 0.0)
    # uniform init 0, 3.33, 6.67, 10: the two middle clusters are empty and stay put
    np.testing.assert_allclose(G[0], [0.01, 10.0 / 3, 20.0 / 3, 10.0], rtol=1e-12)


def test_tr_loss_monotone_for_diagonal_hessian_p1():
    """Diagonal H and p = 1: omega_i is proportional to H_ii + lambda, there is no
    propagation, and the layer loss with the damped H equals the Eq. 5 objective
    summed over rows, so it cannot increase from one Lloyd iteration to the next."""
    g = RNG(11)
    c, r = 40, 5
    h = np.exp(g.standard_normal(c))
    H = np.diag(h)
    U, d = orc.cholesky_inv(H, 0.01)
    Hd = orc.dampen(H, 0.01)
    W = g.standard_normal((r, c))
    prev = np.inf
    for it in range(1, 12):
        G = orc.fit_grid_nu(W, d, 2, 1.0, max_iter=it)
        What, _, row_loss = orc.quantize_layer(W, U, G, "nu", 2, B=8)
        loss = orc.layer_loss(W, What, Hd)
        assert loss <= prev * (1 + 1e-12)
        assert loss == pytest.approx(2.0 * row_loss.sum(), rel=1e-10)
        prev = loss


# ------------------------------------------------------------------ step 3, affine
def test_eq5_objective_hand_computed():
    """Eq. 5 by hand: three weights, two grid points, distinct importance weights.
    row 0: w = (0.1, 0.4, 0.9), G = (0, 1): nearest points (0, 0, 1), errors (0.1, 0.4, 0.1),
           omega = (1, 2, 3) -> 1 * 0.01 + 2 * 0.16 + 3 * 0.01 = 0.36
    row 1: w = (-1, 0.6, 0.5), G = (-1, 0.5): errors (0, 0.1, 0) -> 2 * 0.01 = 0.02
    (dropping omega would give 0.18 and 0.01; squaring omega 0.92 and 0.04)."""
    w = np.array([[0.1, 0.4, 0.9], [-1.0, 0.6, 0.5]])
    G = np.array([[0.0, 1.0], [-1.0, 0.5]])
    om = np.array([1.0, 2.0, 3.0])
    np.testing.assert_allclose(orc.eq5_objective(w, om, G), [0.36, 0.02], rtol=1e-12)
    # one row alone, and a weight exactly on a midpoint (either neighbour: same distance)
    np.testing.assert_allclose(orc.eq5_objective(w[0], om, G[0]), 0.36, rtol=1e-12)
    np.testing.assert_allclose(orc.eq5_objective(np.array([0.5]), np.array([7.0]), np.array([0.0, 1.0])), 1.75, rtol=1e-12)


def test_eq7_objective_hand_computed():
    """Eq. 7 by hand at b = 2 with S = 0.5, Z = 1, i.e. the grid (code - Z) S = (-0.5, 0, 0.5, 1):
    w = 0.3: round(0.6) + 1 = 2 -> 0.5, error 0.2;  w = -0.9: round(-1.8) + 1 = -1 -> clipped to
    0 -> -0.5, error 0.4;  w = 1.4: round(2.8) + 1 = 4 -> clipped to 3 -> 1.0, error 0.4;
    omega = (2, 1, 4) -> 2 * 0.04 + 1 * 0.16 + 4 * 0.16 = 0.88 (0.36 without omega; 0.24 without
    the clipping, whose grid would reach -1 and 1.5)."""
    w = np.array([0.3, -0.9, 1.4])
    om = np.array([2.0, 1.0, 4.0])
    assert orc.eq7_objective(w, om, 0.5, 1.0, 2) == pytest.approx(0.88, rel=1e-12)
    # a grid that contains every weight scores zero; scaling omega scales the objective
    assert orc.eq7_objective(np.array([-0.5, 0.0, 1.0]), om, 0.5, 1.0, 2) == 0.0
    assert orc.eq7_objective(w, 3.0 * om, 0.5, 1.0, 2) == pytest.approx(2.64, rel=1e-12)


def test_t0_is_minmax_grid():
    """No shrinkage (t = 0) leaves the min-max S and Z of Section 2.1."""
    g = RNG(12)
    W = g.standard_normal((3, 32))
    d = np.exp(g.standard_normal(32))
    SZ = orc.fit_grid_aff(W, d, 4, 4.0, group_size=16, T=2048, t=0)
    for k in range(3):
        for gi in range(2):
            S, Z = orc.minmax_affine(W[k, gi * 16:(gi + 1) * 16], 4)
            assert SZ[k, gi, 0] == pytest.approx(S, rel=1e-14) and SZ[k, gi, 1] == Z


def test_shrink_steps_eq8():
    assert [orc.shrink_steps(b, 2048) for b in (4, 3, 2)] == [409, 614, 819]
    assert [orc.shrink_steps(b, 10) for b in (4, 3, 2)] == [2, 3, 4]


def test_affine_search_bruteforce_small():
    """Eq. 7 enumerated in a separately written triple loop with scalar arithmetic."""
    g = RNG(13)
    bits, T, t = 2, 8, 3
    for trial in range(6):
        w = g.standard_normal(6)
        om = np.exp(3 * g.standard_normal(6))
        S, Z, loss, tmin, tmax = orc.fit_group_aff(w, om, bits, T, t)
        R = max(w) - min(w)
        best = None
        for a, b in itertools.product(range(t + 1), range(t + 1)):
            lo = min(w) + a * R / T
            hi = max(w) - b * R / T
            s = (hi - lo) / (2 ** bits - 1)
            z = -round(lo / s)          # python round() is half-to-even too
            tot = 0.0
            for wi, oi in zip(w, om):
                code = min(max(round(wi / s) + z, 0), 2 ** bits - 1)
                tot += oi * ((code - z) * s - wi) ** 2
            if best is None or tot < best[0]:
                best = (tot, a, b, s, z)
        assert (tmin, tmax) == (best[1], best[2])
        assert S == pytest.approx(best[3], rel=1e-13) and Z == best[4]
        assert loss == pytest.approx(best[0], rel=1e-12)
        # (0, 0) is a candidate: never worse than the min-max grid
        S0, Z0 = orc.minmax_affine(w, bits)
        assert loss <= orc.eq7_objective(w, om, S0, Z0, bits) * (1 + 1e-12)


def test_affine_grouping_uses_group_columns_only():
    g = RNG(14)
    W = g.standard_normal((2, 24))
    d = np.exp(g.standard_normal(24))
    SZ = orc.fit_grid_aff(W, d, 3, 4.0, group_size=8, T=16, t=4)
    om = orc.importance(d, 4.0)
    for gi in range(3):
        S, Z, *_ = orc.fit_group_aff(W[1, gi * 8:(gi + 1) * 8], om[gi * 8:(gi + 1) * 8], 3, 16, 4)
        assert (SZ[1, gi, 0], SZ[1, gi, 1]) == (S, Z)
    assert orc.fit_grid_aff(np.full((1, 8), 0.3), np.ones(8), 3, 4.0, T=16)[0, 0].tolist() == [1.0, 0.0]


# ------------------------------------------------------------------ step 4
def _fixed_grid(r, K, seed):
    return np.sort(RNG(seed).standard_normal((r, K)) * 0.8, axis=1)


@pytest.mark.parametrize("c", [1, 2, 5, 6])
def test_loop_equals_exhaustive_obs(c):
    """Tiny layers: Algorithm 1's loop with the Cholesky factor reproduces the
    per-column OBS update (Eq. 3) with the explicit inverse downdated by Eq. 9."""
    X = _spd_case(c, 30, 20 + c, outliers=1)
    H = orc.hessian(X)
    U, _ = orc.cholesky_inv(H, 0.01)
    Hd = orc.dampen(H, 0.01)
    W = RNG(30 + c).standard_normal((4, c))
    G = _fixed_grid(4, 4, 40 + c)
    What, codes, row_loss = orc.quantize_layer(W, U, G, "nu", 2, B=3)
    ref, eps = orc.obs_fixed_order(W, Hd, lambda j, col: orc.quant_nu(col[:, None], G)[0][:, 0])
    np.testing.assert_allclose(What, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(row_loss, eps, rtol=1e-9)
    # affine flavour
    SZ = np.stack([np.full((4, 1), 0.37), np.full((4, 1), 3.0)], axis=-1)
    Wa, _, la = orc.quantize_layer(W, U, SZ, "aff", 3, B=2)
    refa, epsa = orc.obs_fixed_order(W, Hd, lambda j, col: orc.quant_aff(col, 0.37, 3.0, 3)[0])
    np.testing.assert_allclose(Wa, refa, atol=1e-12)
    np.testing.assert_allclose(la, epsa, rtol=1e-9)


def test_block_size_invariance():
    """Lazy batching only re-associates the updates (Section 2.2): any B, same result."""
    c, r = 37, 6
    X = _spd_case(c, 150, 50)
    U, _ = orc.cholesky_inv(orc.hessian(X), 0.01)
    W = RNG(51).standard_normal((r, c))
    G = _fixed_grid(r, 8, 52)
    base = orc.quantize_layer(W, U, G, "nu", 3, B=1)
    for B in (2, 16, 128, c):
        out = orc.quantize_layer(W, U, G, "nu", 3, B=B)
        np.testing.assert_array_equal(out[1], base[1])
        np.testing.assert_allclose(out[0], base[0], atol=1e-13)
        np.testing.assert_allclose(out[2], base[2], rtol=1e-11)


def test_energy_identity():
    """Per row: sum_j E_kj^2 = (w - w_hat)(H + lambda I)(w - w_hat)^T, i.e. the summed
    loss errors of Eq. 3 equal half the damped layer loss of that row."""
    c, r = 29, 5
    X = _spd_case(c, 100, 60)
    H = orc.hessian(X)
    U, _ = orc.cholesky_inv(H, 0.01)
    Hd = orc.dampen(H, 0.01)
    W = RNG(61).standard_normal((r, c))
    What, _, row_loss = orc.quantize_layer(W, U, _fixed_grid(r, 4, 62), "nu", 2, B=8)
    D = W - What
    np.testing.assert_allclose(2.0 * row_loss, np.einsum("ki,ij,kj->k", D, Hd, D), rtol=1e-9)


def test_diagonal_hessian_no_propagation():
    c, r = 16, 4
    H = np.diag(np.exp(RNG(70).standard_normal(c)))
    U, _ = orc.cholesky_inv(H, 0.01)
    W = RNG(71).standard_normal((r, c))
    G = _fixed_grid(r, 4, 72)
    What, codes, _ = orc.quantize_layer(W, U, G, "nu", 2, B=4)
    q, idx = orc.quant_nu(W, G)
    np.testing.assert_array_equal(What, q)
    np.testing.assert_array_equal(codes, idx)


def test_identity_hessian_t0_is_minmax_rtn():
    """H = I, t = 0: affine mode is the min-max grid plus round-to-nearest."""
    W = RNG(73).standard_normal((3, 32))
    out = orc.leanquant_layer(W, np.eye(32), "aff", 4, p=0.0, B=8, group_size=16, t=0)
    for k in range(3):
        for gi in range(2):
            sl = slice(gi * 16, (gi + 1) * 16)
            S, Z = orc.minmax_affine(W[k, sl], 4)
            q, wi = orc.quant_aff(W[k, sl], S, Z, 4)
            np.testing.assert_array_equal(out["W_hat"][k, sl], q)
            np.testing.assert_array_equal(out["codes"][k, sl], wi)


def test_propagation_lowers_loss_vs_rtn_on_same_grid():
    """The compensated result can not be worse than plain rounding in expectation;
    on this fixed seeded case it is strictly better (guards a flipped update sign)."""
    c, r = 48, 16
    X = _spd_case(c, 80, 80, outliers=4)
    X[:, 1:] += 0.9 * X[:, :-1]                 # correlated channels
    H = orc.hessian(X)
    U, d = orc.cholesky_inv(H, 0.01)
    W = RNG(81).standard_normal((r, c)) * 0.05
    G = orc.fit_grid_nu(W, d, 3, 4.0)
    What, _, _ = orc.quantize_layer(W, U, G, "nu", 3, B=16)
    rtn, _ = orc.quant_nu(W, G)
    assert orc.layer_loss(W, What, H) < 0.9 * orc.layer_loss(W, rtn, H)


# ------------------------------------------------------------------ whole pass
def test_invariances_of_whole_pass():
    c, r = 32, 8
    X = _spd_case(c, 120, 90, outliers=3)
    H = orc.hessian(X)
    W = RNG(91).standard_normal((r, c)) * 0.02
    base = orc.leanquant_layer(W, H, "nu", 3, B=8)
    # scaling H changes neither codes nor grid
    sc = orc.leanquant_layer(W, 37.5 * H, "nu", 3, B=8)
    np.testing.assert_array_equal(sc["codes"], base["codes"])
    np.testing.assert_allclose(sc["grid"], base["grid"], rtol=1e-9)
    # scaling W scales the grid, same codes
    sw = orc.leanquant_layer(4.0 * W, H, "nu", 3, B=8)
    np.testing.assert_array_equal(sw["codes"], base["codes"])
    np.testing.assert_allclose(sw["grid"], 4.0 * base["grid"], rtol=1e-12)
    # rows are independent: a row alone gives what it gives in the batch (Eq. 1)
    perm = np.array([5, 2, 7])
    sub = orc.leanquant_layer(W[perm], H, "nu", 3, B=8)
    np.testing.assert_array_equal(sub["codes"], base["codes"][perm])
    np.testing.assert_allclose(sub["W_hat"], base["W_hat"][perm], rtol=1e-12)
    # affine mode, same checks on codes
    ba = orc.leanquant_layer(W, H, "aff", 3, B=8, group_size=16, T=32)
    sa = orc.leanquant_layer(W, 0.01 * H, "aff", 3, B=8, group_size=16, T=32)
    np.testing.assert_array_equal(sa["codes"], ba["codes"])


# ------------------------------------------------------------------ k-means++ seeding
def test_kmeanspp_hand_computed_draws():
    # w = [0, 1, 3], equal masses.  u0 = 0.5: cumulative masses [1, 2, 3], target 1.5 -> index 1
    # (w = 1).  Then D^2 = [1, 0, 4], cumulative [1, 1, 5], u1 = 0.5 -> target 2.5 -> index 2.
    G = orc.kmeanspp_init(np.array([[0.0, 1.0, 3.0]]), np.ones(3), 1, 1.0, np.array([[0.5, 0.5]]))
    assert G.tolist() == [[1.0, 3.0]]
    # u1 = 0.1 -> target 0.5 -> index 0 (w = 0)
    G = orc.kmeanspp_init(np.array([[0.0, 1.0, 3.0]]), np.ones(3), 1, 1.0, np.array([[0.5, 0.1]]))
    assert G.tolist() == [[0.0, 1.0]]


def test_kmeanspp_centres_are_distinct_points_of_the_row_and_follow_the_masses():
    rng = np.random.default_rng(11)
    W = rng.standard_normal((40, 64))
    d = np.exp(rng.standard_normal(64))
    G = orc.kmeanspp_init(W, d, 3, 4.0, rng.random((40, 8)))
    for k in range(40):
        assert np.all(np.isin(G[k], W[k]))
        assert len(np.unique(G[k])) == 8            # a chosen point has D^2 = 0 afterwards
        assert np.all(np.diff(G[k]) > 0)
    # first centre: frequency of column i over many draws is proportional to omega_i
    om = orc.importance(np.array([1.0, 2.0 ** -0.25, 1.0]), 4.0)      # masses 1 : 2 : 1 -> scaled
    w = np.array([[-1.0, 0.0, 1.0]])
    picks = [orc.kmeanspp_init(w, np.array([1.0, 2.0 ** -0.25, 1.0]), 0, 4.0, np.array([[u]]))[0, 0]
             for u in (np.arange(1000) + 0.5) / 1000]
    share = np.mean(np.array(picks) == 0.0)
    assert abs(share - om[1] / om.sum()) < 2e-3


def test_lloyd_from_kmeanspp_init_does_not_increase_the_objective():
    rng = np.random.default_rng(12)
    W = rng.standard_normal((6, 200)) * 0.02
    d = np.exp(rng.standard_normal(200))
    init = orc.kmeanspp_init(W, d, 3, 4.0, rng.random((6, 8)))
    hist = []
    G = orc.fit_grid_nu(W, d, 3, 4.0, init=init, history=hist)
    H = np.array(hist)
    assert np.all(np.diff(H, axis=0) <= 1e-18 + 1e-12 * H[:-1])
    assert np.all(np.diff(G, axis=1) >= 0)


# ------------------------------------------------------------------ LeanQuant-Exact (Algorithm 2)
def _exact_case(c, n, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, c)) * (1.0 + 3.0 * (rng.random(c) < 0.2))
    H = orc.hessian(X)
    w = rng.standard_normal(c) * 0.05
    return w, H


def test_exact_greedy_choice_and_downdate_against_submatrix_inverses():
    """At every step the running inverse equals the inverse of the damped Hessian restricted
    to the weights not yet quantized (what Eq. 9 maintains), and the chosen weight is the
    brute-force argmin of Eq. 3 computed from that submatrix inverse."""
    w0, H = _exact_case(6, 40, 21)
    Hd = orc.dampen(H, 0.01)
    G = np.linspace(-0.1, 0.1, 4)
    quant = lambda v: orc.quant_nu(v, G)
    w_hat, codes, order, eps = orc.exact_row(w0, np.linalg.inv(Hd), quant)
    # replay with explicit submatrix inverses
    w = w0.copy()
    live = list(range(6))
    tot = 0.0
    for step in range(6):
        sub = np.linalg.inv(Hd[np.ix_(live, live)])
        q, _ = quant(w[live])
        score = (q - w[live]) ** 2 / (2.0 * np.diag(sub))
        j = int(np.argmin(score))
        assert live[j] == order[step]
        tot += score[j]
        delta = -(w[live][j] - q[j]) / sub[j, j] * sub[:, j]
        for a, idx in enumerate(live):
            w[idx] += delta[a]
        assert abs(w[live[j]] - q[j]) < 1e-12
        assert abs(w_hat[live[j]] - q[j]) < 1e-12
        live.pop(j)
    assert abs(tot - eps) <= 1e-10 * max(eps, 1e-30)


def test_exact_energy_identity_and_grid_membership():
    w0, H = _exact_case(24, 200, 22)
    Hd = orc.dampen(H, 0.01)
    G = np.sort(np.random.default_rng(3).standard_normal(8) * 0.05)
    w_hat, codes, order, eps = orc.exact_row(w0, np.linalg.inv(Hd), lambda v: orc.quant_nu(v, G))
    assert sorted(order.tolist()) == list(range(24))
    assert np.array_equal(w_hat, G[codes])
    dlt = w0 - w_hat
    assert abs(eps - 0.5 * dlt @ Hd @ dlt) <= 1e-9 * eps      # OBS steps are H_d-conjugate


def test_exact_with_diagonal_hessian_is_round_to_nearest():
    rng = np.random.default_rng(23)
    w0 = rng.standard_normal(16) * 0.05
    Hinv = np.diag(1.0 / (1.0 + rng.random(16)))
    w_hat, codes, order, eps = orc.exact_row(w0, Hinv, lambda v: orc.quant_aff(v, 0.01, 3.0, 3))
    q, wi = orc.quant_aff(w0, 0.01, 3.0, 3)
    assert np.array_equal(w_hat, q) and np.array_equal(codes, wi.astype(np.int64))
    # the order is by increasing loss error of the untouched weights
    score = (q - w0) ** 2 / (2.0 * np.diag(Hinv))
    assert np.array_equal(order, np.argsort(score, kind="stable"))


def test_exact_layer_wrapper_uses_damped_inverse_and_original_grid():
    rng = np.random.default_rng(24)
    X = rng.standard_normal((300, 20))
    W = rng.standard_normal((3, 20)) * 0.05
    H = orc.hessian(X)
    out = orc.leanquant_exact(W, H, "nu", 2)
    assert np.allclose(out["Hinv"] @ orc.dampen(H, 0.01), np.eye(20), atol=1e-9)
    assert np.array_equal(out["grid"], orc.fit_grid_nu(W, out["d"], 2, 4.0))
    for k in range(3):
        assert np.array_equal(out["W_hat"][k], out["grid"][k][out["codes"][k]])
    # never worse than fixed-order OBS on the same grid?  Not guaranteed; only report the ratio
    # of the summed loss errors so that a gross mistake (eps orders of magnitude off) shows
    _, eps_fixed = orc.obs_fixed_order(W, orc.dampen(H, 0.01),
                                       lambda j, col: orc.quant_nu(col[:, None], out["grid"])[0][:, 0])
    assert np.all(out["eps"] < 10 * eps_fixed) and np.all(eps_fixed < 10 * out["eps"])
