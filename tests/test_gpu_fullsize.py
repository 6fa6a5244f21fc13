"""The large benchmark layers (configurations 3, 4 and 5, the latter with both grid kinds) at
their FULL sizes, calibration tokens accumulated in chunks.

The float64 oracle cannot run this end to end in minutes, so the checks are
  * properties that hold at any size, over every row: W_hat is exactly grid[row][code],
    grids ascend, the per-row loss is the energy identity 1/2 (w - w_hat) H_d (w - w_hat)^T
    (sampled rows, float64 on the host);
  * the Gram matrix against the oracle on sampled 128 x 128 tiles, and U^T U H_d = I on
    sampled columns;
  * stage-isolated parity on a seeded sample of rows: the oracle's grid fit and column loop
    run from the device's d and U (upcast), which is exact for those rows because rows are
    independent problems (Eq. 1).
"""
import time

import numpy as np
import pytest

import lq_synth
from oracle import leanquant_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2407_10032_amd as lq
    from tests import lq_harness as hx


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("name", ["c5nu", "c3"])
def test_non_uniform_configurations_at_full_size(name):
    """c5nu: 53248 x 16384 weights, 65536 tokens, 3 bits; c3: 4096 x 11008 weights, 262144
    tokens of the gated-activation kind, 3 bits."""
    cfg = lq_synth.CONFIGS[name]
    P = hx.params_for(cfg)
    r, c, n = cfg.r, cfg.c, cfg.n_tokens
    t0 = time.time()
    _say(f"{name} full size: W {r} x {c}, X {n} x {c}")

    # ---- stage A in chunks; oracle Gram on sampled tiles
    H = torch.zeros((c, c), dtype=torch.float32, device="cuda")
    ws = lq.alloc_workspace(lq.lq_workspace_bytes(lq.LQ_CALL_HESSIAN, 0, c, lq_synth.TOKEN_CHUNK))
    rng = np.random.default_rng(5150)
    tiles = [(int(a), int(b)) for a, b in rng.integers(0, c // 128, size=(6, 2))] + [(3, 3), (c // 128 - 1, c // 128 - 1)]
    ref_tiles = [np.zeros((128, 128)) for _ in tiles]
    for k in range(lq_synth.n_token_chunks(cfg)):
        xc = lq_synth.activation_chunk(cfg, k)
        lq.lq_hessian_accumulate(H, torch.from_numpy(xc).cuda(), ws)
        for ti, (a, b) in enumerate(tiles):
            xa = xc[:, a * 128:(a + 1) * 128].astype(np.float64)
            xb = xc[:, b * 128:(b + 1) * 128].astype(np.float64)
            ref_tiles[ti] += 2.0 * xa.T @ xb
    torch.cuda.synchronize()
    _say(f"  Gram accumulated in {lq_synth.n_token_chunks(cfg)} calls ({time.time() - t0:.0f} s)")
    Hd = torch.diagonal(H).double().cpu().numpy()
    for (a, b), ref in zip(tiles, ref_tiles):
        got = H[a * 128:(a + 1) * 128, b * 128:(b + 1) * 128].double().cpu().numpy()
        sc = np.sqrt(np.outer(Hd[a * 128:(a + 1) * 128], Hd[b * 128:(b + 1) * 128]))
        assert np.max(np.abs(got - ref) / sc) < 2e-6 * np.sqrt(n)
        gotT = H[b * 128:(b + 1) * 128, a * 128:(a + 1) * 128].double().cpu().numpy()
        assert np.array_equal(gotT.T, got)                      # both triangles are kept equal

    # ---- stage B; U^T U H_d = I on sampled columns (float64 on the host)
    U, d, info = hx.gpu_cholesky(H, P.damp)
    assert info == 0
    lam = P.damp * Hd.mean()
    cols = rng.integers(0, c, size=4)
    Ucpu = U.cpu().numpy()
    Hcpu = H.cpu().numpy()
    for j in cols:
        hj = Hcpu[:, j].astype(np.float64)
        hj[j] += lam
        y = np.zeros(c)
        # U is upper triangular: do the two products in row blocks to bound host memory
        uh = np.zeros(c)
        for s0 in range(0, c, 2048):
            uh[s0:s0 + 2048] = Ucpu[s0:s0 + 2048].astype(np.float64) @ hj
        for s0 in range(0, c, 2048):
            y += Ucpu[s0:s0 + 2048].astype(np.float64).T @ uh[s0:s0 + 2048]
        y[j] -= 1.0
        assert np.max(np.abs(y)) < 5e-4, (j, np.max(np.abs(y)))
    dcpu = d.cpu().numpy()
    _say(f"  U, d done ({time.time() - t0:.0f} s)")

    # ---- stages C, D on every row
    W = torch.from_numpy(lq_synth.weights(cfg)).cuda()
    grid = hx.gpu_fit_grid(W, d, P)
    What, codes, row_loss = hx.gpu_quantize(W, U, grid, P)
    assert bool(torch.all(grid[:, 1:] >= grid[:, :-1]))
    assert bool(torch.all(codes < (1 << cfg.bits)))
    assert torch.equal(What, torch.gather(grid, 1, codes.long()))
    assert bool(torch.all(torch.isfinite(row_loss))) and bool(torch.all(row_loss >= 0))
    _say(f"  fit + loop on all rows done ({time.time() - t0:.0f} s)")

    # ---- sampled rows against the oracle, from the device's d and U
    rows = np.sort(rng.choice(r, size=16, replace=False))
    Wr = W[rows].cpu().numpy()
    U64 = Ucpu.astype(np.float64)
    Gref = orc.fit_grid_nu(Wr, dcpu, cfg.bits, cfg.p)
    Gg = grid[rows].cpu().numpy()
    ok = hx.nu_grid_match(Gg, Gref)
    What_ref, codes_ref, loss_ref = orc.quantize_layer(Wr, U64, Gref, "nu", cfg.bits, B=cfg.block)
    cg = codes[rows].cpu().numpy()
    # every sampled row: the oracle's grid, or an equally good one followed through the oracle's loop
    share, agree, redone = hx.compare_rows_strict("nu", cfg.bits, Wr, dcpu, U64, Gg, cg, Gref, codes_ref,
                                                  p=cfg.p, B=cfg.block, say=_say)
    _say(f"  sampled rows: grids matching {share:.3f}, codes equal over all {len(rows)} rows {agree:.5f} "
         f"({redone} re-run from the device's grid) ({time.time() - t0:.0f} s)")
    assert (~ok).sum() <= 1
    assert agree >= 0.999
    # energy identity for the device's own result (Eq. 3 summed over the row)
    Whr = What[rows].cpu().numpy().astype(np.float64)
    diff = Wr.astype(np.float64) - Whr
    e = np.zeros(len(rows))
    for s0 in range(0, c, 2048):
        blk = Hcpu[s0:s0 + 2048].astype(np.float64)
        blk[np.arange(blk.shape[0]), s0 + np.arange(blk.shape[0])] += lam
        e += np.einsum("kj,kj->k", diff[:, s0:s0 + 2048], diff @ blk.T)
    e *= 0.5
    rl = row_loss[rows].cpu().numpy()
    assert np.max(np.abs(rl - e) / e) < 2e-3, np.max(np.abs(rl - e) / e)
    # and the loss of the matching rows agrees with the oracle's
    assert np.max(np.abs(rl[ok] - loss_ref[ok]) / loss_ref[ok]) < 1e-3


def test_config4_affine_full_size():
    """Configuration 4 at its full size (28672 x 8192 weights, 131072 tokens, 4-bit affine,
    group 128, T = 2048): properties over every row and group, and the oracle's enumerative
    search and column loop on sampled rows from the device's d and U."""
    cfg = lq_synth.CONFIGS["c4"]
    P = hx.params_for(cfg)
    r, c, n = cfg.r, cfg.c, cfg.n_tokens
    g, ng = cfg.group_size, cfg.c // cfg.group_size
    qmax = float((1 << cfg.bits) - 1)
    t0 = time.time()
    _say(f"c4 full size: W {r} x {c}, X {n} x {c}")
    H = torch.zeros((c, c), dtype=torch.float32, device="cuda")
    ws = lq.alloc_workspace(lq.lq_workspace_bytes(lq.LQ_CALL_HESSIAN, 0, c, 2 * lq_synth.TOKEN_CHUNK))
    nchunks = lq_synth.n_token_chunks(cfg)
    for k in range(0, nchunks, 2):                      # two generator chunks (16384 tokens) per call
        xc = np.concatenate([lq_synth.activation_chunk(cfg, k), lq_synth.activation_chunk(cfg, k + 1)])
        lq.lq_hessian_accumulate(H, torch.from_numpy(xc).cuda(), ws)
    torch.cuda.synchronize()
    _say(f"  Gram accumulated in {nchunks // 2} calls ({time.time() - t0:.0f} s)")
    U, d, info = hx.gpu_cholesky(H, P.damp)
    assert info == 0
    W = torch.from_numpy(lq_synth.weights(cfg)).cuda()
    SZ = hx.gpu_fit_grid(W, d, P)
    What, codes, row_loss = hx.gpu_quantize(W, U, SZ, P)
    _say(f"  fit + loop on all rows done ({time.time() - t0:.0f} s)")
    # properties over everything: positive scales, integer zero-points, codes in range, and
    # W_hat = (code - Z) S with the group's pair (Section 2.1), exactly as the kernel forms it
    S = SZ[..., 0].repeat_interleave(g, dim=1)
    Z = SZ[..., 1].repeat_interleave(g, dim=1)
    assert bool(torch.all(SZ[..., 0] > 0)) and bool(torch.all(SZ[..., 1] == torch.round(SZ[..., 1])))
    assert bool(torch.all(codes <= int(qmax)))
    assert torch.equal(What, (codes.float() - Z) * S)
    assert bool(torch.all(torch.isfinite(row_loss))) and bool(torch.all(row_loss >= 0))
    # the search can only improve on the plain min-max grid of the same group (candidate (0, 0))
    rng = np.random.default_rng(4242)
    rows = np.sort(rng.choice(r, size=8, replace=False))
    Wr = W[rows].cpu().numpy()
    dcpu = d.cpu().numpy()
    t1 = time.time()
    SZref = orc.fit_grid_aff(Wr, dcpu, cfg.bits, cfg.p, group_size=g, T=cfg.T)
    _say(f"  oracle affine search on {rows.size} rows: {time.time() - t1:.0f} s")
    SZg = SZ[rows].cpu().numpy()
    ok = hx.aff_grid_match(SZg, SZref)
    U64 = U.cpu().numpy().astype(np.float64)
    _, codes_ref, loss_ref = orc.quantize_layer(Wr, U64, SZref, "aff", cfg.bits, group_size=g, B=cfg.block)
    # every sampled row: groups with another (S, Z) must score within 1e-5 (Eq. 7, float64), and such a
    # row is compared with the oracle's column loop run from the device's grids
    share, agree, redone = hx.compare_rows_strict("aff", cfg.bits, Wr, dcpu, U64, SZg, codes[rows].cpu().numpy(),
                                                  SZref, codes_ref, p=cfg.p, group_size=g, B=cfg.block, say=_say)
    _say(f"  sampled groups identical: {share:.4f}; codes equal over all {rows.size} rows {agree:.5f} "
         f"({redone} re-run from the device's grids) ({time.time() - t0:.0f} s)")
    assert share >= 0.99
    assert agree >= 0.999
    row_ok = ok.all(axis=1)
    if row_ok.any():
        rl = row_loss[rows].cpu().numpy()[row_ok]
        assert np.max(np.abs(rl - loss_ref[row_ok]) / loss_ref[row_ok]) < 1e-3


def test_config5_affine_full_size():
    """Configuration 5 with 2-bit affine grids of 64 columns (13.6 M groups, t = 0.4 T) at its
    full size.  The oracle's enumeration takes a quarter of a second per group, so stage C is
    checked on sampled groups and stage D on sampled rows from the device's own grids (rows
    and groups are independent problems)."""
    cfg = lq_synth.CONFIGS["c5"]
    P = hx.params_for(cfg)
    r, c, n = cfg.r, cfg.c, cfg.n_tokens
    g = cfg.group_size
    qmax = float((1 << cfg.bits) - 1)
    t0 = time.time()
    _say(f"c5 affine full size: W {r} x {c}, X {n} x {c}, groups of {g}")
    H = torch.zeros((c, c), dtype=torch.float32, device="cuda")
    ws = lq.alloc_workspace(lq.lq_workspace_bytes(lq.LQ_CALL_HESSIAN, 0, c, lq_synth.TOKEN_CHUNK))
    for k in range(lq_synth.n_token_chunks(cfg)):
        lq.lq_hessian_accumulate(H, torch.from_numpy(lq_synth.activation_chunk(cfg, k)).cuda(), ws)
    U, d, info = hx.gpu_cholesky(H, P.damp)
    assert info == 0
    del H
    _say(f"  H, U, d done ({time.time() - t0:.0f} s)")
    W = torch.from_numpy(lq_synth.weights(cfg)).cuda()
    SZ = hx.gpu_fit_grid(W, d, P)
    What, codes, row_loss = hx.gpu_quantize(W, U, SZ, P)
    _say(f"  fit + loop on all rows done ({time.time() - t0:.0f} s)")
    assert bool(torch.all(SZ[..., 0] > 0)) and bool(torch.all(SZ[..., 1] == torch.round(SZ[..., 1])))
    assert bool(torch.all(codes <= int(qmax)))
    for s0 in range(0, r, 8192):                        # W_hat = (code - Z) S, in row slabs
        sl = slice(s0, min(r, s0 + 8192))
        S = SZ[sl, :, 0].repeat_interleave(g, dim=1)
        Z = SZ[sl, :, 1].repeat_interleave(g, dim=1)
        assert torch.equal(What[sl], (codes[sl].float() - Z) * S)
    assert bool(torch.all(torch.isfinite(row_loss))) and bool(torch.all(row_loss >= 0))
    # stage C: sampled groups against the enumeration
    rng = np.random.default_rng(5252)
    dcpu = d.cpu().numpy()
    om = orc.importance(dcpu, cfg.p)
    t_lim = orc.shrink_steps(cfg.bits, cfg.T)
    same = 0
    picks = [(int(rng.integers(r)), int(rng.integers(c // g))) for _ in range(64)]
    for k, gi in picks:
        sl = slice(gi * g, (gi + 1) * g)
        w = W[k, sl].cpu().numpy()
        S_ref, Z_ref, loss_ref, _, _ = orc.fit_group_aff(w, om[sl], cfg.bits, cfg.T, t_lim)
        S_g, Z_g = float(SZ[k, gi, 0]), float(SZ[k, gi, 1])
        if abs(S_g - S_ref) <= 1e-4 * abs(S_ref) and Z_g == Z_ref:
            same += 1
        else:
            got = orc.eq7_objective(w, om[sl], S_g, Z_g, cfg.bits)
            assert got <= loss_ref * (1 + 1e-5), (k, gi, got, loss_ref)
    _say(f"  sampled groups identical: {same} of {len(picks)} ({time.time() - t0:.0f} s)")
    assert same >= 0.9 * len(picks)
    # stage D: sampled rows, the oracle's column loop from the device's grids and U
    rows = np.sort(rng.choice(r, size=8, replace=False))
    U64 = U.cpu().numpy().astype(np.float64)
    _, codes_ref, loss_ref = orc.quantize_layer(W[rows].cpu().numpy(), U64, SZ[rows].cpu().numpy().astype(np.float64),
                                                "aff", cfg.bits, group_size=g, B=cfg.block)
    agree = hx.code_agreement(codes[rows].cpu().numpy(), codes_ref)
    _say(f"  codes equal on sampled rows: {agree:.5f} ({time.time() - t0:.0f} s)")
    assert agree >= 0.999
    rl = row_loss[rows].cpu().numpy()
    assert np.max(np.abs(rl - loss_ref) / loss_ref) < 1e-3
