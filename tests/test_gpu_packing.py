"""GPU parity of the stored form (lq_pack_layer / lq_unpack_layer) against the packing oracle,
and of a quantization pass shared by several projections with the same input."""
import numpy as np
import pytest

import lq_synth
from oracle import packing_oracle as po
from tests import lq_harness as hx

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _lq():
    import paper_2407_10032_amd as lq
    lq.load()
    return lq


def _pack_gpu(lq, codes, grid, P, pad=0):
    r, c = codes.shape
    rb = lq.lq_packed_row_bytes(c, P.bits)
    packed = torch.full((r, rb + pad), 0xEE, dtype=torch.uint8, device="cuda")[:, :rb] if pad else \
        torch.empty((r, rb), dtype=torch.uint8, device="cuda")
    table = torch.empty(grid.size, dtype=torch.int16, device="cuda")
    lq.lq_pack_layer(hx.to_dev(codes, torch.uint8), hx.to_dev(grid.astype(np.float32)), P, packed, table)
    torch.cuda.synchronize()
    return packed, table


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("r,c", [(1, 1), (3, 13), (5, 67), (64, 128), (37, 1000), (16, 4096)])
def test_pack_unpack_non_uniform_bit_exact(bits, r, c):
    lq = _lq()
    rng = np.random.default_rng(1000 * bits + r + c)
    K = 1 << bits
    codes = rng.integers(0, K, size=(r, c)).astype(np.uint8)
    grid = np.sort(rng.normal(0, 0.02, size=(r, K)), axis=1).astype(np.float32)
    P = lq.lq_params_default(bits=bits, mode=lq.LQ_GRID_NONUNIFORM)
    packed, table = _pack_gpu(lq, codes, grid, P, pad=3)
    exp_packed = po.pack_codes(codes, bits)
    exp_table = po.table_nu(grid)
    assert np.array_equal(packed.cpu().numpy(), exp_packed)
    assert np.array_equal(table.cpu().numpy().view(np.uint16).reshape(r, K), exp_table)
    W = torch.empty((r, c + 5), dtype=torch.float32, device="cuda")[:, :c]
    out_codes = torch.empty((r, c), dtype=torch.uint8, device="cuda")
    lq.lq_unpack_layer(packed, table, c, P, W, out_codes)
    torch.cuda.synchronize()
    assert np.array_equal(out_codes.cpu().numpy(), codes)
    assert np.array_equal(W.cpu().numpy(), po.dequantize(exp_packed, exp_table, c, bits, "nu"))


@pytest.mark.parametrize("bits,group", [(2, 64), (4, 128), (3, 0), (4, 8)])
@pytest.mark.parametrize("r,c", [(3, 128), (9, 1024)])
def test_pack_unpack_affine_bit_exact(bits, group, r, c):
    lq = _lq()
    rng = np.random.default_rng(77 * bits + group + r)
    g = group if group else c
    ng = c // g
    codes = rng.integers(0, 1 << bits, size=(r, c)).astype(np.uint8)
    S = np.abs(rng.normal(0.01, 0.003, size=(r, ng))) + 1e-4
    Z = rng.integers(-40, 40, size=(r, ng)).astype(np.float64)
    Z[0, 0] = 50000.0                                           # saturates to int16
    grid = np.stack([S, Z], axis=-1).astype(np.float32)
    P = lq.lq_params_default(bits=bits, mode=lq.LQ_GRID_AFFINE, group_size=group)
    packed, table = _pack_gpu(lq, codes, grid, P)
    exp_packed = po.pack_codes(codes, bits)
    exp_table = po.table_aff(grid)
    assert np.array_equal(packed.cpu().numpy(), exp_packed)
    assert np.array_equal(table.cpu().numpy().view(np.uint16).reshape(r, ng, 2), exp_table)
    W = torch.empty((r, c), dtype=torch.float32, device="cuda")
    lq.lq_unpack_layer(packed, table, c, P, W, None)
    torch.cuda.synchronize()
    assert np.array_equal(W.cpu().numpy(), po.dequantize(exp_packed, exp_table, c, bits, "aff", group))


def test_bits_per_weight_and_row_bytes_through_the_library():
    lq = _lq()
    for bits in (2, 3, 4):
        for c in (1, 13, 4096, 11008):
            assert lq.lq_packed_row_bytes(c, bits) == po.packed_row_bytes(c, bits)
            P = lq.lq_params_default(bits=bits, mode=lq.LQ_GRID_NONUNIFORM)
            assert lq.lq_bits_per_weight(7, c, P) == po.bits_per_weight(7, c, bits, "nu")
    P = lq.lq_params_default(bits=4, mode=lq.LQ_GRID_AFFINE, group_size=128)
    assert lq.lq_bits_per_weight(7, 4096, P) == 4.25


def test_quantized_layer_round_trips_through_the_stored_form():
    """c1 end to end: W_hat from the stored form equals the loop's W_hat up to the binary16
    rounding of the grid, and the codes come back unchanged."""
    lq = _lq()
    cfg = lq_synth.CONFIGS["c1"]
    P = hx.params_for(cfg)
    out = hx.gpu_layer_pass(lq_synth.weights(cfg), lq_synth.activation_chunks(cfg), P)
    assert out["info"] == 0
    codes, What, grid = hx.to_dev(out["codes"], torch.uint8), hx.to_dev(out["W_hat"]), hx.to_dev(out["grid"])
    r, c = codes.shape
    rb = lq.lq_packed_row_bytes(c, P.bits)
    packed = torch.empty((r, rb), dtype=torch.uint8, device="cuda")
    table = torch.empty(grid.numel(), dtype=torch.int16, device="cuda")
    lq.lq_pack_layer(codes, grid, P, packed, table)
    W2 = torch.empty_like(What)
    codes2 = torch.empty_like(codes)
    lq.lq_unpack_layer(packed, table, c, P, W2, codes2)
    torch.cuda.synchronize()
    assert torch.equal(codes2, codes)
    rel = ((W2 - What).abs() / What.abs().clamp_min(1e-30)).max().item()
    assert rel <= 2.0 ** -11 + 1e-7, rel
    assert packed.numel() * 8 + table.numel() * 16 == round(lq.lq_bits_per_weight(r, c, P) * r * c)


def test_projections_sharing_an_input_are_quantized_in_one_pass():
    """q/k/v-style sharing: stacking the projections' rows and running the grid fit and the
    loop once against the shared U gives bit-identical results to one call per projection."""
    lq = _lq()
    cfg = lq_synth.CONFIGS["c1"].scaled(r=192, c=384, n_tokens=1536)
    P = hx.params_for(cfg)
    H = hx.gpu_hessian(lq_synth.activation_chunks(cfg), cfg.c)
    U, d, info = hx.gpu_cholesky(H, P.damp)
    assert info == 0
    Ws = [lq_synth.weights(cfg.scaled(seed=cfg.seed + k)) for k in range(3)]
    singles = []
    for W in Ws:
        grid = hx.gpu_fit_grid(hx.to_dev(W), d, P)
        singles.append((grid,) + hx.gpu_quantize(hx.to_dev(W), U, grid, P))
    Wall = hx.to_dev(np.concatenate(Ws, axis=0))
    grid_all = hx.gpu_fit_grid(Wall, d, P)
    What_all, codes_all, loss_all = hx.gpu_quantize(Wall, U, grid_all, P)
    r = cfg.r
    for k, (grid, What, codes, loss) in enumerate(singles):
        sl = slice(k * r, (k + 1) * r)
        assert torch.equal(grid_all[sl], grid)
        assert torch.equal(codes_all[sl], codes)
        assert torch.equal(What_all[sl], What)
        assert torch.equal(loss_all[sl], loss)


@pytest.mark.parametrize("mode,bits,group", [("nu", 4, 0), ("nu", 3, 0), ("nu", 2, 0),
                                             ("aff", 4, 128), ("aff", 2, 64), ("aff", 3, 0)])
@pytest.mark.parametrize("r,c,nb", [(5, 32, 1), (37, 1024, 3), (100, 4096, 1), (19, 11008, 2), (16, 16384, 1),
                                    (64, 2048, 7), (40, 11008, 5)])
def test_matvec_from_the_stored_form(mode, bits, group, r, c, nb):
    lq = _lq()
    if mode == "aff" and group and c % group:
        pytest.skip("group does not divide c")
    rng = np.random.default_rng(31 * bits + r + c)
    K = 1 << bits
    codes = rng.integers(0, K, size=(r, c)).astype(np.uint8)
    if mode == "nu":
        grid = np.sort(rng.normal(0, 0.02, size=(r, K)), axis=1).astype(np.float32)
        P = lq.lq_params_default(bits=bits, mode=lq.LQ_GRID_NONUNIFORM)
    else:
        ng = c // (group if group else c)
        S = np.abs(rng.normal(0.01, 0.003, size=(r, ng))) + 1e-4
        Z = rng.integers(-3, K + 3, size=(r, ng)).astype(np.float64)
        grid = np.stack([S, Z], axis=-1).astype(np.float32)
        P = lq.lq_params_default(bits=bits, mode=lq.LQ_GRID_AFFINE, group_size=group)
    # packed rows padded to 16 bytes so that every bit width meets its alignment
    rb = lq.lq_packed_row_bytes(c, bits)
    ld = (rb + 15) // 16 * 16
    packed = torch.zeros((r, ld), dtype=torch.uint8, device="cuda")[:, :rb]
    table = torch.empty(grid.size, dtype=torch.int16, device="cuda")
    lq.lq_pack_layer(hx.to_dev(codes, torch.uint8), hx.to_dev(grid), P, packed, table)
    X = rng.standard_normal((nb, c)).astype(np.float32)
    Y = torch.empty((nb, r), dtype=torch.float32, device="cuda")
    lq.lq_matvec_packed(packed, table, c, P, hx.to_dev(X), Y)
    torch.cuda.synchronize()
    exp_packed = po.pack_codes(codes, bits)
    exp_table = po.table_nu(grid) if mode == "nu" else po.table_aff(grid)
    ref = po.matvec_packed(exp_packed, exp_table, X, c, bits, mode, group)
    Wh = po.dequantize(exp_packed, exp_table, c, bits, mode, group).astype(np.float64)
    scale = np.abs(X.astype(np.float64)) @ np.abs(Wh).T          # sum_j |w_kj| |x_j|
    err = np.abs(Y.cpu().numpy() - ref)
    # fp32 accumulation of c products: error within c eps of the absolute sum, far below in practice
    assert np.all(err <= 4e-6 * scale + 1e-30), float(np.max(err / (scale + 1e-30)))


@pytest.mark.parametrize("mode,bits,group", [("nu", 4, 0), ("nu", 3, 0), ("nu", 2, 0),
                                             ("aff", 4, 128), ("aff", 2, 64), ("aff", 3, 0)])
@pytest.mark.parametrize("r,c,nb", [(37, 1024, 16), (200, 4096, 33), (130, 2048, 64), (64, 11008, 40),
                                    (257, 160, 17), (16, 16384, 32), (300, 4128, 100), (5, 32, 1),
                                    (24613, 64, 64), (12330, 96, 100), (41003, 32, 7)])
def test_matmul_from_the_stored_form(mode, bits, group, r, c, nb):
    """The batched (matrix-core) product with a stored layer against the float64 oracle, at the
    tolerance of the one-vector product: ragged row counts (tiles of 32 and of 128), batches that are not
    multiples of 32 / 64, column counts that are not multiples of the 64-column stage.  The library
    picks its kernel by the number of 128-row workgroups (below 192, or 320 for up to 32 vectors: the
    32-row kernel); the last three
    shapes have enough rows for the 128-row kernel and end inside a tile."""
    lq = _lq()
    if mode == "aff" and group and c % group:
        pytest.skip("group does not divide c")
    rng = np.random.default_rng(17 * bits + r + c + nb)
    K = 1 << bits
    codes = rng.integers(0, K, size=(r, c)).astype(np.uint8)
    if mode == "nu":
        grid = np.sort(rng.normal(0, 0.02, size=(r, K)), axis=1).astype(np.float32)
        P = lq.lq_params_default(bits=bits, mode=lq.LQ_GRID_NONUNIFORM)
    else:
        ng = c // (group if group else c)
        S = np.abs(rng.normal(0.01, 0.003, size=(r, ng))) + 1e-4
        Z = rng.integers(-3, K + 3, size=(r, ng)).astype(np.float64)
        grid = np.stack([S, Z], axis=-1).astype(np.float32)
        P = lq.lq_params_default(bits=bits, mode=lq.LQ_GRID_AFFINE, group_size=group)
    rb = lq.lq_packed_row_bytes(c, bits)
    ld = (rb + 15) // 16 * 16
    packed = torch.zeros((r, ld), dtype=torch.uint8, device="cuda")[:, :rb]
    table = torch.empty(grid.size, dtype=torch.int16, device="cuda")
    lq.lq_pack_layer(hx.to_dev(codes, torch.uint8), hx.to_dev(grid), P, packed, table)
    X = rng.standard_normal((nb, c)).astype(np.float32)
    Y = torch.full((nb, r), float("nan"), dtype=torch.float32, device="cuda")
    lq.lq_matmul_packed(packed, table, c, P, hx.to_dev(X), Y)
    torch.cuda.synchronize()
    exp_packed = po.pack_codes(codes, bits)
    exp_table = po.table_nu(grid) if mode == "nu" else po.table_aff(grid)
    ref = po.matvec_packed(exp_packed, exp_table, X, c, bits, mode, group)
    Wh = po.dequantize(exp_packed, exp_table, c, bits, mode, group).astype(np.float64)
    scale = np.abs(X.astype(np.float64)) @ np.abs(Wh).T          # sum_j |w_kj| |x_j|
    got = Y.cpu().numpy()
    assert np.all(np.isfinite(got))
    err = np.abs(got - ref)
    assert np.all(err <= 4e-6 * scale + 1e-30), float(np.max(err / (scale + 1e-30)))
    # and it agrees with the one-vector kernel far inside that tolerance (same weights, fp32 sums)
    if c <= 16384:
        Y1 = torch.empty((nb, r), dtype=torch.float32, device="cuda")
        lq.lq_matvec_packed(packed, table, c, P, hx.to_dev(X), Y1)
        torch.cuda.synchronize()
        assert np.all(np.abs(got - Y1.cpu().numpy()) <= 4e-6 * scale + 1e-30)


@pytest.mark.parametrize("mode,bits,group,r,c,nb", [("nu", 3, 0, 53248, 16384, 96), ("aff", 4, 128, 28672, 8192, 256),
                                                    ("aff", 2, 64, 53248, 16384, 40)])
def test_matmul_at_the_size_of_the_large_layers(mode, bits, group, r, c, nb):
    """The batched product at the row and column counts of configurations 4 and 5 (several hundred
    row tiles, batches that end inside a tile).  Seeded codes and tables; the library packs and
    multiplies the whole layer, the oracle packs and multiplies sampled rows (first and last tile
    included) from the same seeded codes."""
    lq = _lq()
    rng = np.random.default_rng(7 + bits + nb)
    K = 1 << bits
    codes = rng.integers(0, K, size=(r, c), dtype=np.uint8)
    if mode == "nu":
        grid = np.sort(rng.normal(0, 0.02, size=(r, K)), axis=1).astype(np.float32)
        P = lq.lq_params_default(bits=bits, mode=lq.LQ_GRID_NONUNIFORM)
    else:
        ng = c // group
        S = (rng.random((r, ng)) * 0.01 + 1e-3)
        Z = rng.integers(-3, K + 3, size=(r, ng)).astype(np.float64)
        grid = np.stack([S, Z], axis=-1).astype(np.float32)
        P = lq.lq_params_default(bits=bits, mode=lq.LQ_GRID_AFFINE, group_size=group)
    rb = lq.lq_packed_row_bytes(c, bits)
    packed = torch.zeros((r, rb), dtype=torch.uint8, device="cuda")
    table = torch.empty(grid.size, dtype=torch.int16, device="cuda")
    lq.lq_pack_layer(hx.to_dev(codes, torch.uint8), hx.to_dev(grid), P, packed, table)
    X = rng.standard_normal((nb, c)).astype(np.float32)
    Y = torch.full((nb, r), float("nan"), device="cuda")
    lq.lq_matmul_packed(packed, table, c, P, hx.to_dev(X), Y)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Y).all())
    rows = np.unique(np.concatenate([np.arange(0, 3), np.arange(r - 3, r), rng.integers(0, r, size=26)]))
    exp_packed = po.pack_codes(codes[rows], bits)
    exp_table = po.table_nu(grid[rows]) if mode == "nu" else po.table_aff(grid[rows])
    ref = po.matvec_packed(exp_packed, exp_table, X, c, bits, mode, group)          # [nb x rows]
    Wh = po.dequantize(exp_packed, exp_table, c, bits, mode, group).astype(np.float64)
    scale = np.abs(X.astype(np.float64)) @ np.abs(Wh).T
    got = Y[:, torch.as_tensor(rows, device="cuda")].cpu().numpy()
    err = np.abs(got - ref)
    assert np.all(err <= 4e-6 * scale + 1e-30), float(np.max(err / (scale + 1e-30)))
