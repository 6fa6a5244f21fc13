"""Pins of the packing oracle (CPU only): the paper's printed sizes, hand-computed bytes,
round trips, and numpy's own bit packing as an independent routine."""
import os

import numpy as np
import pytest

from oracle import packing_oracle as po

HERE = os.path.dirname(__file__)

# Linear layers (r = out, c = in) of one transformer block; every block of a model is the same.
LLAMA3_8B = [(4096, 4096), (1024, 4096), (1024, 4096), (4096, 4096),
             (14336, 4096), (14336, 4096), (4096, 14336)]
LLAMA2_7B = [(4096, 4096)] * 4 + [(11008, 4096), (11008, 4096), (4096, 11008)]
MISTRAL_7B = LLAMA3_8B     # same projection shapes (grouped-query attention, 14336-wide MLP)


def _golden():
    rows = []
    for line in open(os.path.join(HERE, "golden", "bits_per_weight.txt")):
        if line.strip() and not line.startswith("#"):
            m, b, g, v = line.split()
            rows.append((m, int(b), int(g), float(v)))
    return rows


@pytest.mark.parametrize("shapes", [LLAMA3_8B, LLAMA2_7B, MISTRAL_7B])
def test_bit_accounting_reproduces_the_papers_bits_columns(shapes):
    for mode, bits, group, printed in _golden():
        v = po.model_bits_per_weight(shapes, bits, mode, group)
        # the tables print two decimals; the values agree to the printed precision
        assert abs(v - printed) < 0.0075, (mode, bits, group, v, printed)
        if mode == "aff":
            assert v == printed


def test_bits_per_weight_closed_forms():
    assert po.bits_per_weight(4096, 4096, 4, "nu") == 4 + 256 / 4096
    assert po.bits_per_weight(10, 11008, 3, "nu") == 3 + 128 / 11008
    assert po.bits_per_weight(10, 4096, 2, "aff", 64) == 2.5
    assert po.bits_per_weight(10, 4096, 4, "aff", 0) == 4 + 32 / 4096


def test_pack_hand_computed_bytes():
    # eight 3-bit codes make exactly three bytes: sum code_j << 3j = 0x1F58D1, little-endian
    codes = np.array([[1, 2, 3, 4, 5, 6, 7, 0]])
    assert po.pack_codes(codes, 3).tolist() == [[0xD1, 0x58, 0x1F]]
    # 4-bit: low nibble first; 2-bit: four codes per byte, first code in the low bits
    assert po.pack_codes(np.array([[0xA, 0x3, 0xF]]), 4).tolist() == [[0x3A, 0x0F]]
    assert po.pack_codes(np.array([[1, 2, 3, 0, 2]]), 2).tolist() == [[0b00111001, 0b10]]


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("c", [1, 5, 8, 13, 64, 67])
def test_pack_round_trip_and_row_bytes(bits, c):
    rng = np.random.default_rng(100 * bits + c)
    codes = rng.integers(0, 1 << bits, size=(7, c))
    packed = po.pack_codes(codes, bits)
    assert packed.shape == (7, (c * bits + 7) // 8) == (7, po.packed_row_bytes(c, bits))
    assert np.array_equal(po.unpack_codes(packed, c, bits), codes)
    # unused high bits of the last byte are zero
    used = c * bits - 8 * (packed.shape[1] - 1)
    assert np.all((packed[:, -1] >> used) == 0) if used < 8 else True


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_pack_matches_numpy_packbits(bits):
    # independent routine: expand every code to its bits (LSB first) and let numpy pack
    # the row's bit string in little-endian bit order
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, 1 << bits, size=(5, 37))
    bitsarr = ((codes[:, :, None] >> np.arange(bits)) & 1).reshape(5, -1).astype(np.uint8)
    ref = np.packbits(bitsarr, axis=1, bitorder="little")
    assert np.array_equal(po.pack_codes(codes, bits), ref)


def test_tables_are_nearest_even_binary16_and_int16():
    # 1 + 2^-11 is half way between two binary16 numbers: ties go to the even mantissa
    g = np.array([[1.0, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 65504.0, -0.333251953125]])
    t = po.table_nu(g).view(np.float16)
    assert t.tolist() == [[1.0, 1.0, 1.0 + 2.0 ** -9, 65504.0, -0.333251953125]]
    sz = np.array([[[0.1, -7.0], [2.0, 40000.0], [3.0, -40000.0]]])
    ta = po.table_aff(sz)
    assert ta[0, :, 1].view(np.int16).tolist() == [-7, 32767, -32768]
    assert ta[0, :, 0].view(np.float16).tolist() == [np.float16(0.1), 2.0, 3.0]


def test_dequantize_follows_the_grid_definitions():
    rng = np.random.default_rng(5)
    # non-uniform: a grid that is exact in binary16 comes back exactly
    grid = np.sort(rng.integers(-512, 512, size=(6, 8)) / 1024.0, axis=1)
    codes = rng.integers(0, 8, size=(6, 21))
    w = po.dequantize(po.pack_codes(codes, 3), po.table_nu(grid), 21, 3, "nu")
    assert np.array_equal(w, np.take_along_axis(grid, codes, axis=1).astype(np.float32))
    # affine (Section 2.1): (w_int - Z) S per group
    S = np.array([[0.5, 0.25], [0.125, 2.0]])
    Z = np.array([[3.0, -2.0], [0.0, 7.0]])
    codes = rng.integers(0, 16, size=(2, 8))
    w = po.dequantize(po.pack_codes(codes, 4), po.table_aff(np.stack([S, Z], -1)), 8, 4, "aff", 4)
    gi = np.arange(8) // 4
    assert np.array_equal(w, ((codes - Z[:, gi]) * S[:, gi]).astype(np.float32))


def test_matvec_packed_is_the_product_with_the_dequantized_weights():
    rng = np.random.default_rng(9)
    # identity-like check: a grid that is exact in binary16 and one-hot inputs read out columns
    grid = np.sort(rng.integers(-512, 512, size=(5, 4)) / 1024.0, axis=1)
    codes = rng.integers(0, 4, size=(5, 12))
    packed, table = po.pack_codes(codes, 2), po.table_nu(grid)
    W = np.take_along_axis(grid, codes, axis=1)
    Y = po.matvec_packed(packed, table, np.eye(12), 12, 2, "nu")
    assert np.array_equal(Y, W.T)
    x = rng.standard_normal((3, 12))
    assert np.allclose(po.matvec_packed(packed, table, x, 12, 2, "nu"), x @ W.T, rtol=0, atol=1e-15)
