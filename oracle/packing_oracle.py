"""CPU oracle for the stored form of a quantized layer: packed codes + 16-bit tables.

TEST INFRASTRUCTURE ONLY (as leanquant_oracle.py): only tests/, __graft_entry__.smoke()
and the cpu_baseline leg of bench.py may import it; it shares no code with the HIP path.

What the paper fixes is the size of the stored layer: the "Bits" columns of its result
tables (4.05 / 3.02 / 2.01 for non-uniform grids at b = 4 / 3 / 2, 4.25 for affine 4-bit
grids at group size 128) are b bits per weight plus sixteen bits per grid point per row
(non-uniform, Section 2.1: one set of 2^b points per row) or a sixteen-bit scale and a
sixteen-bit zero-point per group (affine).  The byte layout itself is this build's choice
and is stated here in full:

  * codes: every row is a little-endian bit stream, code j of the row occupies bits
    [j b, (j + 1) b) of it (bit k of the stream is bit k % 8 of byte k // 8); a row takes
    ceil(c b / 8) bytes and the unused high bits of its last byte are zero;
  * non-uniform table: [r x 2^b] IEEE binary16, the grid rounded to nearest-even;
  * affine table: [r x c/g x 2] 16-bit words, (binary16 scale S rounded to nearest-even,
    zero-point Z as a two's-complement int16, saturated to [-32768, 32767]).

Dequantized weights from the stored form: non-uniform G16[k, code]; affine
(code - Z) * S16 (Section 2.1, quant_aff).  They differ from Algorithm 1's W_hat only by the
16-bit rounding of the table.
"""
from __future__ import annotations

import numpy as np


def bits_per_weight(r, c, bits, mode, group_size=0):
    """Stored bits per weight of an r x c layer ('Bits' columns of the result tables)."""
    if mode == "nu":
        return bits + 16.0 * (1 << bits) / c
    g = group_size if group_size else c
    return bits + 32.0 / g


def model_bits_per_weight(shapes, bits, mode, group_size=0):
    """Size-weighted average over a list of (r, c) layer shapes."""
    tot = sum(r * c for r, c in shapes)
    return sum(r * c * bits_per_weight(r, c, bits, mode, group_size) for r, c in shapes) / tot


def packed_row_bytes(c, bits):
    return (c * bits + 7) // 8


def pack_codes(codes, bits):
    """codes [r x c] integers in [0, 2^bits) -> uint8 [r x ceil(c bits / 8)]."""
    codes = np.asarray(codes)
    r, c = codes.shape
    out = np.zeros((r, packed_row_bytes(c, bits)), dtype=np.uint8)
    for k in range(r):
        for j in range(c):
            v = int(codes[k, j])
            for b in range(bits):
                if (v >> b) & 1:
                    pos = j * bits + b
                    out[k, pos // 8] |= np.uint8(1 << (pos % 8))
    return out


def unpack_codes(packed, c, bits):
    packed = np.asarray(packed, dtype=np.uint8)
    r = packed.shape[0]
    out = np.zeros((r, c), dtype=np.uint8)
    for k in range(r):
        for j in range(c):
            v = 0
            for b in range(bits):
                pos = j * bits + b
                v |= ((int(packed[k, pos // 8]) >> (pos % 8)) & 1) << b
            out[k, j] = v
    return out


def table_nu(grid):
    """[r x K] grid -> uint16 bit patterns of the binary16 roundings."""
    return np.asarray(grid, dtype=np.float64).astype(np.float16).view(np.uint16)


def table_aff(grid):
    """[r x ngroups x 2] (S, Z) -> uint16 words (binary16 S, int16 Z)."""
    g = np.asarray(grid, dtype=np.float64)
    s16 = g[..., 0].astype(np.float16).view(np.uint16)
    z = np.clip(np.rint(g[..., 1]), -32768, 32767).astype(np.int16).view(np.uint16)
    return np.stack([s16, z], axis=-1)


def dequantize(packed, table, c, bits, mode, group_size=0):
    """Stored form -> float32 weights [r x c]."""
    codes = unpack_codes(packed, c, bits).astype(np.int64)
    table = np.asarray(table, dtype=np.uint16)
    r = codes.shape[0]
    if mode == "nu":
        lut = table.view(np.float16).astype(np.float64)
        return np.take_along_axis(lut, codes, axis=1).astype(np.float32)
    g = group_size if group_size else c
    S = table[..., 0].copy().view(np.float16).astype(np.float64)       # [r x ngroups]
    Z = table[..., 1].copy().view(np.int16).astype(np.float64)
    gi = np.arange(c) // g
    return ((codes - Z[:, gi]) * S[:, gi]).astype(np.float32)


def matvec_packed(packed, table, X, c, bits, mode, group_size=0):
    """Y[n, k] = sum_j W_hat[k, j] X[n, j] with W_hat the weights the stored form stands for
    (dequantize above), in float64.  X [nb x c]; returns [nb x r]: what the inference kernel
    of a quantized linear layer computes (the paper's appendix on inference efficiency)."""
    Wh = dequantize(packed, table, c, bits, mode, group_size).astype(np.float64)
    return np.asarray(X, dtype=np.float64) @ Wh.T
