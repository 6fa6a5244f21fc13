"""Timing of the products with a stored (packed) layer: one vector at a time against batches.

    python -m paper_2407_10032_amd.stored_layer_bench [--shapes c2,c4,c5] [--reps 10]

For each layer shape (rows x columns, bit width, grid kind of the paper's configurations) random
codes and tables are packed with lq_pack_layer, and y = W_hat x is computed for batches of input
vectors with lq_matmul_packed (matrix cores) and with lq_matvec_packed (vector ALU, which walks
the codes once per 4 vectors, or per 2 on rows longer than 8192).  Printed per batch
size: the time of both, the flop rate of the batched kernel against the fp32 matrix-core peak, and
the rate at which the stored bytes are consumed (what bounds the one-vector product).  This is the
decoding-time operation the paper's appendix on inference efficiency builds a kernel for; nothing
here needs a model or data.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as lq

FP32_MFMA_PEAK_TFLOPS = 157.3

SHAPES = {
    # name: (rows, columns, bits, grid kind, group size, batch sizes)
    "c2": (4096, 4096, 4, "nu", 0, (1, 4, 16, 64, 256, 1024)),
    "c3": (4096, 11008, 3, "nu", 0, (1, 4, 64, 256)),
    "c4": (28672, 8192, 4, "aff", 128, (1, 4, 32, 64, 256)),
    "c5": (53248, 16384, 2, "aff", 64, (1, 4, 64)),
    "c5nu": (53248, 16384, 3, "nu", 0, (1, 4, 64, 128)),
    "c5nu4": (53248, 16384, 4, "nu", 0, (1, 4, 64, 128)),
}


def _time(fn, reps):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e-3           # seconds


def run(name, reps):
    r, c, bits, kind, group, batches = SHAPES[name]
    K = 1 << bits
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234)
    mode = lq.LQ_GRID_AFFINE if kind == "aff" else lq.LQ_GRID_NONUNIFORM
    P = lq.lq_params_default(bits=bits, mode=mode, group_size=group)
    codes = torch.randint(0, K, (r, c), dtype=torch.uint8, device="cuda", generator=gen)
    if kind == "nu":
        grid = torch.sort(torch.randn((r, K), device="cuda", generator=gen) * 0.02, dim=1).values.contiguous()
    else:
        ng = c // (group if group else c)
        S = torch.rand((r, ng), device="cuda", generator=gen) * 0.01 + 1e-3
        Z = torch.randint(0, K, (r, ng), device="cuda", generator=gen).float()
        grid = torch.stack([S, Z], dim=-1).contiguous()
    rb = lq.lq_packed_row_bytes(c, bits)
    packed = torch.zeros((r, rb), dtype=torch.uint8, device="cuda")
    table = torch.empty(grid.numel(), dtype=torch.int16, device="cuda")
    lq.lq_pack_layer(codes, grid, P, packed, table)
    stored = packed.numel() + 2 * table.numel()
    print(f"{name}: {r} x {c}, {bits}-bit {'affine g' + str(group) if kind == 'aff' else 'non-uniform'}, "
          f"stored form {stored / 1e6:.1f} MB ({lq.lq_bits_per_weight(r, c, P):.3f} bits per weight)", flush=True)
    for nb in batches:
        X = torch.randn((nb, c), device="cuda", generator=gen)
        Y = torch.empty((nb, r), device="cuda")
        Y1 = torch.empty((nb, r), device="cuda")
        tm = _time(lambda: lq.lq_matmul_packed(packed, table, c, P, X, Y), reps)
        tv = _time(lambda: lq.lq_matvec_packed(packed, table, c, P, X, Y1), reps) if c <= 16384 else float("nan")
        flop = 2.0 * nb * r * c
        per_pass = 4 if c <= 8192 else 2                # vectors that share one walk over the codes
        passes = (nb + per_pass - 1) // per_pass
        diff = float((Y - Y1).abs().max()) if c <= 16384 else float("nan")
        print(f"  nb {nb:5d}: matmul {tm * 1e6:9.1f} us = {flop / tm / 1e12:6.1f} TFLOP/s "
              f"({100 * flop / tm / 1e12 / FP32_MFMA_PEAK_TFLOPS:4.1f} % of the fp32 MFMA peak), "
              f"{stored / tm / 1e12:5.2f} TB/s of stored bytes | matvec passes {tv * 1e6:9.1f} us = "
              f"{stored * passes / tv / 1e12:5.2f} TB/s of stored bytes | max |difference| {diff:.2e}",
              flush=True)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--shapes", default="c2,c4,c5nu", help="comma-separated: " + ", ".join(SHAPES))
    ap.add_argument("--reps", type=int, default=10)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("stored_layer_bench needs a GPU")
    lq.load()
    for name in args.shapes.split(","):
        run(name, args.reps)


if __name__ == "__main__":
    main()
