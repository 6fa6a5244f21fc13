"""Benchmark of the LeanQuant per-layer quantization pass on one MI355X.

A step is one pass of the whole hot path (Hessian accumulation over all calibration
tokens, Cholesky of the damped inverse, grid fit, blocked quantize-and-propagate
loop) on the Llama-2-7B-shaped 4096 x 4096 layer with 262144 x 4096 activations
(4-bit non-uniform, B = 128), inputs seeded, synthetic and resident in HBM.

Prints ONE JSON line: layer quantization throughput in weights/s, plus the roofline
of the dominant kernel (the fp32 MFMA Gram product) and the float64 oracle timed
on a bounded sample on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP32_MFMA_PEAK_TFLOPS = 157.3
# HBM-side bytes of one Gram-kernel launch on the c2 workload: NOT measured by this run (bench.py
# cannot read hardware counters).  It is the figure of the two rocprofv3 --pmc runs of this very
# command (FETCH_SIZE, then WRITE_SIZE, each scaled by a plain copy of known size) that
# profiles/bench_c2_gram_kernel_counters.md summarises; only valid for that workload.
GRAM_TRAFFIC_BYTES_C2 = 48.1e9
GRAM_TRAFFIC_SOURCE = "profiles/bench_c2_gram_kernel_counters.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command; not measured in this run)"


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def load_inputs(cfg, torch, lq_synth):
    """X [n_tokens x c] and W [r x c] on the device, generated chunk by chunk on the host."""
    X = torch.empty((cfg.n_tokens, cfg.c), dtype=torch.float32, device="cuda")
    nchunks = lq_synth.n_token_chunks(cfg)
    t0 = time.time()
    with ThreadPoolExecutor(max_workers=8) as ex:
        for k, xc in enumerate(ex.map(lambda k: lq_synth.activation_chunk(cfg, k), range(nchunks))):
            t = k * lq_synth.TOKEN_CHUNK
            X[t:t + xc.shape[0]].copy_(torch.from_numpy(xc))
            if k % 8 == 7:
                log("  generated %d / %d activation chunks (%.0f s)" % (k + 1, nchunks, time.time() - t0))
    W = torch.from_numpy(lq_synth.weights(cfg)).cuda()
    torch.cuda.synchronize()
    return X, W


def cpu_baseline(cfg, lq_synth):
    """The float64 oracle, as it stands, on a bounded sample of the same workload."""
    from oracle import leanquant_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    tok = 32768
    rows = 512
    sub = cfg.scaled(n_tokens=tok)
    t0 = time.time()
    H = None
    for k in range(lq_synth.n_token_chunks(sub)):
        H = orc.hessian(lq_synth.activation_chunk(sub, k), H)
    t_h = time.time() - t0
    log("  oracle: Gram on %d tokens %.1f s" % (tok, t_h))
    t0 = time.time()
    U, d = orc.cholesky_inv(H, cfg.damp)
    t_c = time.time() - t0
    log("  oracle: inverse + Cholesky %.1f s" % t_c)
    W = lq_synth.weights(cfg, list(range(rows)))
    t0 = time.time()
    G = orc.fit_grid_nu(W, d, cfg.bits, cfg.p)
    t_g = time.time() - t0
    t0 = time.time()
    orc.quantize_layer(W, U, G, "nu", cfg.bits, B=cfg.block)
    t_q = time.time() - t0
    log("  oracle: grid fit %.1f s, column loop %.1f s on %d rows" % (t_g, t_q, rows))
    total = t_h * (cfg.n_tokens / tok) + t_c + (t_g + t_q) * (cfg.r / rows)
    return {
        "value": cfg.r * cfg.c / total, "unit": "weights/s", "cores": int(cores), "kind": "oracle",
        "sample": "float64 numpy oracle: Gram on %d of %d tokens (%.1f s), full inverse+Cholesky "
                  "(%.1f s), grid fit + column loop on %d of %d rows (%.1f s + %.1f s); the token "
                  "and row parts scaled linearly to the full layer (%.0f s)"
                  % (tok, cfg.n_tokens, t_h, t_c, rows, cfg.r, t_g, t_q, total),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="c2", help="lq_synth configuration (the metric is quoted on c2)")
    ap.add_argument("--tokens", type=int, default=0, help="override the token count (not the metric's workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch

    import lq_synth
    import paper_2407_10032_amd as lq

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    lq.load()
    cfg = lq_synth.CONFIGS[args.config]
    if args.tokens:
        cfg = cfg.scaled(n_tokens=args.tokens)
    P = lq.params_for(cfg)
    r, c, n = cfg.r, cfg.c, cfg.n_tokens
    log("generating %s: W %d x %d, X %d x %d" % (cfg.name, r, c, n, c))
    X, W = load_inputs(cfg, torch, lq_synth)

    H = torch.zeros((c, c), dtype=torch.float32, device="cuda")
    U = torch.empty((c, c), dtype=torch.float32, device="cuda")
    d = torch.empty(c, dtype=torch.float32, device="cuda")
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    grid = torch.empty(lq.grid_shape(P, r, c), dtype=torch.float32, device="cuda")
    Wq = torch.empty_like(W)
    codes = torch.empty((r, c), dtype=torch.uint8, device="cuda")
    row_loss = torch.empty(r, dtype=torch.float32, device="cuda")
    ws = lq.alloc_workspace(max(lq.lq_workspace_bytes(k, r, c, n, P) for k in range(4)))

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]

    def step(e=None):
        H.zero_()
        Wq.copy_(W)
        if e: e[0].record()
        lq.lq_hessian_accumulate(H, X, ws)
        if e: e[1].record()
        lq.lq_cholesky_inv(H, P.damp, U, d, info, ws)
        if e: e[2].record()
        lq.lq_fit_grid(W, d, P, grid, ws)
        if e: e[3].record()
        lq.lq_quantize_layer(Wq, U, grid, P, codes, row_loss, ws)
        if e: e[4].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(ev[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    assert int(info.item()) == 0, "damped Hessian reported as not positive definite"

    # the stored form of the result (packed codes + 16-bit tables): timed apart, it is not a
    # step of Algorithm 1 and not part of `value`
    packed = torch.empty((r, lq.lq_packed_row_bytes(c, P.bits)), dtype=torch.uint8, device="cuda")
    table = torch.empty(grid.numel(), dtype=torch.int16, device="cuda")
    pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    lq.lq_pack_layer(codes, grid, P, packed, table)
    pe[0].record()
    for _ in range(5):
        lq.lq_pack_layer(codes, grid, P, packed, table)
    pe[1].record()
    torch.cuda.synchronize()
    pack_ms = pe[0].elapsed_time(pe[1]) / 5

    # product of the stored layer with one input vector (decoding-time use of the result):
    # also apart from `value`; the kernel needs c to be a multiple of 32 and at most 16384
    matvec_us = None
    if c % 32 == 0 and c <= 16384 and (P.mode == lq.LQ_GRID_NONUNIFORM or (P.group_size or c) % 32 == 0) \
            and packed.stride(0) % 16 == 0:
        xv = torch.randn((1, c), dtype=torch.float32, device="cuda")
        yv = torch.empty((1, r), dtype=torch.float32, device="cuda")
        lq.lq_matvec_packed(packed, table, c, P, xv, yv)
        pe2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        pe2[0].record()
        for _ in range(20):
            lq.lq_matvec_packed(packed, table, c, P, xv, yv)
        pe2[1].record()
        torch.cuda.synchronize()
        matvec_us = 1e3 * pe2[0].elapsed_time(pe2[1]) / 20

    # the batched product (64 input vectors) on the fp32 matrix cores: apart from `value` as well
    matmul_us = None
    if c % 32 == 0 and (P.mode == lq.LQ_GRID_NONUNIFORM or (P.group_size or c) % 32 == 0) \
            and packed.stride(0) % 16 == 0:
        xb = torch.randn((64, c), dtype=torch.float32, device="cuda")
        yb = torch.empty((64, r), dtype=torch.float32, device="cuda")
        lq.lq_matmul_packed(packed, table, c, P, xb, yb)
        pe3 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        pe3[0].record()
        for _ in range(10):
            lq.lq_matmul_packed(packed, table, c, P, xb, yb)
        pe3[1].record()
        torch.cuda.synchronize()
        matmul_us = 1e3 * pe3[0].elapsed_time(pe3[1]) / 10

    stage = np.array([[ev[k][i].elapsed_time(ev[k][i + 1]) for i in range(4)] for k in range(args.steps)])
    stage_ms = stage.mean(axis=0)
    # fp32 MFMA Gram product.  Algorithmic work of H += 2 X^T X with the symmetry used: the
    # c (c + 1) / 2 distinct entries take N multiply-adds each, N c (c + 1) flop per launch; the kernel
    # executes whole 128 x 128 tiles above the diagonal and, of a diagonal tile, the ten 32 x 32
    # sub-tiles on and above the diagonal (four of them compute both halves), reported next to it
    # as flops_executed.
    T = (c + 127) // 128
    flops_executed = 2.0 * n * (128 * 128 * (T * (T - 1) // 2) + 10 * 32 * 32 * T)
    flops = float(n) * c * (c + 1)
    achieved = flops / (stage_ms[0] * 1e-3) / 1e12
    out = {
        "metric": "layer quantization throughput (weights/s) at 4096x4096; %MFMA / %HBM peak",
        "value": r * c / (ms_per_step * 1e-3), "unit": "weights/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: W %dx%d fp32, X %dx%d fp32, %d-bit %s, B=%d, damp %.2f, p=%g"
                   % (cfg.name, r, c, n, c, cfg.bits, "non-uniform" if cfg.mode == "nu" else "affine g%d" % cfg.group_size,
                      cfg.block, cfg.damp, cfg.p),
                   "stage_ms": {"hessian": stage_ms[0], "cholesky_inv": stage_ms[1], "fit_grid": stage_ms[2],
                                "quantize_layer": stage_ms[3]},
                   # the same pass when H is reused from a projection with the same input
                   "weights_per_s_without_hessian": r * c / (float(stage_ms[1:].sum()) * 1e-3),
                   "pack_layer_ms": pack_ms, "matvec_packed_us": matvec_us,
                   "matmul_packed_nb64_us": matmul_us,
                   "matmul_packed_nb64_tflops": (2.0 * 64 * r * c / (matmul_us * 1e-6) / 1e12) if matmul_us else None,
                   "bits_per_weight": lq.lq_bits_per_weight(r, c, P)},
        "roofline": {"bound": "mfma", "kernel": "tn_gemm_kernel (H += 2 X^T X, upper tiles) + partial-sum reduce",
                     "achieved": achieved, "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / FP32_MFMA_PEAK_TFLOPS,
                     "traffic": GRAM_TRAFFIC_BYTES_C2 if (cfg.name == "c2" and not args.tokens) else None,
                     "traffic_source": GRAM_TRAFFIC_SOURCE if (cfg.name == "c2" and not args.tokens) else None,
                     "algorithmic_bytes": 4.0 * n * c,
                     "flops_per_launch": flops, "flops_executed": flops_executed,
                     "frac_executed": flops_executed / (stage_ms[0] * 1e-3) / 1e12 / FP32_MFMA_PEAK_TFLOPS,
                     "ms_per_launch": float(stage_ms[0])},
    }
    if not args.no_cpu_baseline:
        log("timing the float64 oracle on a bounded sample")
        out["cpu_baseline"] = cpu_baseline(cfg, lq_synth)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
