"""lq_hessian_accumulate_host: activations streamed from (pinned) host memory in chunks, the
upload of one chunk overlapping the accumulation of the previous one.  Bit-identical to one
device call per chunk, and within the Hessian tolerance of the float64 oracle."""
import numpy as np
import pytest

import lq_synth
from oracle import leanquant_oracle as orc
from tests import lq_harness as hx

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _lq():
    import paper_2407_10032_amd as lq
    lq.load()
    return lq


def _check_against_oracle(H, X64, scale=1.0):
    ref = scale * orc.hessian(X64)
    sc = np.sqrt(np.outer(np.diag(ref), np.diag(ref))) + 1e-30
    # fp32 products summed over n tokens: error ~ sqrt(n) * 2^-24 relative to |x_i||x_j|
    n = X64.shape[0]
    assert np.max(np.abs(H.cpu().numpy() - ref) / sc) < 2e-6 * max(4.0, np.sqrt(n))


def _host_call(lq, Xh, c, chunk):
    H = torch.zeros((c, c), dtype=torch.float32, device="cuda")
    ws = lq.alloc_workspace(lq.lq_hessian_host_workspace_bytes(c, Xh.shape[0], chunk))
    lq.lq_hessian_accumulate_host(H, Xh, chunk, ws)
    torch.cuda.synchronize()
    return H


@pytest.mark.parametrize("c,n,chunk", [(256, 1000, 256), (384, 4096, 1024), (200, 777, 1000),
                                       (512, 2048, 2048), (130, 900, 128), (1024, 5000, 2048)])
def test_host_streaming_equals_one_device_call_per_chunk(c, n, chunk):
    lq = _lq()
    print(f"hessian from host c={c} n={n} chunk={chunk}", flush=True)
    rng = np.random.default_rng(c + n + chunk)
    X = rng.standard_normal((n, c)).astype(np.float32)
    Xh = torch.from_numpy(X).pin_memory()
    H = _host_call(lq, Xh, c, chunk)
    Hd = hx.gpu_hessian([X[i:i + chunk] for i in range(0, n, chunk)], c)
    assert torch.equal(H, Hd)
    _check_against_oracle(H, X.astype(np.float64))


def test_host_streaming_strided_rows_pageable_memory_and_two_calls():
    """Leading dimension larger than c (2-D copies), pageable host memory (correct, only
    slower), and two calls in a row that add up."""
    lq = _lq()
    c, n, chunk = 192, 1500, 400
    rng = np.random.default_rng(5)
    big = rng.standard_normal((n, c + 37)).astype(np.float32)
    Xv = torch.from_numpy(big)[:, :c]                 # pageable, ld = c + 37
    H = torch.zeros((c, c), dtype=torch.float32, device="cuda")
    ws = lq.alloc_workspace(lq.lq_hessian_host_workspace_bytes(c, n, chunk))
    lq.lq_hessian_accumulate_host(H, Xv, chunk, ws)
    lq.lq_hessian_accumulate_host(H, Xv, chunk, ws)
    torch.cuda.synchronize()
    _check_against_oracle(H, big[:, :c].astype(np.float64), scale=2.0)


def test_host_streaming_on_the_small_configuration():
    lq = _lq()
    cfg = lq_synth.CONFIGS["c1"]
    X = np.concatenate(list(lq_synth.activation_chunks(cfg)), axis=0)
    Xh = torch.from_numpy(np.ascontiguousarray(X, dtype=np.float32)).pin_memory()
    H = _host_call(lq, Xh, cfg.c, 512)
    _check_against_oracle(H, X.astype(np.float64))
