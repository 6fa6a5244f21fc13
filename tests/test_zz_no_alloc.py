"""lq_fit_grid_static -- the entry point for callers that cannot allocate -- against lq_fit_grid.

Called through the C ABI (ctypes symbols, raw device pointers).  The same kernels run with the
library's built-in scratch instead of a caller workspace, so the grids must be bit-identical.
Two calls in a row, the second on a smaller input (the scratch keeps the first call's
contents), in both grid modes; sizes beyond the built-in scratch are refused on the host.
"""
import ctypes

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2407_10032_amd as lq


def _layer(r, c, seed):
    g = np.random.default_rng(seed)
    W = (g.standard_normal((r, c)) * 0.02).astype(np.float32)
    W[g.random((r, c)) < 0.01] *= 8
    d = np.exp(g.standard_normal(c) * 0.7).astype(np.float32)
    return torch.from_numpy(W).cuda(), torch.from_numpy(d).cuda()


def _fit_both(W, d, P):
    """(grid from lq_fit_grid with a workspace, grid from lq_fit_grid_static), raw C calls."""
    lib = lq.load()
    r, c = W.shape
    stream = torch.cuda.current_stream().cuda_stream
    ref = torch.full(lq.grid_shape(P, r, c), float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full(lq.grid_shape(P, r, c), float("nan"), dtype=torch.float32, device="cuda")
    need = lib.lq_workspace_bytes(lq.LQ_CALL_FIT_GRID, r, c, 0, ctypes.byref(P))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    rc = lib.lq_fit_grid(W.data_ptr(), r, c, W.stride(0), d.data_ptr(), ctypes.byref(P), ref.data_ptr(),
                         ws.data_ptr(), ws.numel(), stream)
    assert rc == lq.LQ_OK, lib.lq_last_error()
    rc = lib.lq_fit_grid_static(W.data_ptr(), r, c, W.stride(0), d.data_ptr(), ctypes.byref(P),
                                got.data_ptr(), stream)
    assert rc == lq.LQ_OK, lib.lq_last_error()
    torch.cuda.synchronize()
    return ref, got


@pytest.mark.parametrize("mode", ["nu", "aff"])
def test_static_scratch_matches_workspace_call_twice(mode):
    if mode == "nu":
        P = lq.lq_params_default(bits=4)
    else:
        P = lq.lq_params_default(bits=3, mode=lq.LQ_GRID_AFFINE, group_size=64, T=256)
    for (r, c, seed) in [(96, 4096, 1), (40, 640, 2)]:          # second call: smaller input
        print(f"lq_fit_grid_static {mode} r={r} c={c}", flush=True)
        W, d = _layer(r, c, seed)
        ref, got = _fit_both(W, d, P)
        assert not torch.isnan(got).any()
        assert torch.equal(ref, got)


def test_static_scratch_limit_and_argument_errors():
    lib = lq.load()
    P = lq.lq_params_default(bits=4)
    stream = torch.cuda.current_stream().cuda_stream
    c = 16384 + 256
    W = torch.zeros((2, c), dtype=torch.float32, device="cuda")
    d = torch.ones(c, dtype=torch.float32, device="cuda")
    grid = torch.zeros((2, 16), dtype=torch.float32, device="cuda")
    rc = lib.lq_fit_grid_static(W.data_ptr(), 2, c, c, d.data_ptr(), ctypes.byref(P), grid.data_ptr(), stream)
    assert rc == lq.LQ_ERR_UNSUPPORTED and b"16384" in lib.lq_last_error()
    rc = lib.lq_fit_grid_static(None, 2, 512, 512, d.data_ptr(), ctypes.byref(P), grid.data_ptr(), stream)
    assert rc == lq.LQ_ERR_INVALID_ARG
    torch.cuda.synchronize()
