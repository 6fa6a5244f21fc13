"""The C-ABI boundary without a GPU: the library loads, exports every symbol the header
declares, sizes workspaces, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2407_10032_amd as lq
from paper_2407_10032_amd import binding


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        pytest.fail("libleanquant.so is not built (python -m paper_2407_10032_amd.build)")
    return lq.load()


def test_exports_match_header(lib, repo_root):
    text = open(os.path.join(repo_root, "include", "leanquant.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(lq_[a-z_]+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_defaults_are_the_papers_settings():
    P = lq.lq_params_default()
    assert (P.bits, P.mode, P.group_size, P.block, P.T, P.t_override, P.kmeans_max_iter) == (4, 0, 0, 128, 2048, -1, 100)
    assert P.damp == pytest.approx(0.01) and P.p == 4.0
    assert lq.lq_version() == "0.1"


def test_workspace_sizes():
    P = lq.lq_params_default()
    assert lq.lq_workspace_bytes(lq.LQ_CALL_HESSIAN, 0, 4096, 262144) == 32 * 528 * 128 * 128 * 4
    assert lq.lq_workspace_bytes(lq.LQ_CALL_HESSIAN, 0, 16384, 65536) == 4 * 8256 * 128 * 128 * 4
    assert lq.lq_workspace_bytes(lq.LQ_CALL_CHOLESKY, 0, 200) >= 2 * 256 * 256 * 4 + 2 * 128 * 128 * 4
    assert lq.lq_workspace_bytes(lq.LQ_CALL_QUANTIZE, 100, 512, 0, P) >= (100 + 4 * 128 + 4) * 128 * 4
    assert lq.lq_workspace_bytes(lq.LQ_CALL_FIT_GRID, 10, 512, 0, P) >= 512 * 12
    assert lq.lq_workspace_bytes(99, 1, 1, 1) == 0


def _bad(status, fragment):
    assert status != lq.LQ_OK
    assert fragment in lq.lq_last_error()


def test_argument_errors_are_host_side(lib):
    P = lq.lq_params_default()
    pp = ctypes.byref(P)
    dummy = ctypes.c_void_p(256)   # never dereferenced: every call below fails before a launch
    _bad(lib.lq_hessian_accumulate(None, 8, dummy, 4, 8, 8, dummy, 1 << 30, None), "null")
    assert lib.lq_hessian_accumulate(dummy, 4, dummy, 4, 8, 8, dummy, 1 << 30, None) == lq.LQ_ERR_INVALID_ARG
    assert lib.lq_hessian_accumulate(dummy, 8, dummy, 4, 8, 8, None, 0, None) == lq.LQ_ERR_WORKSPACE
    assert lib.lq_hessian_accumulate(dummy, 8, dummy, 4, 8, 8, dummy, 16, None) == lq.LQ_ERR_WORKSPACE
    assert lib.lq_hessian_accumulate(dummy, 8, dummy, 4, 8, 8, ctypes.c_void_p(260), 1 << 30, None) == lq.LQ_ERR_WORKSPACE
    _bad(lib.lq_hessian_accumulate_host(None, 8, dummy, 4, 8, 8, 2, dummy, 1 << 30, None), "null")
    assert lib.lq_hessian_accumulate_host(dummy, 8, dummy, 4, 8, 8, 0, dummy, 1 << 30, None) == lq.LQ_ERR_INVALID_ARG
    assert lib.lq_hessian_accumulate_host(dummy, 8, dummy, 4, 8, 4, 2, dummy, 1 << 30, None) == lq.LQ_ERR_INVALID_ARG
    assert lib.lq_hessian_accumulate_host(dummy, 8, dummy, 4, 8, 8, 2, dummy, 16, None) == lq.LQ_ERR_WORKSPACE
    assert lib.lq_hessian_accumulate_host(dummy, 8, dummy, 0, 8, 8, 2, None, 0, None) == lq.LQ_OK   # no tokens: no-op
    _bad(lib.lq_kmeanspp_seed(dummy, 4, 8, 8, dummy, pp, None, dummy, dummy, 1 << 30, None), "null")
    assert lib.lq_kmeanspp_seed(dummy, 4, 8, 4, dummy, pp, dummy, dummy, dummy, 1 << 30, None) == lq.LQ_ERR_INVALID_ARG
    assert lib.lq_kmeanspp_seed(dummy, 4, 8, 8, dummy, pp, dummy, dummy, dummy, 8, None) == lq.LQ_ERR_WORKSPACE
    assert lib.lq_kmeanspp_seed(dummy, 4, 32768, 32768, dummy, pp, dummy, dummy, dummy, 1 << 30, None) == lq.LQ_ERR_UNSUPPORTED
    Paff = lq.lq_params_default(bits=4, mode=lq.LQ_GRID_AFFINE, group_size=8)
    assert lib.lq_kmeanspp_seed(dummy, 4, 8, 8, dummy, ctypes.byref(Paff), dummy, dummy, dummy, 1 << 30, None) == lq.LQ_ERR_INVALID_ARG
    assert lib.lq_cholesky_inv(dummy, 8, 8, ctypes.c_float(-1.0), dummy, 8, dummy, dummy, dummy, 1 << 30, None) == lq.LQ_ERR_INVALID_ARG
    assert lib.lq_cholesky_inv(dummy, 8, 8, ctypes.c_float(0.01), dummy, 4, dummy, dummy, dummy, 1 << 30, None) == lq.LQ_ERR_INVALID_ARG
    assert lib.lq_cholesky_inv(dummy, 8, 8, ctypes.c_float(0.01), dummy, 8, dummy, dummy, dummy, 8, None) == lq.LQ_ERR_WORKSPACE
    for field, value, frag in (("bits", 5, "bits"), ("bits", 1, "bits"), ("mode", 7, "mode"), ("block", 0, "block"),
                               ("group_size", 64, "per row"), ("kmeans_max_iter", 0, "kmeans")):
        Q = lq.lq_params_default(**{field: value})
        _bad(lib.lq_fit_grid(dummy, 4, 512, 512, dummy, ctypes.byref(Q), dummy, dummy, 1 << 30, None), frag)
    Q = lq.lq_params_default(mode=lq.LQ_GRID_AFFINE, group_size=100)
    _bad(lib.lq_fit_grid(dummy, 4, 512, 512, dummy, ctypes.byref(Q), dummy, dummy, 1 << 30, None), "divide")
    Q = lq.lq_params_default(mode=lq.LQ_GRID_AFFINE, t_override=2000)
    _bad(lib.lq_fit_grid(dummy, 4, 512, 512, dummy, ctypes.byref(Q), dummy, dummy, 1 << 30, None), "t=")
    assert lib.lq_fit_grid(dummy, 4, 512, 100, dummy, pp, dummy, dummy, 1 << 30, None) == lq.LQ_ERR_INVALID_ARG
    assert lib.lq_fit_grid(dummy, 4, 20000, 20000, dummy, pp, dummy, dummy, 1 << 30, None) == lq.LQ_ERR_UNSUPPORTED
    Q = lq.lq_params_default(block=100)
    assert lib.lq_quantize_layer(dummy, 4, 512, 512, dummy, 512, dummy, ctypes.byref(Q), dummy, None, dummy, 1 << 30, None) == lq.LQ_ERR_UNSUPPORTED
    assert lib.lq_quantize_layer(dummy, 4, 512, 512, dummy, 512, dummy, pp, None, None, dummy, 1 << 30, None) == lq.LQ_ERR_INVALID_ARG
    assert lib.lq_quantize_layer(dummy, 4, 512, 512, dummy, 512, dummy, pp, dummy, None, dummy, 64, None) == lq.LQ_ERR_WORKSPACE


def test_binding_rejects_cpu_tensors():
    import torch
    H = torch.zeros(4, 4)
    with pytest.raises(TypeError):
        lq.lq_hessian_accumulate(H, torch.zeros(2, 4), None)


def test_host_side_packing_helpers_match_the_oracle():
    """lq_packed_row_bytes and lq_bits_per_weight are host-only computations."""
    from oracle import packing_oracle as po
    import paper_2407_10032_amd as lq
    lq.load()
    for bits in (2, 3, 4):
        for c in (1, 7, 8, 4096, 11008, 16384):
            assert lq.lq_packed_row_bytes(c, bits) == po.packed_row_bytes(c, bits)
            P = lq.lq_params_default(bits=bits, mode=lq.LQ_GRID_NONUNIFORM)
            assert lq.lq_bits_per_weight(3, c, P) == po.bits_per_weight(3, c, bits, "nu")
    P = lq.lq_params_default(bits=4, mode=lq.LQ_GRID_AFFINE, group_size=128)
    assert lq.lq_bits_per_weight(3, 4096, P) == 4.25
    P = lq.lq_params_default(bits=2, mode=lq.LQ_GRID_AFFINE, group_size=64)
    assert lq.lq_bits_per_weight(3, 4096, P) == po.bits_per_weight(3, 4096, 2, "aff", 64) == 2.5
    assert lq.lq_packed_row_bytes(-1, 4) == -1 and lq.lq_packed_row_bytes(8, 0) == -1
    bad = lq.lq_params_default(bits=5)
    assert lq.lq_bits_per_weight(3, 4096, bad) == -1.0


def test_host_streaming_workspace_is_partial_sums_plus_two_chunk_buffers(lib):
    """Layout of the scratch of lq_hessian_accumulate_host: the larger partial-sum scratch of
    the two chunk sizes that occur, then two staging buffers, all 256-byte multiples."""
    def part(c, n):
        return lib.lq_workspace_bytes(lq.LQ_CALL_HESSIAN, 0, c, n, None)
    up = lambda x: (x + 255) // 256 * 256
    for c, n, ch in [(4096, 262144, 16384), (512, 2048, 512), (300, 1000, 384), (64, 10, 100), (11008, 40000, 8192)]:
        whole = min(n, ch)
        tail = n % ch if n > ch else 0
        p = max(part(c, whole), part(c, tail) if tail else 0)
        assert lib.lq_hessian_host_workspace_bytes(c, n, ch) == up(p) + 2 * up(whole * c * 4)
    assert lib.lq_hessian_host_workspace_bytes(0, 10, 10) == 0
    assert lib.lq_hessian_host_workspace_bytes(8, 10, 0) == 0


def test_argument_errors_of_the_calls_beyond_the_pass(lib):
    """Stored form, product, Algorithm 2: every bad argument is refused on the host."""
    P = lq.lq_params_default()
    pp = ctypes.byref(P)
    d = ctypes.c_void_p(256)
    # lq_pack_layer(codes, grid, r, c, P, packed, packed_ld, table, stream)
    assert lib.lq_pack_layer(d, d, 0, 64, pp, d, 32, d, None) == lq.LQ_OK           # no rows
    _bad(lib.lq_pack_layer(None, d, 4, 64, pp, d, 32, d, None), "null")
    assert lib.lq_pack_layer(d, d, 4, 64, pp, d, 31, d, None) == lq.LQ_ERR_INVALID_ARG
    # lq_unpack_layer(packed, packed_ld, table, r, c, P, W_hat, ldw, codes, stream)
    assert lib.lq_unpack_layer(d, 32, d, 0, 64, pp, d, 64, None, None) == lq.LQ_OK
    _bad(lib.lq_unpack_layer(d, 32, None, 4, 64, pp, d, 64, None, None), "null")
    assert lib.lq_unpack_layer(d, 32, d, 4, 64, pp, d, 63, None, None) == lq.LQ_ERR_INVALID_ARG
    # lq_matvec_packed(packed, packed_ld, table, r, c, P, X, nb, Y, stream)
    assert lib.lq_matvec_packed(d, 32, d, 0, 64, pp, d, 1, d, None) == lq.LQ_OK
    assert lib.lq_matvec_packed(d, 32, d, 4, 64, pp, d, 0, d, None) == lq.LQ_OK
    _bad(lib.lq_matvec_packed(d, 32, d, 4, 64, pp, None, 1, d, None), "null")
    assert lib.lq_matvec_packed(d, 16, d, 4, 64, pp, d, 1, d, None) == lq.LQ_ERR_INVALID_ARG     # ld < row bytes
    assert lib.lq_matvec_packed(d, 48, d, 4, 72, pp, d, 1, d, None) == lq.LQ_ERR_UNSUPPORTED     # c % 32
    assert lib.lq_matvec_packed(d, 16384, d, 4, 32768, pp, d, 1, d, None) == lq.LQ_ERR_UNSUPPORTED
    assert lib.lq_matvec_packed(d, 40, d, 4, 64, pp, d, 1, d, None) == lq.LQ_ERR_UNSUPPORTED     # rows not 16-byte aligned
    assert lib.lq_matvec_packed(ctypes.c_void_p(260), 32, d, 4, 64, pp, d, 1, d, None) == lq.LQ_ERR_UNSUPPORTED
    Pa = lq.lq_params_default(bits=4, mode=lq.LQ_GRID_AFFINE, group_size=16)
    assert lib.lq_matvec_packed(d, 32, d, 4, 64, ctypes.byref(Pa), d, 1, d, None) == lq.LQ_ERR_UNSUPPORTED
    # lq_quantize_exact(W, r, c, ldw, Hinv, ldh, grid, P, codes, row_loss, order, ws, ws_bytes, stream)
    assert lib.lq_quantize_exact(d, 0, 8, 8, d, 8, d, pp, d, None, None, d, 1 << 30, None) == lq.LQ_OK
    _bad(lib.lq_quantize_exact(d, 4, 8, 8, None, 8, d, pp, d, None, None, d, 1 << 30, None), "null")
    assert lib.lq_quantize_exact(d, 4, 8, 4, d, 8, d, pp, d, None, None, d, 1 << 30, None) == lq.LQ_ERR_INVALID_ARG
    assert lib.lq_quantize_exact(d, 4, 4096, 4096, d, 4096, d, pp, d, None, None, d, 1 << 30, None) == lq.LQ_ERR_UNSUPPORTED
    assert lib.lq_quantize_exact(d, 4, 8, 8, d, 8, d, pp, d, None, None, d, 8, None) == lq.LQ_ERR_WORKSPACE
    Pg = lq.lq_params_default(bits=4, mode=lq.LQ_GRID_AFFINE, group_size=4)
    assert lib.lq_quantize_exact(d, 4, 8, 8, d, 8, d, ctypes.byref(Pg), d, None, None, d, 1 << 30, None) == lq.LQ_ERR_INVALID_ARG
    # lq_hinv_from_factor(U, ldu, c, Hinv, ldh, stream)
    _bad(lib.lq_hinv_from_factor(None, 8, 8, d, 8, None), "null")
    assert lib.lq_hinv_from_factor(d, 4, 8, d, 8, None) == lq.LQ_ERR_INVALID_ARG


def test_bench_refuses_more_than_one_gpu(repo_root):
    """The path is built for one GPU: asked for more, bench.py says so and runs nothing."""
    import subprocess
    import sys
    p = subprocess.run([sys.executable, os.path.join(repo_root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""
