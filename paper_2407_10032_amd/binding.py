"""ctypes binding of libleanquant.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
include/leanquant.h and takes torch CUDA tensors where the C call takes device
pointers.  Nothing is computed here; PyTorch supplies device memory and the
current stream.  Importing works without the library (so that the package can be
built first); the first call fails loudly if libleanquant.so is missing.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libleanquant.so")

LQ_OK, LQ_ERR_INVALID_ARG, LQ_ERR_NOT_PD, LQ_ERR_UNSUPPORTED, LQ_ERR_WORKSPACE, LQ_ERR_HIP = range(6)
LQ_GRID_NONUNIFORM, LQ_GRID_AFFINE = 0, 1
LQ_CALL_HESSIAN, LQ_CALL_CHOLESKY, LQ_CALL_FIT_GRID, LQ_CALL_QUANTIZE, LQ_CALL_EXACT = range(5)

EXPORTS = ("lq_params_default", "lq_hessian_accumulate", "lq_hessian_accumulate_host",
           "lq_hessian_host_workspace_bytes", "lq_cholesky_inv", "lq_fit_grid",
           "lq_fit_grid_static", "lq_fit_grid_from", "lq_kmeanspp_seed", "lq_quantize_layer", "lq_quantize_exact", "lq_hinv_from_factor", "lq_packed_row_bytes", "lq_bits_per_weight", "lq_pack_layer",
           "lq_unpack_layer", "lq_matvec_packed", "lq_matmul_packed", "lq_workspace_bytes", "lq_last_error", "lq_version")


class lq_params(ctypes.Structure):
    _fields_ = [("bits", ctypes.c_int32), ("mode", ctypes.c_int32), ("group_size", ctypes.c_int32),
                ("block", ctypes.c_int32), ("damp", ctypes.c_float), ("p", ctypes.c_float),
                ("T", ctypes.c_int32), ("t_override", ctypes.c_int32),
                ("kmeans_max_iter", ctypes.c_int32)]


class LeanQuantError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("leanquant status %d: %s" % (status, text))
        self.status = status


_lib = None


def load() -> ctypes.CDLL:
    """Load libleanquant.so (built in-tree by paper_2407_10032_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libleanquant.so is not built: run `python -m paper_2407_10032_amd.build` "
                          "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, sz, fp = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
    pp = ctypes.POINTER(lq_params)
    lib.lq_params_default.argtypes = [pp]
    lib.lq_params_default.restype = None
    lib.lq_hessian_accumulate.argtypes = [vp, i64, vp, i64, i64, i64, vp, sz, vp]
    lib.lq_hessian_accumulate.restype = ctypes.c_int
    lib.lq_hessian_accumulate_host.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, sz, vp]
    lib.lq_hessian_accumulate_host.restype = ctypes.c_int
    lib.lq_hessian_host_workspace_bytes.argtypes = [i64, i64, i64]
    lib.lq_hessian_host_workspace_bytes.restype = sz
    lib.lq_cholesky_inv.argtypes = [vp, i64, i64, fp, vp, i64, vp, vp, vp, sz, vp]
    lib.lq_cholesky_inv.restype = ctypes.c_int
    lib.lq_fit_grid.argtypes = [vp, i64, i64, i64, vp, pp, vp, vp, sz, vp]
    lib.lq_fit_grid.restype = ctypes.c_int
    lib.lq_fit_grid_static.argtypes = [vp, i64, i64, i64, vp, pp, vp, vp]
    lib.lq_fit_grid_static.restype = ctypes.c_int
    lib.lq_fit_grid_from.argtypes = [vp, i64, i64, i64, vp, pp, vp, vp, vp, sz, vp]
    lib.lq_fit_grid_from.restype = ctypes.c_int
    lib.lq_kmeanspp_seed.argtypes = [vp, i64, i64, i64, vp, pp, vp, vp, vp, sz, vp]
    lib.lq_kmeanspp_seed.restype = ctypes.c_int
    lib.lq_quantize_layer.argtypes = [vp, i64, i64, i64, vp, i64, vp, pp, vp, vp, vp, sz, vp]
    lib.lq_quantize_layer.restype = ctypes.c_int
    lib.lq_quantize_exact.argtypes = [vp, i64, i64, i64, vp, i64, vp, pp, vp, vp, vp, vp, sz, vp]
    lib.lq_quantize_exact.restype = ctypes.c_int
    lib.lq_hinv_from_factor.argtypes = [vp, i64, i64, vp, i64, vp]
    lib.lq_hinv_from_factor.restype = ctypes.c_int
    lib.lq_packed_row_bytes.argtypes = [i64, ctypes.c_int32]
    lib.lq_packed_row_bytes.restype = i64
    lib.lq_bits_per_weight.argtypes = [i64, i64, pp]
    lib.lq_bits_per_weight.restype = ctypes.c_double
    lib.lq_pack_layer.argtypes = [vp, vp, i64, i64, pp, vp, i64, vp, vp]
    lib.lq_pack_layer.restype = ctypes.c_int
    lib.lq_unpack_layer.argtypes = [vp, i64, vp, i64, i64, pp, vp, i64, vp, vp]
    lib.lq_unpack_layer.restype = ctypes.c_int
    lib.lq_matvec_packed.argtypes = [vp, i64, vp, i64, i64, pp, vp, i64, vp, vp]
    lib.lq_matvec_packed.restype = ctypes.c_int
    lib.lq_matmul_packed.argtypes = [vp, i64, vp, i64, i64, pp, vp, i64, vp, vp]
    lib.lq_matmul_packed.restype = ctypes.c_int
    lib.lq_workspace_bytes.argtypes = [ctypes.c_int, i64, i64, i64, pp]
    lib.lq_workspace_bytes.restype = sz
    lib.lq_last_error.argtypes = []
    lib.lq_last_error.restype = ctypes.c_char_p
    lib.lq_version.argtypes = []
    lib.lq_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != LQ_OK:
        raise LeanQuantError(status, load().lq_last_error().decode())


def _ptr(t: Optional[torch.Tensor], dtype: torch.dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError("%s must be a CUDA (HIP) tensor" % name)
    if t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    return t.data_ptr()


def _ld(t: torch.Tensor, name: str) -> int:
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("%s must be a 2-D tensor with unit column stride" % name)
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def _dense(t: Optional[torch.Tensor], shape, name: str) -> None:
    """The C side reads these with their natural leading dimension: refuse views."""
    if t is None:
        return
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)


def grid_shape(P: "lq_params", r: int, c: int):
    """Shape of the grid tensor lq_fit_grid writes for P: [r x 2^b] or [r x c/group x 2]."""
    if P.mode == LQ_GRID_NONUNIFORM:
        return (r, 1 << P.bits)
    g = P.group_size if P.group_size > 0 else c
    return (r, c // g, 2)


def params_for(cfg, **overrides) -> "lq_params":
    """lq_params from any object with the fields mode ("nu" / "aff"), bits, group_size, block,
    damp, p, T (such as a layer configuration of lq_synth)."""
    kw = dict(bits=cfg.bits, mode=LQ_GRID_AFFINE if cfg.mode == "aff" else LQ_GRID_NONUNIFORM,
              group_size=cfg.group_size, block=cfg.block, damp=cfg.damp, p=cfg.p, T=cfg.T)
    kw.update(overrides)
    return lq_params_default(**kw)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ws(ws: Optional[torch.Tensor]):
    if ws is None:
        return None, 0
    if not ws.is_cuda or ws.dtype != torch.uint8 or not ws.is_contiguous():
        raise TypeError("workspace must be a contiguous CUDA uint8 tensor")
    return ws.data_ptr(), ws.numel()


def lq_params_default(**overrides) -> lq_params:
    P = lq_params()
    load().lq_params_default(ctypes.byref(P))
    for k, v in overrides.items():
        if not hasattr(P, k):
            raise AttributeError(k)
        setattr(P, k, v)
    return P


def lq_workspace_bytes(which_call: int, r: int, c: int, n_tokens: int = 0,
                       P: Optional[lq_params] = None) -> int:
    return int(load().lq_workspace_bytes(which_call, r, c, n_tokens, ctypes.byref(P) if P is not None else None))


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """Device scratch for a call (torch's allocator returns >= 256-byte aligned blocks)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def lq_hessian_accumulate(H: torch.Tensor, X: torch.Tensor, ws: torch.Tensor) -> None:
    """H += 2 X^T X.  H [c x c] fp32, X [n_tokens x c] fp32."""
    c = H.shape[0]
    wp, wn = _ws(ws)
    _check(load().lq_hessian_accumulate(_ptr(H, torch.float32, "H"), _ld(H, "H"),
                                        _ptr(X, torch.float32, "X"), X.shape[0], c, _ld(X, "X"),
                                        wp, wn, _stream()))


def lq_hessian_host_workspace_bytes(c: int, n_tokens: int, chunk_tokens: int) -> int:
    return int(load().lq_hessian_host_workspace_bytes(c, n_tokens, chunk_tokens))


def lq_hessian_accumulate_host(H: torch.Tensor, X_host: torch.Tensor, chunk_tokens: int,
                               ws: torch.Tensor) -> None:
    """H += 2 X^T X with X [n_tokens x c] fp32 in host memory (pinned for overlap); the
    tensor must stay alive and unchanged until the current stream has finished."""
    c = H.shape[0]
    if X_host.is_cuda or X_host.dtype != torch.float32:
        raise TypeError("X_host must be a float32 CPU tensor")
    wp, wn = _ws(ws)
    _check(load().lq_hessian_accumulate_host(_ptr(H, torch.float32, "H"), _ld(H, "H"),
                                             X_host.data_ptr(), X_host.shape[0], c, _ld(X_host, "X_host"),
                                             int(chunk_tokens), wp, wn, _stream()))


def lq_cholesky_inv(H: torch.Tensor, damp: float, U: torch.Tensor, hinv_diag: torch.Tensor,
                    info: torch.Tensor, ws: torch.Tensor) -> None:
    c = H.shape[0]
    wp, wn = _ws(ws)
    _dense(hinv_diag, (c,), "hinv_diag")
    _check(load().lq_cholesky_inv(_ptr(H, torch.float32, "H"), _ld(H, "H"), c, float(damp),
                                  _ptr(U, torch.float32, "U"), _ld(U, "U"),
                                  _ptr(hinv_diag, torch.float32, "hinv_diag"),
                                  _ptr(info, torch.int32, "info"), wp, wn, _stream()))


def lq_fit_grid(W: torch.Tensor, hinv_diag: torch.Tensor, P: lq_params, grid: torch.Tensor,
                ws: torch.Tensor) -> None:
    r, c = W.shape
    wp, wn = _ws(ws)
    _dense(hinv_diag, (c,), "hinv_diag")
    _dense(grid, grid_shape(P, r, c), "grid")
    _check(load().lq_fit_grid(_ptr(W, torch.float32, "W"), r, c, _ld(W, "W"),
                              _ptr(hinv_diag, torch.float32, "hinv_diag"), ctypes.byref(P),
                              _ptr(grid, torch.float32, "grid"), wp, wn, _stream()))


def lq_fit_grid_static(W: torch.Tensor, hinv_diag: torch.Tensor, P: lq_params, grid: torch.Tensor) -> None:
    """lq_fit_grid without a workspace argument (the library's built-in scratch, c <= 16384)."""
    r, c = W.shape
    _dense(hinv_diag, (c,), "hinv_diag")
    _dense(grid, grid_shape(P, r, c), "grid")
    _check(load().lq_fit_grid_static(_ptr(W, torch.float32, "W"), r, c, _ld(W, "W"),
                                     _ptr(hinv_diag, torch.float32, "hinv_diag"), ctypes.byref(P),
                                     _ptr(grid, torch.float32, "grid"), _stream()))


def lq_fit_grid_from(W: torch.Tensor, hinv_diag: torch.Tensor, P: lq_params,
                     init_grid: Optional[torch.Tensor], grid: torch.Tensor, ws: torch.Tensor) -> None:
    r, c = W.shape
    wp, wn = _ws(ws)
    _dense(hinv_diag, (c,), "hinv_diag")
    _dense(grid, grid_shape(P, r, c), "grid")
    if init_grid is not None:
        # (with an affine P the C side refuses a starting grid; only a view is refused here)
        _dense(init_grid, (r, 1 << P.bits) if P.mode == LQ_GRID_NONUNIFORM else tuple(init_grid.shape), "init_grid")
    _check(load().lq_fit_grid_from(_ptr(W, torch.float32, "W"), r, c, _ld(W, "W"),
                                   _ptr(hinv_diag, torch.float32, "hinv_diag"), ctypes.byref(P),
                                   _ptr(init_grid, torch.float32, "init_grid"),
                                   _ptr(grid, torch.float32, "grid"), wp, wn, _stream()))


def lq_kmeanspp_seed(W: torch.Tensor, hinv_diag: torch.Tensor, P: lq_params, u: torch.Tensor,
                     grid_init: torch.Tensor, ws: torch.Tensor) -> None:
    """k-means++ seeding of the non-uniform grids; u [r x 2^b] float64 uniforms in [0, 1)."""
    r, c = W.shape
    wp, wn = _ws(ws)
    _dense(hinv_diag, (c,), "hinv_diag")
    _dense(u, (r, 1 << P.bits), "u")
    _dense(grid_init, (r, 1 << P.bits), "grid_init")
    _check(load().lq_kmeanspp_seed(_ptr(W, torch.float32, "W"), r, c, _ld(W, "W"),
                                   _ptr(hinv_diag, torch.float32, "hinv_diag"), ctypes.byref(P),
                                   _ptr(u, torch.float64, "u"), _ptr(grid_init, torch.float32, "grid_init"),
                                   wp, wn, _stream()))


def lq_quantize_layer(W: torch.Tensor, U: torch.Tensor, grid: torch.Tensor, P: lq_params,
                      codes: torch.Tensor, row_loss: Optional[torch.Tensor], ws: torch.Tensor) -> None:
    r, c = W.shape
    wp, wn = _ws(ws)
    _dense(grid, grid_shape(P, r, c), "grid")
    _dense(codes, (r, c), "codes")
    _dense(row_loss, (r,), "row_loss")
    _check(load().lq_quantize_layer(_ptr(W, torch.float32, "W"), r, c, _ld(W, "W"),
                                    _ptr(U, torch.float32, "U"), _ld(U, "U"),
                                    _ptr(grid, torch.float32, "grid"), ctypes.byref(P),
                                    _ptr(codes, torch.uint8, "codes"),
                                    _ptr(row_loss, torch.float32, "row_loss"), wp, wn, _stream()))


def lq_quantize_exact(W: torch.Tensor, Hinv: torch.Tensor, grid: torch.Tensor, P: lq_params,
                      codes: torch.Tensor, order: Optional[torch.Tensor],
                      row_loss: Optional[torch.Tensor], ws: torch.Tensor) -> None:
    r, c = W.shape
    wp, wn = _ws(ws)
    _dense(grid, grid_shape(P, r, c), "grid")
    _dense(codes, (r, c), "codes")
    _dense(order, (r, c), "order")
    _dense(row_loss, (r,), "row_loss")
    _check(load().lq_quantize_exact(_ptr(W, torch.float32, "W"), r, c, _ld(W, "W"),
                                    _ptr(Hinv, torch.float64, "Hinv"), _ld(Hinv, "Hinv"),
                                    _ptr(grid, torch.float32, "grid"), ctypes.byref(P),
                                    _ptr(codes, torch.uint8, "codes"), _ptr(order, torch.int32, "order"),
                                    _ptr(row_loss, torch.float32, "row_loss"), wp, wn, _stream()))


def lq_hinv_from_factor(U: torch.Tensor, Hinv: torch.Tensor) -> None:
    c = U.shape[0]
    _check(load().lq_hinv_from_factor(_ptr(U, torch.float32, "U"), _ld(U, "U"), c,
                                      _ptr(Hinv, torch.float64, "Hinv"), _ld(Hinv, "Hinv"), _stream()))


def lq_packed_row_bytes(c: int, bits: int) -> int:
    return int(load().lq_packed_row_bytes(c, bits))


def lq_bits_per_weight(r: int, c: int, P: lq_params) -> float:
    return float(load().lq_bits_per_weight(r, c, ctypes.byref(P)))


def lq_pack_layer(codes: torch.Tensor, grid: torch.Tensor, P: lq_params, packed: torch.Tensor,
                  table: torch.Tensor) -> None:
    """codes [r x c] uint8 + grid -> packed [r x >= row_bytes] uint8, table int16 (bit patterns)."""
    r, c = codes.shape
    if not codes.is_contiguous():
        raise ValueError("codes must be contiguous (leading dimension c)")
    _check(load().lq_pack_layer(_ptr(codes, torch.uint8, "codes"), _ptr(grid, torch.float32, "grid"),
                                r, c, ctypes.byref(P), _ptr(packed, torch.uint8, "packed"),
                                _ld(packed, "packed"), _ptr(table, torch.int16, "table"), _stream()))


def lq_unpack_layer(packed: torch.Tensor, table: torch.Tensor, c: int, P: lq_params,
                    W_hat: torch.Tensor, codes: Optional[torch.Tensor]) -> None:
    r = W_hat.shape[0]
    if codes is not None and not codes.is_contiguous():
        raise ValueError("codes must be contiguous (leading dimension c)")
    _check(load().lq_unpack_layer(_ptr(packed, torch.uint8, "packed"), _ld(packed, "packed"),
                                  _ptr(table, torch.int16, "table"), r, c, ctypes.byref(P),
                                  _ptr(W_hat, torch.float32, "W_hat"), _ld(W_hat, "W_hat"),
                                  _ptr(codes, torch.uint8, "codes"), _stream()))


def lq_matvec_packed(packed: torch.Tensor, table: torch.Tensor, c: int, P: lq_params,
                     X: torch.Tensor, Y: torch.Tensor) -> None:
    """Y [nb x r] = X [nb x c] times the transposed stored layer."""
    r = packed.shape[0]
    nb = X.shape[0]
    if not X.is_contiguous() or not Y.is_contiguous() or X.shape[1] != c or tuple(Y.shape) != (nb, r):
        raise ValueError("X must be contiguous [nb x c] and Y contiguous [nb x r]")
    _check(load().lq_matvec_packed(_ptr(packed, torch.uint8, "packed"), _ld(packed, "packed"),
                                   _ptr(table, torch.int16, "table"), r, c, ctypes.byref(P),
                                   _ptr(X, torch.float32, "X"), nb, _ptr(Y, torch.float32, "Y"), _stream()))


def lq_matmul_packed(packed: torch.Tensor, table: torch.Tensor, c: int, P: lq_params,
                     X: torch.Tensor, Y: torch.Tensor) -> None:
    """Y [nb x r] = X [nb x c] times the transposed stored layer, batched form (fp32 MFMA)."""
    r = packed.shape[0]
    nb = X.shape[0]
    if not X.is_contiguous() or not Y.is_contiguous() or X.shape[1] != c or tuple(Y.shape) != (nb, r):
        raise ValueError("X must be contiguous [nb x c] and Y contiguous [nb x r]")
    _check(load().lq_matmul_packed(_ptr(packed, torch.uint8, "packed"), _ld(packed, "packed"),
                                   _ptr(table, torch.int16, "table"), r, c, ctypes.byref(P),
                                   _ptr(X, torch.float32, "X"), nb, _ptr(Y, torch.float32, "Y"), _stream()))


def lq_last_error() -> str:
    return load().lq_last_error().decode()


def lq_version() -> str:
    return load().lq_version().decode()
