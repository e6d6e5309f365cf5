"""Thin ctypes binding of libslope.so (the C ABI declared in include/slope.h).

Argument marshalling only: every step of the path runs in the HIP kernels.  PyTorch supplies
device memory and the current stream.  There is no fallback: if the library is missing or a
call returns an error status, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SLOPE_LIB", os.path.join(HERE, "libslope.so"))

SLOPE_OK = 0
SLOPE_ERR_NULL = -1
SLOPE_ERR_SHAPE = -2
SLOPE_ERR_ALIGN = -3
SLOPE_ERR_UNSUPPORTED = -4
SLOPE_ERR_HIP = -5
SLOPE_ERR_WORKSPACE = -6
SLOPE_STATIC_SCRATCH_BYTES = 72 << 20      # include/slope.h
# slope_call_id
(SLOPE_CALL_PRUNE_ROWS, SLOPE_CALL_DOUBLE_PRUNE, SLOPE_CALL_SPMM_FWD, SLOPE_CALL_SPMM_BWD_X, SLOPE_CALL_WGRAD_MASKED,
 SLOPE_CALL_WGRAD_MASKED_WS, SLOPE_CALL_SPMM_BWD_X_ADAPTER, SLOPE_CALL_WGRAD_ADAPTER,
 SLOPE_CALL_WGRAD_MASKED_T) = range(1, 10)

_P, _I64, _INT, _SZ = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t

# name -> (restype, argtypes); mirrors include/slope.h one to one
SIGNATURES = {
    "slope_version": (_INT, []),
    "slope_last_hip_error": (_INT, []),
    "slope_status_string": (ctypes.c_char_p, [_INT]),
    "slope_packed_vals_bytes": (_SZ, [_I64, _I64]),
    "slope_packed_meta_bytes": (_SZ, [_I64, _I64]),
    "slope_mask_bytes": (_SZ, [_I64, _I64]),
    "slope_workspace_bytes": (_SZ, [_INT, _I64, _I64, _I64, _I64]),
    "slope_spmm_fwd_workspace_bytes": (_SZ, [_I64, _I64, _I64, _I64]),
    "slope_prune_rows": (_INT, [_P, _I64, _I64, _INT, _INT, _P, _P, _P, _P]),
    "slope_double_prune": (_INT, [_P, _P, _I64, _I64, _P, _P, _P, _P]),
    "slope_spmm_fwd": (_INT, [_P, _I64, _P, _P, _I64, _I64, _P, _P, _I64, _P, _P, _P]),
    "slope_spmm_fwd_ws": (_INT, [_P, _I64, _P, _P, _I64, _I64, _P, _P, _I64, _P, _P, _SZ, _P]),
    "slope_spmm_fwd_static": (_INT, [_P, _I64, _P, _P, _I64, _I64, _P, _P, _I64, _P, _P]),
    "slope_spmm_bwd_x": (_INT, [_P, _I64, _P, _P, _I64, _I64, _P, _P]),
    "slope_wgrad_workspace_bytes": (_SZ, [_I64, _I64, _I64]),
    "slope_wgrad_masked": (_INT, [_P, _P, _I64, _P, _I64, _I64, _P, _P]),
    "slope_wgrad_masked_ws": (_INT, [_P, _P, _I64, _P, _I64, _I64, _P, _P, _SZ, _P]),
    "slope_token_copy_bytes": (_SZ, [_I64, _I64]),
    "slope_transpose_tokens": (_INT, [_P, _I64, _I64, _P, _SZ, _P]),
    "slope_wgrad_masked_t": (_INT, [_P, _P, _I64, _P, _I64, _I64, _P, _P, _SZ, _P]),
    "slope_spmm_bwd_x_adapter_workspace_bytes": (_SZ, [_I64, _I64]),
    "slope_spmm_bwd_x_adapter": (_INT, [_P, _I64, _P, _P, _I64, _I64, _P, _P, _I64, _P, _P, _SZ, _P]),
    "slope_wgrad_adapter_workspace_bytes": (_SZ, [_I64, _I64, _I64, _I64]),
    "slope_wgrad_adapter": (_INT, [_P, _P, _I64, _P, _I64, _I64, _P, _P, _I64, _P, _P, _P, _P, _SZ, _P]),
    "slope_prune_mask": (_INT, [_P, _I64, _I64, _INT, _INT, _INT, _P, _P, _P, _P, _P]),
    "slope_gemm_tn": (_INT, [_P, _I64, _P, _I64, _I64, _P, _P]),
    "slope_sparse_add": (_INT, [_P, _P, _I64, _I64, ctypes.c_float, ctypes.c_float, _P, _P]),
    "slope_update_sparse": (_INT, [_P, _P, _I64, _I64, _P, _P, _P, _P]),
    "slope_ceiling_min_bytes": (_SZ, []),
    "slope_ceiling": (_INT, [_INT, _P, _SZ, _INT, _P, _P]),
    "slope_tile_order": (_I64, [_I64, _I64, _P, _P, _I64]),
    "slope_spmm_fwd_plan": (_INT, [_I64, _I64, _I64, _I64, _INT, _P]),
}

_lib = None


class SlopeError(RuntimeError):
    def __init__(self, call: str, status: int):
        self.status = status
        msg = lib().slope_status_string(status).decode()
        if status == SLOPE_ERR_HIP:
            msg += " (hipError_t %d)" % lib().slope_last_hip_error()
        super().__init__("%s failed with status %d: %s" % (call, status, msg))


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (run paper_2405_16325_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_2405_16325_amd.build`" % LIB_PATH)
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(call: str, status: int):
    if status != SLOPE_OK:
        raise SlopeError(call, status)


def _dev(*tensors):
    for t in tensors:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")


def _want(t, dtype, shape, what):
    """A raw pointer is all the library sees: dtype, shape, device and layout are checked here."""
    if t is None:
        raise ValueError("%s is missing" % what)
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("%s must be a contiguous device tensor" % what)
    if t.dtype != dtype:
        raise ValueError("%s must be %s, not %s" % (what, dtype, t.dtype))
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, not %s" % (what, tuple(shape), tuple(t.shape)))
    return t


def _scratch(ws, nbytes, device, what):
    """The caller's workspace (checked for size) or a fresh one; None when no scratch is needed or given."""
    if ws is None:
        return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device) if nbytes > 0 else None
    if not ws.is_cuda or not ws.is_contiguous() or ws.dtype != torch.uint8:
        raise ValueError("%s must be a contiguous uint8 device tensor" % what)
    if ws.numel() < nbytes:
        raise ValueError("%s holds %d bytes, the call needs %d" % (what, ws.numel(), nbytes))
    return ws


BF16, U8 = torch.bfloat16, torch.uint8


def slope_workspace_bytes(call_id: int, b: int, d_in: int, d_out: int, r: int = 0) -> int:
    return int(lib().slope_workspace_bytes(call_id, b, d_in, d_out, r))


def slope_prune_rows(W: torch.Tensor, want_mask: bool = False, out=None):
    """W bf16[d_out, d_in] -> (vals bf16[d_out, d_in/2], meta u8[d_out, d_in/8], mask u8 or None)."""
    _dev(W)
    if W.dim() != 2 or W.dtype != BF16:
        raise ValueError("W must be a bf16 matrix")
    d_out, d_in = W.shape
    if out is None:
        vals = torch.empty((d_out, d_in // 2), dtype=BF16, device=W.device)
        meta = torch.empty((d_out, d_in // 8), dtype=U8, device=W.device)
        mask = torch.empty((d_out, d_in // 8), dtype=U8, device=W.device) if want_mask else None
    else:
        vals, meta, mask = out
        _want(vals, BF16, (d_out, d_in // 2), "vals")
        _want(meta, U8, (d_out, d_in // 8), "meta")
        if mask is not None:
            _want(mask, U8, (d_out, d_in // 8), "mask")
    _check("slope_prune_rows", lib().slope_prune_rows(_ptr(W), d_out, d_in, 2, 4, _ptr(vals), _ptr(meta),
                                                      _ptr(mask), _stream()))
    return vals, meta, mask


def _packed(vals, meta, what):
    """(rows, cols) of a packed pair after checking that the two tensors belong together."""
    if vals is None or vals.dim() != 2:
        raise ValueError("%s values must be a matrix" % what)
    rows, cols = vals.shape[0], vals.shape[1] * 2
    _want(vals, BF16, (rows, cols // 2), what + " values")
    _want(meta, U8, (rows, cols // 8), what + " metadata")
    return rows, cols


def slope_double_prune(vals: torch.Tensor, meta: torch.Tensor, want_mask: bool = False, out=None):
    """Packed W^R -> (valsT bf16[d_in, d_out/2], metaT u8[d_in, d_out/8], maskrc u8[d_out, d_in/8] or None)."""
    d_out, d_in = _packed(vals, meta, "W^R")
    if out is None:
        vals_t = torch.empty((d_in, d_out // 2), dtype=BF16, device=vals.device)
        meta_t = torch.empty((d_in, d_out // 8), dtype=U8, device=vals.device)
        mask = torch.empty((d_out, d_in // 8), dtype=U8, device=vals.device) if want_mask else None
    else:
        vals_t, meta_t, mask = out
        _want(vals_t, BF16, (d_in, d_out // 2), "valsT")
        _want(meta_t, U8, (d_in, d_out // 8), "metaT")
        if mask is not None:
            _want(mask, U8, (d_out, d_in // 8), "maskrc")
    _check("slope_double_prune", lib().slope_double_prune(_ptr(vals), _ptr(meta), d_out, d_in, _ptr(vals_t),
                                                          _ptr(meta_t), _ptr(mask), _stream()))
    return vals_t, meta_t, mask


def slope_spmm_fwd_workspace_bytes(b: int, d_in: int, d_out: int, r: int) -> int:
    return int(lib().slope_spmm_fwd_workspace_bytes(b, d_in, d_out, r))


def _fwd_args(X, vals, meta, L, R, out):
    d_out, d_in = _packed(vals, meta, "W^R")
    if X is None or X.dim() != 2:
        raise ValueError("X must be a matrix")
    b = X.shape[0]
    _want(X, BF16, (b, d_in), "X")
    r = 0
    if L is not None or R is not None:
        if L is None or R is None or L.dim() != 2:
            raise ValueError("L and R come together")
        r = L.shape[1]
        _want(L, BF16, (d_in, r), "L")
        _want(R, BF16, (r, d_out), "R")
    if out is not None:
        _want(out, BF16, (b, d_out), "out")
    return b, d_in, d_out, r


def slope_spmm_fwd(X: torch.Tensor, vals: torch.Tensor, meta: torch.Tensor, L=None, R=None, out=None,
                   workspace=None):
    """Y = X (W^R)^T [+ (X L) R].  X bf16[b, d_in]; packed W^R; L bf16[d_in, r]; R bf16[r, d_out].
    workspace: a uint8 device tensor of slope_spmm_fwd_workspace_bytes(...) bytes, or None (allocated here)."""
    b, d_in, d_out, r = _fwd_args(X, vals, meta, L, R, out)
    nbytes = slope_spmm_fwd_workspace_bytes(b, d_in, d_out, r)
    workspace = _scratch(workspace, nbytes, X.device, "workspace")
    Y = out if out is not None else torch.empty((b, d_out), dtype=BF16, device=X.device)
    _check("slope_spmm_fwd_ws", lib().slope_spmm_fwd_ws(_ptr(X), b, _ptr(vals), _ptr(meta), d_out, d_in, _ptr(L), _ptr(R),
                                                        r, _ptr(Y), _ptr(workspace),
                                                        0 if workspace is None else workspace.numel(), _stream()))
    return Y


def slope_spmm_fwd_static(X: torch.Tensor, vals: torch.Tensor, meta: torch.Tensor, L=None, R=None, out=None):
    """slope_spmm_fwd on the library's own scratch buffer: the call itself allocates nothing (pass `out`
    to keep this wrapper from allocating Y)."""
    b, d_in, d_out, r = _fwd_args(X, vals, meta, L, R, out)
    Y = out if out is not None else torch.empty((b, d_out), dtype=BF16, device=X.device)
    _check("slope_spmm_fwd_static", lib().slope_spmm_fwd_static(_ptr(X), b, _ptr(vals), _ptr(meta), d_out, d_in,
                                                                _ptr(L), _ptr(R), r, _ptr(Y), _stream()))
    return Y


def slope_spmm_bwd_x(dY: torch.Tensor, vals_t: torch.Tensor, meta_t: torch.Tensor, out=None):
    """dX = dY W^{R,C}.  dY bf16[b, d_out]; packed (W^{R,C})^T with rows = d_in."""
    d_in, d_out = _packed(vals_t, meta_t, "(W^{R,C})^T")
    if dY is None or dY.dim() != 2:
        raise ValueError("dY must be a matrix")
    b = dY.shape[0]
    _want(dY, BF16, (b, d_out), "dY")
    dX = _want(out, BF16, (b, d_in), "out") if out is not None else torch.empty((b, d_in), dtype=BF16, device=dY.device)
    _check("slope_spmm_bwd_x", lib().slope_spmm_bwd_x(_ptr(dY), b, _ptr(vals_t), _ptr(meta_t), d_out, d_in, _ptr(dX),
                                                      _stream()))
    return dX


def slope_wgrad_workspace_bytes(b: int, d_in: int, d_out: int) -> int:
    return int(lib().slope_wgrad_workspace_bytes(b, d_in, d_out))


def _wgrad_args(dY, X, meta, out):
    if dY is None or X is None or meta is None or dY.dim() != 2 or X.dim() != 2 or meta.dim() != 2:
        raise ValueError("dY, X and meta must be matrices")
    b, d_out = dY.shape
    d_in = X.shape[1]
    _want(dY, BF16, (b, d_out), "dY")
    _want(X, BF16, (b, d_in), "X")
    _want(meta, U8, (d_out, d_in // 8), "meta")
    G = _want(out, BF16, (d_out, d_in // 2), "out") if out is not None \
        else torch.empty((d_out, d_in // 2), dtype=BF16, device=dY.device)
    return b, d_in, d_out, G


def slope_wgrad_masked(dY: torch.Tensor, X: torch.Tensor, meta: torch.Tensor, out=None, workspace="auto"):
    """dW = dY^T X at W^R's kept positions, packed bf16[d_out, d_in/2].
    workspace: None = slope_wgrad_masked (no scratch, in-place kernel); a uint8 device tensor or "auto"
    (allocated here) = slope_wgrad_masked_ws (token-contiguous copies in the workspace)."""
    b, d_in, d_out, G = _wgrad_args(dY, X, meta, out)
    if workspace is None:
        _check("slope_wgrad_masked", lib().slope_wgrad_masked(_ptr(dY), _ptr(X), b, _ptr(meta), d_out, d_in, _ptr(G),
                                                              _stream()))
        return G
    nbytes = slope_wgrad_workspace_bytes(b, d_in, d_out)
    workspace = _scratch(None if isinstance(workspace, str) else workspace, nbytes, dY.device, "workspace")
    _check("slope_wgrad_masked_ws", lib().slope_wgrad_masked_ws(_ptr(dY), _ptr(X), b, _ptr(meta), d_out, d_in, _ptr(G),
                                                                _ptr(workspace), workspace.numel(), _stream()))
    return G


def slope_token_copy_bytes(b: int, d: int) -> int:
    return int(lib().slope_token_copy_bytes(b, d))


def slope_transpose_tokens(A: torch.Tensor, out=None):
    """Token-contiguous copy of an activation or output gradient A bf16[b, d] for slope_wgrad_masked_t;
    returns the uint8 buffer that holds it (layout private to the library)."""
    if A is None or A.dim() != 2:
        raise ValueError("A must be a matrix")
    b, d = A.shape
    _want(A, BF16, (b, d), "A")
    At = _scratch(out, slope_token_copy_bytes(b, d), A.device, "out")
    _check("slope_transpose_tokens", lib().slope_transpose_tokens(_ptr(A), b, d, _ptr(At), At.numel(), _stream()))
    return At


def slope_wgrad_masked_t(dYt: torch.Tensor, Xt: torch.Tensor, b: int, meta: torch.Tensor, out=None, workspace="auto"):
    """dW from copies made by slope_transpose_tokens (dYt of a [b, d_out], Xt of a [b, d_in] tensor).
    workspace: "auto" (allocated here when the shape wants one), None (no cut of the last partial round
    of tiles) or a uint8 tensor of slope_workspace_bytes(SLOPE_CALL_WGRAD_MASKED_T, b, d_in, d_out) bytes."""
    if meta is None or meta.dim() != 2:
        raise ValueError("meta must be a matrix")
    d_out, d_in = meta.shape[0], meta.shape[1] * 8
    _want(meta, U8, (d_out, d_in // 8), "meta")
    _scratch(dYt, slope_token_copy_bytes(b, d_out), meta.device, "dYt")
    _scratch(Xt, slope_token_copy_bytes(b, d_in), meta.device, "Xt")
    need = slope_workspace_bytes(SLOPE_CALL_WGRAD_MASKED_T, b, d_in, d_out)
    ws = None
    if workspace is not None and need:
        ws = _scratch(None if isinstance(workspace, str) else workspace, need, meta.device, "workspace")
    G = _want(out, BF16, (d_out, d_in // 2), "out") if out is not None \
        else torch.empty((d_out, d_in // 2), dtype=BF16, device=meta.device)
    _check("slope_wgrad_masked_t", lib().slope_wgrad_masked_t(_ptr(dYt), _ptr(Xt), b, _ptr(meta), d_out, d_in, _ptr(G),
                                                              _ptr(ws), ws.numel() if ws is not None else 0, _stream()))
    return G


def slope_spmm_bwd_x_adapter(dY, vals_t, meta_t, L, R, out=None, workspace=None):
    """dX = dY W^{R,C} + (dY R^T) L^T.  L bf16[d_in, r]; R bf16[r, d_out]."""
    d_in, d_out = _packed(vals_t, meta_t, "(W^{R,C})^T")
    if dY is None or dY.dim() != 2 or L is None or L.dim() != 2:
        raise ValueError("dY and L must be matrices")
    b, r = dY.shape[0], L.shape[1]
    _want(dY, BF16, (b, d_out), "dY")
    _want(L, BF16, (d_in, r), "L")
    _want(R, BF16, (r, d_out), "R")
    dX = _want(out, BF16, (b, d_in), "out") if out is not None else torch.empty((b, d_in), dtype=BF16, device=dY.device)
    workspace = _scratch(workspace, int(lib().slope_spmm_bwd_x_adapter_workspace_bytes(b, r)), dY.device, "workspace")
    _check("slope_spmm_bwd_x_adapter",
           lib().slope_spmm_bwd_x_adapter(_ptr(dY), b, _ptr(vals_t), _ptr(meta_t), d_out, d_in, _ptr(L), _ptr(R), r,
                                          _ptr(dX), _ptr(workspace), workspace.numel(), _stream()))
    return dX


def slope_wgrad_adapter_workspace_bytes(b: int, d_in: int, d_out: int, r: int) -> int:
    return int(lib().slope_wgrad_adapter_workspace_bytes(b, d_in, d_out, r))


def slope_wgrad_adapter(dY, X, meta, L, R, out=None, workspace=None):
    """(dW packed, dL, dR) of a layer with adapters; one call, shared token-contiguous copies."""
    b, d_in, d_out, _ = _wgrad_args(dY, X, meta, None if out is None else out[0])
    if L is None or L.dim() != 2:
        raise ValueError("L must be a matrix")
    r = L.shape[1]
    _want(L, BF16, (d_in, r), "L")
    _want(R, BF16, (r, d_out), "R")
    if out is None:
        out = (torch.empty((d_out, d_in // 2), dtype=BF16, device=dY.device),
               torch.empty((d_in, r), dtype=BF16, device=dY.device),
               torch.empty((r, d_out), dtype=BF16, device=dY.device))
    G, dL, dR = out
    _want(G, BF16, (d_out, d_in // 2), "dW")
    _want(dL, BF16, (d_in, r), "dL")
    _want(dR, BF16, (r, d_out), "dR")
    workspace = _scratch(workspace, slope_wgrad_adapter_workspace_bytes(b, d_in, d_out, r), dY.device, "workspace")
    _check("slope_wgrad_adapter",
           lib().slope_wgrad_adapter(_ptr(dY), _ptr(X), b, _ptr(meta), d_out, d_in, _ptr(L), _ptr(R), r, _ptr(G),
                                     _ptr(dL), _ptr(dR), _ptr(workspace), workspace.numel(), _stream()))
    return G, dL, dR


def slope_prune_mask(W: torch.Tensor, n: int, m: int, axis: int = 0, candidates=None, masked=True, masked_t=False):
    """General N:M magnitude mask (m in 2, 4, 8) of W bf16[rows, cols]; returns (mask u8[rows, cols/8],
    masked W or None, transposed masked W or None)."""
    if W is None or W.dim() != 2:
        raise ValueError("W must be a matrix")
    rows, cols = W.shape
    _want(W, BF16, (rows, cols), "W")
    if candidates is not None:
        _want(candidates, U8, (rows, cols // 8), "candidates")
    mask = torch.empty((rows, cols // 8), dtype=U8, device=W.device)
    wm = torch.empty_like(W) if masked else None
    wt = torch.empty((cols, rows), dtype=BF16, device=W.device) if masked_t else None
    _check("slope_prune_mask", lib().slope_prune_mask(_ptr(W), rows, cols, n, m, axis, _ptr(candidates), _ptr(mask),
                                                      _ptr(wm), _ptr(wt), _stream()))
    return mask, wm, wt


def slope_gemm_tn(B: torch.Tensor, A: torch.Tensor, out=None):
    """C[n, m] = B[n, K] A[m, K]^T (dense bf16, fp32 accumulation)."""
    if B is None or A is None or B.dim() != 2 or A.dim() != 2:
        raise ValueError("B and A must be matrices")
    n, K = B.shape
    m = A.shape[0]
    _want(B, BF16, (n, K), "B")
    _want(A, BF16, (m, K), "A")
    C = _want(out, BF16, (n, m), "out") if out is not None else torch.empty((n, m), dtype=BF16, device=B.device)
    _check("slope_gemm_tn", lib().slope_gemm_tn(_ptr(B), n, _ptr(A), m, K, _ptr(C), _stream()))
    return C


def slope_sparse_add(A_vals: torch.Tensor, B_vals: torch.Tensor, beta: float, gamma: float, out=None):
    """beta * A + gamma * B on packed values bf16[rows, cols/2] of two matrices with one pattern."""
    if A_vals is None or A_vals.dim() != 2:
        raise ValueError("A_vals must be a matrix")
    rows, half = A_vals.shape
    _want(A_vals, BF16, (rows, half), "A_vals")
    _want(B_vals, BF16, (rows, half), "B_vals")
    G = _want(out, BF16, (rows, half), "out") if out is not None else torch.empty_like(A_vals)
    _check("slope_sparse_add", lib().slope_sparse_add(_ptr(A_vals), _ptr(B_vals), rows, 2 * half, beta, gamma,
                                                      _ptr(G), _stream()))
    return G


def slope_update_sparse(Wnew_vals: torch.Tensor, meta: torch.Tensor, vals: torch.Tensor, meta_t: torch.Tensor,
                        vals_t: torch.Tensor):
    """New packed values into W^R (vals) and into packed (W^{R,C})^T (vals_t); metadata unchanged."""
    d_out, d_in = _packed(Wnew_vals, meta, "new W^R")
    _want(vals, BF16, (d_out, d_in // 2), "vals")
    _want(meta_t, U8, (d_in, d_out // 8), "metaT")
    _want(vals_t, BF16, (d_in, d_out // 2), "valsT")
    _check("slope_update_sparse", lib().slope_update_sparse(_ptr(Wnew_vals), _ptr(meta), d_out, d_in, _ptr(vals),
                                                            _ptr(meta_t), _ptr(vals_t), _stream()))
    return vals, vals_t


(SLOPE_CEILING_SPARSE_MFMA, SLOPE_CEILING_DENSE_MFMA, SLOPE_CEILING_READ, SLOPE_CEILING_COPY,
 SLOPE_CEILING_SPARSE_MFMA_32, SLOPE_CEILING_DENSE_MFMA_32) = range(6)


def slope_ceiling(kind: int, buf: torch.Tensor, iters: int = 1) -> float:
    """Queues one micro-benchmark launch on buf (uint8 device tensor); returns its flops or bytes."""
    if buf is None or not buf.is_cuda or buf.dtype != U8 or not buf.is_contiguous():
        raise ValueError("buf must be a contiguous uint8 device tensor")
    work = ctypes.c_double(0.0)
    _check("slope_ceiling", lib().slope_ceiling(kind, _ptr(buf), buf.numel(), iters, ctypes.byref(work), _stream()))
    return work.value


# ---------------------------------------------------------------- host <-> device helpers (plumbing)
def bf16_to_device(bits, device="cuda"):
    """numpy uint16 bit patterns -> bf16 device tensor."""
    import numpy as np
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)


def bf16_to_host(t):
    """bf16 tensor -> numpy uint16 bit patterns."""
    import numpy as np
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def slope_tile_order(tiles_m: int, tiles_n: int):
    """Workgroup -> tile assignment of the tile kernels (host only): two int32 arrays, -1 = idle."""
    import numpy as np
    cap = (tiles_m * tiles_n + 255) // 256 * 256 + 8 * 256 * ((tiles_m + 7) // 8 + (tiles_n + 3) // 4 + 1)
    tm = np.empty(cap, dtype=np.int32)
    tn = np.empty(cap, dtype=np.int32)
    grid = lib().slope_tile_order(tiles_m, tiles_n, tm.ctypes.data, tn.ctypes.data, cap)
    if grid < 0:
        raise ValueError("slope_tile_order: extents must be positive")
    return tm[:grid].copy(), tn[:grid].copy()


def slope_spmm_fwd_plan(b: int, d_in: int, d_out: int, r: int = 0, with_workspace: bool = True):
    """Kernels slope_spmm_fwd would launch for a shape (host only): dict of the six plan fields."""
    import numpy as np
    plan = np.zeros(6, dtype=np.int32)
    _check("slope_spmm_fwd_plan", lib().slope_spmm_fwd_plan(b, d_in, d_out, r, int(with_workspace), plan.ctypes.data))
    names = ["product", "rows", "tokens", "slabs", "xl", "xl_chunks"]
    return dict(zip(names, (int(v) for v in plan)))
