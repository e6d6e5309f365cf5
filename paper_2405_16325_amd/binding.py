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

_P, _I64, _INT, _SZ = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t

# name -> (restype, argtypes); mirrors include/slope.h one to one
SIGNATURES = {
    "slope_version": (_INT, []),
    "slope_last_hip_error": (_INT, []),
    "slope_status_string": (ctypes.c_char_p, [_INT]),
    "slope_packed_vals_bytes": (_SZ, [_I64, _I64]),
    "slope_packed_meta_bytes": (_SZ, [_I64, _I64]),
    "slope_mask_bytes": (_SZ, [_I64, _I64]),
    "slope_spmm_fwd_workspace_bytes": (_SZ, [_I64, _I64, _I64, _I64]),
    "slope_prune_rows": (_INT, [_P, _I64, _I64, _INT, _INT, _P, _P, _P, _P]),
    "slope_double_prune": (_INT, [_P, _P, _I64, _I64, _P, _P, _P, _P]),
    "slope_spmm_fwd": (_INT, [_P, _I64, _P, _P, _I64, _I64, _P, _P, _I64, _P, _P, _P]),
    "slope_spmm_fwd_static": (_INT, [_P, _I64, _P, _P, _I64, _I64, _P, _P, _I64, _P, _P]),
    "slope_spmm_bwd_x": (_INT, [_P, _I64, _P, _P, _I64, _I64, _P, _P]),
    "slope_wgrad_workspace_bytes": (_SZ, [_I64, _I64, _I64]),
    "slope_wgrad_masked": (_INT, [_P, _P, _I64, _P, _I64, _I64, _P, _P, _P]),
    "slope_spmm_bwd_x_adapter_workspace_bytes": (_SZ, [_I64, _I64]),
    "slope_spmm_bwd_x_adapter": (_INT, [_P, _I64, _P, _P, _I64, _I64, _P, _P, _I64, _P, _P, _P]),
    "slope_wgrad_adapter_workspace_bytes": (_SZ, [_I64, _I64, _I64, _I64]),
    "slope_wgrad_adapter": (_INT, [_P, _P, _I64, _P, _I64, _I64, _P, _P, _I64, _P, _P, _P, _P, _P]),
    "slope_prune_mask": (_INT, [_P, _I64, _I64, _INT, _INT, _INT, _P, _P, _P, _P, _P]),
    "slope_gemm_tn": (_INT, [_P, _I64, _P, _I64, _I64, _P, _P]),
    "slope_sparse_add": (_INT, [_P, _P, _I64, _I64, ctypes.c_float, ctypes.c_float, _P, _P]),
    "slope_update_sparse": (_INT, [_P, _P, _I64, _I64, _P, _P, _P, _P]),
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


def slope_prune_rows(W: torch.Tensor, want_mask: bool = False, out=None):
    """W bf16[d_out, d_in] -> (vals bf16[d_out, d_in/2], meta u8[d_out, d_in/8], mask u8 or None)."""
    _dev(W)
    d_out, d_in = W.shape
    if out is None:
        vals = torch.empty((d_out, d_in // 2), dtype=torch.bfloat16, device=W.device)
        meta = torch.empty((d_out, d_in // 8), dtype=torch.uint8, device=W.device)
        mask = torch.empty((d_out, d_in // 8), dtype=torch.uint8, device=W.device) if want_mask else None
    else:
        vals, meta, mask = out
    _check("slope_prune_rows", lib().slope_prune_rows(_ptr(W), d_out, d_in, 2, 4, _ptr(vals), _ptr(meta),
                                                      _ptr(mask), _stream()))
    return vals, meta, mask


def slope_double_prune(vals: torch.Tensor, meta: torch.Tensor, want_mask: bool = False, out=None):
    """Packed W^R -> (valsT bf16[d_in, d_out/2], metaT u8[d_in, d_out/8], maskrc u8[d_out, d_in/8] or None)."""
    _dev(vals, meta)
    d_out, d_in = vals.shape[0], vals.shape[1] * 2
    if out is None:
        vals_t = torch.empty((d_in, d_out // 2), dtype=torch.bfloat16, device=vals.device)
        meta_t = torch.empty((d_in, d_out // 8), dtype=torch.uint8, device=vals.device)
        mask = torch.empty((d_out, d_in // 8), dtype=torch.uint8, device=vals.device) if want_mask else None
    else:
        vals_t, meta_t, mask = out
    _check("slope_double_prune", lib().slope_double_prune(_ptr(vals), _ptr(meta), d_out, d_in, _ptr(vals_t),
                                                          _ptr(meta_t), _ptr(mask), _stream()))
    return vals_t, meta_t, mask


def slope_spmm_fwd_workspace_bytes(b: int, d_in: int, d_out: int, r: int) -> int:
    return int(lib().slope_spmm_fwd_workspace_bytes(b, d_in, d_out, r))


def slope_spmm_fwd(X: torch.Tensor, vals: torch.Tensor, meta: torch.Tensor, L=None, R=None, out=None,
                   workspace=None):
    """Y = X (W^R)^T [+ (X L) R].  X bf16[b, d_in]; packed W^R; L bf16[d_in, r]; R bf16[r, d_out]."""
    _dev(X, vals, meta, L, R)
    b, d_in = X.shape
    d_out = vals.shape[0]
    r = 0 if L is None else L.shape[1]
    Y = out if out is not None else torch.empty((b, d_out), dtype=torch.bfloat16, device=X.device)
    if workspace is None:
        nbytes = slope_spmm_fwd_workspace_bytes(b, d_in, d_out, r)
        if nbytes > 0:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=X.device)
    _check("slope_spmm_fwd", lib().slope_spmm_fwd(_ptr(X), b, _ptr(vals), _ptr(meta), d_out, d_in, _ptr(L), _ptr(R),
                                                  r, _ptr(Y), _ptr(workspace), _stream()))
    return Y


def slope_spmm_fwd_static(X: torch.Tensor, vals: torch.Tensor, meta: torch.Tensor, L=None, R=None, out=None):
    """slope_spmm_fwd on the library's own scratch buffer: the call itself allocates nothing (pass `out`
    to keep this wrapper from allocating Y)."""
    _dev(X, vals, meta, L, R)
    b, d_in = X.shape
    d_out = vals.shape[0]
    r = 0 if L is None else L.shape[1]
    Y = out if out is not None else torch.empty((b, d_out), dtype=torch.bfloat16, device=X.device)
    _check("slope_spmm_fwd_static", lib().slope_spmm_fwd_static(_ptr(X), b, _ptr(vals), _ptr(meta), d_out, d_in,
                                                                _ptr(L), _ptr(R), r, _ptr(Y), _stream()))
    return Y


def slope_spmm_bwd_x(dY: torch.Tensor, vals_t: torch.Tensor, meta_t: torch.Tensor, out=None):
    """dX = dY W^{R,C}.  dY bf16[b, d_out]; packed (W^{R,C})^T with rows = d_in."""
    _dev(dY, vals_t, meta_t)
    b, d_out = dY.shape
    d_in = vals_t.shape[0]
    dX = out if out is not None else torch.empty((b, d_in), dtype=torch.bfloat16, device=dY.device)
    _check("slope_spmm_bwd_x", lib().slope_spmm_bwd_x(_ptr(dY), b, _ptr(vals_t), _ptr(meta_t), d_out, d_in, _ptr(dX),
                                                      _stream()))
    return dX


def slope_wgrad_workspace_bytes(b: int, d_in: int, d_out: int) -> int:
    return int(lib().slope_wgrad_workspace_bytes(b, d_in, d_out))


def slope_wgrad_masked(dY: torch.Tensor, X: torch.Tensor, meta: torch.Tensor, out=None, workspace="auto"):
    """dW = dY^T X at W^R's kept positions, packed bf16[d_out, d_in/2].
    workspace: a uint8 device tensor, None (in-place kernel), or "auto" (allocate scratch here)."""
    _dev(dY, X, meta)
    b, d_out = dY.shape
    d_in = X.shape[1]
    G = out if out is not None else torch.empty((d_out, d_in // 2), dtype=torch.bfloat16, device=dY.device)
    if isinstance(workspace, str):
        workspace = torch.empty(slope_wgrad_workspace_bytes(b, d_in, d_out), dtype=torch.uint8, device=dY.device)
    _check("slope_wgrad_masked", lib().slope_wgrad_masked(_ptr(dY), _ptr(X), b, _ptr(meta), d_out, d_in, _ptr(G),
                                                          _ptr(workspace), _stream()))
    return G


def slope_spmm_bwd_x_adapter(dY, vals_t, meta_t, L, R, out=None, workspace=None):
    """dX = dY W^{R,C} + (dY R^T) L^T.  L bf16[d_in, r]; R bf16[r, d_out]."""
    _dev(dY, vals_t, meta_t, L, R)
    b, d_out = dY.shape
    d_in, r = L.shape
    dX = out if out is not None else torch.empty((b, d_in), dtype=torch.bfloat16, device=dY.device)
    if workspace is None:
        workspace = torch.empty(int(lib().slope_spmm_bwd_x_adapter_workspace_bytes(b, r)), dtype=torch.uint8,
                                device=dY.device)
    _check("slope_spmm_bwd_x_adapter",
           lib().slope_spmm_bwd_x_adapter(_ptr(dY), b, _ptr(vals_t), _ptr(meta_t), d_out, d_in, _ptr(L), _ptr(R), r,
                                          _ptr(dX), _ptr(workspace), _stream()))
    return dX


def slope_wgrad_adapter_workspace_bytes(b: int, d_in: int, d_out: int, r: int) -> int:
    return int(lib().slope_wgrad_adapter_workspace_bytes(b, d_in, d_out, r))


def slope_wgrad_adapter(dY, X, meta, L, R, out=None, workspace=None):
    """(dW packed, dL, dR) of a layer with adapters; one call, shared token-contiguous copies."""
    _dev(dY, X, meta, L, R)
    b, d_out = dY.shape
    d_in, r = L.shape
    if out is None:
        out = (torch.empty((d_out, d_in // 2), dtype=torch.bfloat16, device=dY.device),
               torch.empty((d_in, r), dtype=torch.bfloat16, device=dY.device),
               torch.empty((r, d_out), dtype=torch.bfloat16, device=dY.device))
    G, dL, dR = out
    if workspace is None:
        workspace = torch.empty(slope_wgrad_adapter_workspace_bytes(b, d_in, d_out, r), dtype=torch.uint8,
                                device=dY.device)
    _check("slope_wgrad_adapter",
           lib().slope_wgrad_adapter(_ptr(dY), _ptr(X), b, _ptr(meta), d_out, d_in, _ptr(L), _ptr(R), r, _ptr(G),
                                     _ptr(dL), _ptr(dR), _ptr(workspace), _stream()))
    return G, dL, dR


def slope_prune_mask(W: torch.Tensor, n: int, m: int, axis: int = 0, candidates=None, masked=True, masked_t=False):
    """General N:M magnitude mask (m in 2, 4, 8) of W bf16[rows, cols]; returns (mask u8[rows, cols/8],
    masked W or None, transposed masked W or None)."""
    _dev(W, candidates)
    rows, cols = W.shape
    mask = torch.empty((rows, cols // 8), dtype=torch.uint8, device=W.device)
    wm = torch.empty_like(W) if masked else None
    wt = torch.empty((cols, rows), dtype=torch.bfloat16, device=W.device) if masked_t else None
    _check("slope_prune_mask", lib().slope_prune_mask(_ptr(W), rows, cols, n, m, axis, _ptr(candidates), _ptr(mask),
                                                      _ptr(wm), _ptr(wt), _stream()))
    return mask, wm, wt


def slope_gemm_tn(B: torch.Tensor, A: torch.Tensor, out=None):
    """C[n, m] = B[n, K] A[m, K]^T (dense bf16, fp32 accumulation)."""
    _dev(B, A)
    n, K = B.shape
    m = A.shape[0]
    C = out if out is not None else torch.empty((n, m), dtype=torch.bfloat16, device=B.device)
    _check("slope_gemm_tn", lib().slope_gemm_tn(_ptr(B), n, _ptr(A), m, K, _ptr(C), _stream()))
    return C


def slope_sparse_add(A_vals: torch.Tensor, B_vals: torch.Tensor, beta: float, gamma: float, out=None):
    """beta * A + gamma * B on packed values bf16[rows, cols/2] of two matrices with one pattern."""
    _dev(A_vals, B_vals)
    rows, half = A_vals.shape
    G = out if out is not None else torch.empty_like(A_vals)
    _check("slope_sparse_add", lib().slope_sparse_add(_ptr(A_vals), _ptr(B_vals), rows, 2 * half, beta, gamma,
                                                      _ptr(G), _stream()))
    return G


def slope_update_sparse(Wnew_vals: torch.Tensor, meta: torch.Tensor, vals: torch.Tensor, meta_t: torch.Tensor,
                        vals_t: torch.Tensor):
    """New packed values into W^R (vals) and into packed (W^{R,C})^T (vals_t); metadata unchanged."""
    _dev(Wnew_vals, meta, vals, meta_t, vals_t)
    d_out, d_in = Wnew_vals.shape[0], 2 * Wnew_vals.shape[1]
    _check("slope_update_sparse", lib().slope_update_sparse(_ptr(Wnew_vals), _ptr(meta), d_out, d_in, _ptr(vals),
                                                            _ptr(meta_t), _ptr(vals_t), _stream()))
    return vals, vals_t


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
