"""CPU oracle for the double-pruned 2:4 sparse linear layer (SLoPe).

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition that the HIP
kernels are checked against.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import it; it shares no code with the HIP path and imports
nothing from the product package.

bf16 tensors are numpy ``uint16`` bit patterns.  Every product is evaluated in
fp64 from the exact bf16 values; nothing is blocked, fused or reordered.

Notation (paper Sec. 2, Eq. 1-3): W in R^{d_out x d_in}, X in R^{b x d_in},
Y and dY in R^{b x d_out}.  "R" pruning groups run along d_in (inside a row of W,
the reduction dimension of FWD); "C" pruning groups run along d_out (inside a
column of W, the reduction dimension of BWD-2).

Readings taken where the paper is silent (all listed in the design notes):
  * magnitude order: bf16 bits with the sign cleared, compared as integers;
    on equal magnitude the lower index inside the group wins;
  * row pruning keeps exactly N positions per group even when values are zero,
    so the mask is the kept-position set, not (value != 0);
  * double pruning ranks only positions kept by the row prune; a group with fewer
    than N candidates keeps them all;
  * packed 2:4 form: two values per group in ascending index order, one metadata
    nibble idx0 | idx1 << 2 per group, low nibble = even group; a group with
    fewer than two kept positions is padded with its lowest free positions, which
    carry +0.0;
  * the weight gradient is restricted to the row-prune (forward) mask;
  * adapter shapes follow Eq. 11: L is d_in x r, R is r x d_out; its backward pass is
    the chain rule of Eq. 11 (the sparse term still uses W^{R,C}, Eq. 6).
Parity pins: every function here is pinned by tests/test_oracle_*.py.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- bf16
def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of each bf16 bit pattern as fp64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def magnitude_key(bits: np.ndarray) -> np.ndarray:
    """Integer that orders bf16 values by magnitude (sign bit cleared)."""
    return (np.asarray(bits, dtype=np.uint16) & np.uint16(0x7FFF)).astype(np.int64)


# ----------------------------------------------------------------------------- masks
def _keep_top_n(key: np.ndarray, candidate: np.ndarray, n: int) -> np.ndarray:
    """key, candidate: [..., m].  Keep, per group, the first n candidates in the
    order (magnitude descending, index ascending)."""
    m = key.shape[-1]
    # non-candidates sort after every candidate; stable sort gives index-ascending ties
    score = np.where(candidate, key, -1)
    order = np.argsort(-score, axis=-1, kind="stable")
    rank = np.empty_like(order)
    np.put_along_axis(rank, order, np.broadcast_to(np.arange(m), order.shape), axis=-1)
    return candidate & (rank < n)


def prune_rows(w_bits: np.ndarray, n: int = 2, m: int = 4) -> np.ndarray:
    """Row-wise N:M magnitude mask of W (Sec. 2.1, W^R): in every aligned group of
    m consecutive elements along d_in keep the n largest magnitudes.  bool[d_out,d_in]."""
    d_out, d_in = w_bits.shape
    if d_in % m:
        raise ValueError("d_in must be a multiple of m")
    key = magnitude_key(w_bits).reshape(d_out, d_in // m, m)
    keep = _keep_top_n(key, np.ones_like(key, dtype=bool), n)
    return keep.reshape(d_out, d_in)


def double_prune(w_bits: np.ndarray, mask_r: np.ndarray, n: int = 2, m: int = 4) -> np.ndarray:
    """Mask of W^{R,C} (Sec. 2.1, Eq. 6): transpose the row-pruned matrix, then impose
    N:M once more, i.e. groups of m along d_out inside each column of W; only positions
    that survived the row prune compete.  bool[d_out, d_in], a subset of mask_r."""
    d_out, d_in = w_bits.shape
    if d_out % m:
        raise ValueError("d_out must be a multiple of m")
    key_t = magnitude_key(w_bits).T.reshape(d_in, d_out // m, m)
    cand_t = np.asarray(mask_r, dtype=bool).T.reshape(d_in, d_out // m, m)
    keep_t = _keep_top_n(key_t, cand_t, n)
    return keep_t.reshape(d_in, d_out).T.copy()


def mask_to_bits(mask: np.ndarray) -> np.ndarray:
    """1 bit per element, bit (c & 7) of byte c // 8.  uint8[rows, cols/8]."""
    return np.packbits(np.asarray(mask, dtype=bool), axis=1, bitorder="little")


# ----------------------------------------------------------------------------- packed 2:4 form
def pack_2to4(bits: np.ndarray, mask: np.ndarray):
    """Compressed form of (bits * mask) for a mask with at most 2 kept per aligned group
    of 4 along the columns.  Returns vals uint16[rows, cols/2], meta uint8[rows, cols/8]."""
    rows, cols = bits.shape
    if cols % 8:
        raise ValueError("cols must be a multiple of 8")
    g = cols // 4
    mk = np.asarray(mask, dtype=bool).reshape(rows, g, 4)
    if (mk.sum(-1) > 2).any():
        raise ValueError("mask is not 2:4 along the columns")
    v = np.asarray(bits, dtype=np.uint16).reshape(rows, g, 4)
    # slots: kept positions first, then free positions, each by ascending index; take two
    order = np.argsort(~mk, axis=-1, kind="stable")[..., :2]
    order.sort(axis=-1)
    taken = np.take_along_axis(mk, order, axis=-1)
    vals = np.where(taken, np.take_along_axis(v, order, axis=-1), np.uint16(0))
    nib = (order[..., 0] | (order[..., 1] << 2)).astype(np.uint8)
    meta = nib[:, 0::2] | (nib[:, 1::2] << 4)
    return vals.reshape(rows, cols // 2).astype(np.uint16), meta.astype(np.uint8)


def unpack_2to4(vals: np.ndarray, meta: np.ndarray) -> np.ndarray:
    """Dense bits[rows, cols] named by a packed pair (zeros elsewhere)."""
    rows, half = vals.shape
    g = half // 2
    nib = np.empty((rows, g), dtype=np.uint8)
    nib[:, 0::2] = meta & 0xF
    nib[:, 1::2] = meta >> 4
    idx = np.stack([nib & 3, (nib >> 2) & 3], axis=-1).astype(np.int64)
    dense = np.zeros((rows, g, 4), dtype=np.uint16)
    np.put_along_axis(dense, idx, vals.reshape(rows, g, 2), axis=-1)
    return dense.reshape(rows, g * 4)


def meta_to_mask(meta: np.ndarray) -> np.ndarray:
    """Positions named by the metadata, bool[rows, cols]."""
    rows, gb = meta.shape
    g = gb * 2
    nib = np.empty((rows, g), dtype=np.uint8)
    nib[:, 0::2] = meta & 0xF
    nib[:, 1::2] = meta >> 4
    idx = np.stack([nib & 3, (nib >> 2) & 3], axis=-1).astype(np.int64)
    mask = np.zeros((rows, g, 4), dtype=bool)
    np.put_along_axis(mask, idx, True, axis=-1)
    return mask.reshape(rows, g * 4)


def prune_rows_packed(w_bits: np.ndarray):
    """What slope_prune_rows emits: vals, meta, mask bits of W^R (2:4)."""
    mask_r = prune_rows(w_bits, 2, 4)
    vals, meta = pack_2to4(w_bits, mask_r)
    return vals, meta, mask_to_bits(mask_r)


def double_prune_packed(wr_vals: np.ndarray, wr_meta: np.ndarray):
    """What slope_double_prune emits from packed W^R: packed (W^{R,C})^T, i.e. rows = d_in
    and groups along d_out, plus the mask bits of W^{R,C} in W's own orientation."""
    w_r = unpack_2to4(wr_vals, wr_meta)
    mask_r = meta_to_mask(wr_meta)
    mask_rc = double_prune(w_r, mask_r, 2, 4)
    vals_t, meta_t = pack_2to4(np.ascontiguousarray(w_r.T), np.ascontiguousarray(mask_rc.T))
    return vals_t, meta_t, mask_to_bits(mask_rc)


# ----------------------------------------------------------------------------- products (fp64)
def masked_weight(w_bits: np.ndarray, mask: np.ndarray) -> np.ndarray:
    return np.where(np.asarray(mask, dtype=bool), bf16_to_f64(w_bits), 0.0)


def spmm_fwd(x_bits, w_bits, mask_r, l_bits=None, r_bits=None) -> np.ndarray:
    """Y = X (W^R)^T  [+ (X L) R with adapters]   (Eq. 4 and Eq. 11).  fp64[b, d_out]."""
    x = bf16_to_f64(x_bits)
    y = x @ masked_weight(w_bits, mask_r).T
    if l_bits is not None and r_bits is not None and l_bits.shape[1] > 0:
        y = y + (x @ bf16_to_f64(l_bits)) @ bf16_to_f64(r_bits)
    return y


def spmm_bwd_x(dy_bits, w_bits, mask_rc, l_bits=None, r_bits=None) -> np.ndarray:
    """dX = dY W^{R,C}   (Eq. 6)  [+ (dY R^T) L^T with adapters: the derivative of the low-rank
    term of Eq. 11 with respect to X, which the paper leaves to autograd].  fp64[b, d_in]."""
    dy = bf16_to_f64(dy_bits)
    dx = dy @ masked_weight(w_bits, mask_rc)
    if l_bits is not None and r_bits is not None and l_bits.shape[1] > 0:
        dx = dx + (dy @ bf16_to_f64(r_bits).T) @ bf16_to_f64(l_bits).T
    return dx


def adapter_grads(dy_bits, x_bits, l_bits, r_bits):
    """Gradients of the low-rank term Y2 = (X L) R of Eq. 11 (Sec. 2.2), by the chain rule:
    dL = X^T (dY R^T)  fp64[d_in, r],   dR = (X L)^T dY  fp64[r, d_out]."""
    x = bf16_to_f64(x_bits)
    dy = bf16_to_f64(dy_bits)
    dl = x.T @ (dy @ bf16_to_f64(r_bits).T)
    dr = (x @ bf16_to_f64(l_bits)).T @ dy
    return dl, dr


def wgrad_masked(dy_bits, x_bits, wr_meta) -> np.ndarray:
    """dW = dY^T X (Eq. 5) at the positions named by W^R's metadata, in W^R's packed
    layout (Alg. 1 lines 12-13).  fp64[d_out, d_in/2]."""
    g = bf16_to_f64(dy_bits).T @ bf16_to_f64(x_bits)
    d_out, d_in = g.shape
    gb = wr_meta.shape[1]
    nib = np.empty((d_out, gb * 2), dtype=np.uint8)
    nib[:, 0::2] = wr_meta & 0xF
    nib[:, 1::2] = wr_meta >> 4
    idx = np.stack([nib & 3, (nib >> 2) & 3], axis=-1).astype(np.int64)
    return np.take_along_axis(g.reshape(d_out, d_in // 4, 4), idx, axis=-1).reshape(d_out, d_in // 2)


# ----------------------------------------------------------------------------- optimizer side
def sparse_add(a_vals: np.ndarray, b_vals: np.ndarray, beta: float, gamma: float) -> np.ndarray:
    """beta A + gamma B on the packed values of two matrices that share one sparsity pattern
    (App. K "sparse matrix addition"; Alg. 1 line 15 is the case A = masked gradient,
    beta = 1 / gradient scale, B = W^R, gamma = weight decay).  The two scalars cross the C ABI
    as fp32, so they are rounded to fp32 first; the sum itself is fp64.  fp64, shape of a_vals."""
    be = float(np.float32(beta))
    ga = float(np.float32(gamma))
    return be * bf16_to_f64(a_vals) + ga * bf16_to_f64(b_vals)


def update_sparse(wnew_vals: np.ndarray, wr_meta: np.ndarray, wrct_meta: np.ndarray):
    """The two sparse copies after the optimizer produced new values for W^R's kept positions
    (Alg. 1 lines 17-18, App. K "update sparse matrix").  Masks are static (Sec. 2.1), so both
    metadata arrays stay as they are: W^R's packed values become wnew_vals, and every slot of
    packed (W^{R,C})^T takes the new value of the position it names.  A slot that names a
    position outside the row-prune mask is padding and stays +0.0.  wr_meta must name exactly
    W^R's kept positions (what the row prune emits).  Returns (wr_vals, wrct_vals) as bf16 bits."""
    w_new = unpack_2to4(wnew_vals, wr_meta)                     # dense bits [d_out, d_in], zero off the mask
    mask_r = meta_to_mask(wr_meta)
    dense_t = np.ascontiguousarray(np.where(mask_r, w_new, np.uint16(0)).T)   # [d_in, d_out]
    d_in, gb = wrct_meta.shape
    nib = np.empty((d_in, gb * 2), dtype=np.uint8)
    nib[:, 0::2] = wrct_meta & 0xF
    nib[:, 1::2] = wrct_meta >> 4
    idx = np.stack([nib & 3, (nib >> 2) & 3], axis=-1).astype(np.int64)
    vals_t = np.take_along_axis(dense_t.reshape(d_in, gb * 2, 4), idx, axis=-1).reshape(d_in, gb * 4)
    return np.array(wnew_vals, dtype=np.uint16, copy=True), vals_t.astype(np.uint16)


# ----------------------------------------------------------------------------- comparison helper
def rel_fro(got: np.ndarray, want: np.ndarray) -> float:
    """||got - want||_F / ||want||_F in fp64."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = np.linalg.norm(want)
    num = np.linalg.norm(got - want)
    return float(num / den) if den > 0 else float(num)
