"""General N:M masks on the GPU (the patterns without a sparse MFMA) vs the CPU oracle, through the C ABI.

Masks and masked weights are bit-exact.  The emulated products (dense MFMA on the masked weight) meet
the same bar as the sparse ones: ||gpu - oracle||_F / ||oracle||_F <= 1e-2 and the element-wise bound.
"""
import numpy as np
import pytest
import torch

from oracle import slope_oracle as so
from paper_2405_16325_amd import binding as sl
from paper_2405_16325_amd import inputs
from tests.parity_util import check_product
from tests.test_gpu_parity import dev, host, say, special_weights

pytestmark = pytest.mark.gpu

PATTERNS = [(1, 2), (2, 4), (2, 8), (1, 4), (4, 8), (3, 4), (8, 8)]


def weights(kind, rows, cols, seed):
    if kind == "gauss":
        return inputs.gaussian_bf16((rows, cols), 0.02, seed, 0)
    if kind == "ties":
        return inputs.coarse_weights(rows, cols, seed)
    return special_weights()


@pytest.mark.parametrize("n,m", PATTERNS)
@pytest.mark.parametrize("kind,rows,cols", [("gauss", 320, 448), ("ties", 64, 192), ("special", 64, 64), ("gauss", 8, 8),
                                            ("gauss", 3072, 768)])
def test_prune_mask_rows_then_columns(n, m, kind, rows, cols):
    say(f"prune_mask {n}:{m} {kind} {rows}x{cols}")
    w = weights(kind, rows, cols, seed=rows + m)
    mask_r = so.prune_rows(w, n, m)
    mask_rc = so.double_prune(w, mask_r, n, m)
    d_w = dev(w)
    m1, wm1, wt1 = sl.slope_prune_mask(d_w, n, m, axis=0, masked_t=True)
    m2, wm2, wt2 = sl.slope_prune_mask(d_w, n, m, axis=1, candidates=m1, masked_t=True)
    torch.cuda.synchronize()
    assert (m1.cpu().numpy() == so.mask_to_bits(mask_r)).all()
    assert (host(wm1) == np.where(mask_r, w, np.uint16(0))).all()
    assert (host(wt1) == np.where(mask_r, w, np.uint16(0)).T).all()
    assert (m2.cpu().numpy() == so.mask_to_bits(mask_rc)).all()
    assert (host(wm2) == np.where(mask_rc, w, np.uint16(0))).all()
    assert (host(wt2) == np.where(mask_rc, w, np.uint16(0)).T).all()


@pytest.mark.parametrize("n,m", [(1, 2), (2, 8), (2, 4)])
@pytest.mark.parametrize("b,d_out,d_in", [(300, 448, 320), (2048, 3072, 768), (17, 192, 64), (4100, 4160, 256)])
def test_emulated_products(n, m, b, d_out, d_in):
    say(f"emulated {n}:{m} b={b} d_out={d_out} d_in={d_in}")
    t = inputs.layer_inputs(b, d_out, d_in, 0, seed=b + m)
    mask_r = so.prune_rows(t["W"], n, m)
    mask_rc = so.double_prune(t["W"], mask_r, n, m)
    d_w = dev(t["W"])
    m1, wm_r, _ = sl.slope_prune_mask(d_w, n, m, axis=0)
    _, _, wt_rc = sl.slope_prune_mask(d_w, n, m, axis=1, candidates=m1, masked=False, masked_t=True)
    y = sl.slope_gemm_tn(dev(t["X"]), wm_r)                       # Y  = X (W^R)^T
    dx = sl.slope_gemm_tn(dev(t["dY"]), wt_rc)                    # dX = dY W^{R,C}
    torch.cuda.synchronize()
    e_y = check_product(host(y), so.spmm_fwd(t["X"], t["W"], mask_r), "Y")
    e_x = check_product(host(dx), so.spmm_bwd_x(t["dY"], t["W"], mask_rc), "dX")
    say(f"  rel_fro Y {e_y:.3e} dX {e_x:.3e}")


def test_two_to_four_mask_agrees_with_the_packed_path():
    """The 2:4 case of the general kernel names exactly the positions that slope_prune_rows and
    slope_double_prune encode in their metadata."""
    w = inputs.gaussian_bf16((512, 384), 0.02, 99, 0)
    d_w = dev(w)
    m1, _, _ = sl.slope_prune_mask(d_w, 2, 4, axis=0, masked=False)
    m2, _, _ = sl.slope_prune_mask(d_w, 2, 4, axis=1, candidates=m1, masked=False)
    vals, meta, mask_bits = sl.slope_prune_rows(d_w, want_mask=True)
    _, _, mask_rc_bits = sl.slope_double_prune(vals, meta, want_mask=True)
    torch.cuda.synchronize()
    assert (m1.cpu().numpy() == mask_bits.cpu().numpy()).all()
    assert (m2.cpu().numpy() == mask_rc_bits.cpu().numpy()).all()
    assert (m2.cpu().numpy() == so.mask_to_bits(so.double_prune(w, so.prune_rows(w)))).all()
