"""Backward pass of a layer with adapters (chain rule of Eq. 11): HIP path vs CPU oracle through the C ABI.

Same bar as the other products: ||gpu - oracle||_F / ||oracle||_F <= 1e-2 and the element-wise bound
of tests/parity_util.py (bf16 operands, fp32 accumulation, bf16 results; the intermediate products
X L and dY R^T are rounded to bf16 on the GPU and kept in fp64 by the oracle).  The packed dW of the combined call must equal the one of
slope_wgrad_masked bit for bit: it is the same kernel on the same copies.
"""
import numpy as np
import pytest
import torch

from oracle import slope_oracle as so
from paper_2405_16325_amd import binding as sl
from tests.parity_util import check_product
from tests.test_gpu_parity import host, layer_on_device, say, u8

pytestmark = pytest.mark.gpu

# (b, d_out, d_in, r): OPT-125m FC1 with rank 64; ragged tokens and features; rank not a multiple of 64;
# a rank above 128 (two row tiles of the skinny kernels); the 256 x 256 sparse tile with ragged edges
CASES = [(2048, 3072, 768, 64), (300, 448, 320, 32), (4100, 4160, 256, 128), (50, 128, 192, 160), (1, 64, 64, 32),
         (4000, 512, 4032, 128), (777, 1280, 1024, 96)]


@pytest.mark.parametrize("b,d_out,d_in,r", CASES)
def test_spmm_bwd_x_adapter(b, d_out, d_in, r):
    say(f"spmm_bwd_x_adapter b={b} d_out={d_out} d_in={d_in} r={r}")
    t, d, _, mask_rc = layer_on_device(b, d_out, d_in, r, seed=3 * r + b)
    dx = sl.slope_spmm_bwd_x_adapter(d["dY"], d["vals_t"], d["meta_t"], d["L"], d["R"])
    torch.cuda.synchronize()
    want = so.spmm_bwd_x(t["dY"], t["W"], mask_rc, t["L"], t["R"])
    base = so.spmm_bwd_x(t["dY"], t["W"], mask_rc)
    err = check_product(host(dx), want, "dX with adapters", two_stage=True)
    say(f"  rel_fro {err:.3e} (adapter share of the norm {np.linalg.norm(want - base) / np.linalg.norm(want):.3f})")
    # the low-rank term itself, isolated by subtracting the plain product computed on the GPU
    dx0 = sl.slope_spmm_bwd_x(d["dY"], d["vals_t"], d["meta_t"])
    low = so.bf16_to_f64(host(dx)) - so.bf16_to_f64(host(dx0))
    assert so.rel_fro(low, want - base) <= 5e-2


@pytest.mark.parametrize("b,d_out,d_in,r", CASES)
def test_wgrad_adapter(b, d_out, d_in, r):
    say(f"wgrad_adapter b={b} d_out={d_out} d_in={d_in} r={r}")
    t, d, _, _ = layer_on_device(b, d_out, d_in, r, seed=5 * r + b)
    g, dl, dr = sl.slope_wgrad_adapter(d["dY"], d["X"], d["meta"], d["L"], d["R"])
    torch.cuda.synchronize()
    want_g = so.wgrad_masked(t["dY"], t["X"], u8(d["meta"]))
    want_dl, want_dr = so.adapter_grads(t["dY"], t["X"], t["L"], t["R"])
    e_g = check_product(host(g), want_g, "dW")
    e_l = check_product(host(dl), want_dl, "dL", two_stage=True)
    e_r = check_product(host(dr), want_dr, "dR", two_stage=True)
    say(f"  rel_fro dW {e_g:.3e} dL {e_l:.3e} dR {e_r:.3e}")
    # same kernel, same copies as slope_wgrad_masked with a workspace
    ws = torch.empty(sl.slope_wgrad_adapter_workspace_bytes(b, d_in, d_out, r), dtype=torch.uint8, device="cuda")
    g2, _, _ = sl.slope_wgrad_adapter(d["dY"], d["X"], d["meta"], d["L"], d["R"], workspace=ws)
    torch.cuda.synchronize()
    assert (host(g2) == host(g)).all()


def test_adapter_backward_with_zero_adapters():
    t, d, _, mask_rc = layer_on_device(300, 448, 320, 32, seed=91)
    zl, zr = torch.zeros_like(d["L"]), torch.zeros_like(d["R"])
    dx = sl.slope_spmm_bwd_x_adapter(d["dY"], d["vals_t"], d["meta_t"], zl, d["R"])
    dx0 = sl.slope_spmm_bwd_x(d["dY"], d["vals_t"], d["meta_t"])
    g, dl, dr = sl.slope_wgrad_adapter(d["dY"], d["X"], d["meta"], d["L"], zr)
    torch.cuda.synchronize()
    assert (host(dx) == host(dx0)).all()
    assert (so.bf16_to_f64(host(dl)) == 0).all()              # dL needs R
    assert np.abs(so.bf16_to_f64(host(dr))).max() > 0          # dR does not
