"""Seeded random layer shapes through every product call (needs an MI355X): a sweep over the
dispatch regimes that the hand-picked shapes of test_gpu_parity.py may miss.  Same bar as there:
relative Frobenius error of at most 1e-2 against the fp64 oracle, plus the element-wise bound."""
import numpy as np
import pytest
import torch

from oracle import slope_oracle as so
from paper_2405_16325_amd import binding as sl
from tests.parity_util import check_product
from tests.test_gpu_parity import host, layer_on_device, say, u8

pytestmark = pytest.mark.gpu


def random_cases(count=28, seed=20240527):
    rng = np.random.default_rng(seed)
    token_pool = [1, 3, 16, 17, 31, 32, 33, 40, 64, 65, 100, 128, 129, 190, 256, 257, 300, 512, 513, 700, 1100]
    cases = []
    for _ in range(count):
        b = int(rng.choice(token_pool))
        d_out, d_in = (64 * int(rng.integers(1, 17)) for _ in range(2))       # 64 .. 1024
        if rng.random() < 0.4:
            d_in = 256 * int(rng.integers(1, 9))                               # the fast kernels' contraction lengths
        if rng.random() < 0.25:
            d_out = 256 * int(rng.integers(1, 13))
        r = int(rng.choice([0, 32, 64, 96, 160]))
        cases.append((b, d_out, d_in, r))
    return cases


@pytest.mark.parametrize("b,d_out,d_in,r", random_cases())
def test_random_layer(b, d_out, d_in, r):
    say(f"random layer b={b} d_out={d_out} d_in={d_in} r={r}")
    t, d, mask_r, mask_rc = layer_on_device(b, d_out, d_in, r, seed=b * 7 + d_out + d_in + r)
    if r:
        y = sl.slope_spmm_fwd(d["X"], d["vals"], d["meta"], d["L"], d["R"])
        want_y = so.spmm_fwd(t["X"], t["W"], mask_r, t["L"], t["R"])
    else:
        y = sl.slope_spmm_fwd(d["X"], d["vals"], d["meta"])
        want_y = so.spmm_fwd(t["X"], t["W"], mask_r)
    dx = sl.slope_spmm_bwd_x(d["dY"], d["vals_t"], d["meta_t"])
    g_ws = sl.slope_wgrad_masked(d["dY"], d["X"], d["meta"], workspace="auto")
    g_in = sl.slope_wgrad_masked(d["dY"], d["X"], d["meta"], workspace=None)
    torch.cuda.synchronize()
    want_g = so.wgrad_masked(t["dY"], t["X"], u8(d["meta"]))
    errs = {
        "fwd": check_product(host(y), want_y, "Y", two_stage=bool(r)),
        "bwd_x": check_product(host(dx), so.spmm_bwd_x(t["dY"], t["W"], mask_rc), "dX"),
        "wgrad(workspace)": check_product(host(g_ws), want_g, "dW (workspace)"),
        "wgrad(in place)": check_product(host(g_in), want_g, "dW (in place)"),
    }
    if r:                                                      # backward pass with adapters (chain rule of Eq. 11)
        dxa = sl.slope_spmm_bwd_x_adapter(d["dY"], d["vals_t"], d["meta_t"], d["L"], d["R"])
        ga, dl, dr = sl.slope_wgrad_adapter(d["dY"], d["X"], d["meta"], d["L"], d["R"])
        torch.cuda.synchronize()
        want_dl, want_dr = so.adapter_grads(t["dY"], t["X"], t["L"], t["R"])
        errs["bwd_x(adapter)"] = check_product(host(dxa), so.spmm_bwd_x(t["dY"], t["W"], mask_rc, t["L"], t["R"]),
                                               "dX with adapters", two_stage=True)
        errs["dL"] = check_product(host(dl), want_dl, "dL", two_stage=True)
        errs["dR"] = check_product(host(dr), want_dr, "dR", two_stage=True)
        assert (host(ga) == host(g_ws)).all()
    say("  " + "  ".join(f"{k} {v:.2e}" for k, v in errs.items()))
