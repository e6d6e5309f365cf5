"""slope_spmm_fwd_static (the entry point that allocates nothing: its scratch memory is a buffer inside
the library's device image) against slope_spmm_fwd with a caller-supplied workspace, through the C ABI.
Same kernels on the same inputs, so the two must agree bit for bit, which is inside the bar of the other
product tests; the result is checked against the fp64 oracle as well.  Calls follow each other on one
stream and shrink, so a later call finds the larger call's leftovers in the shared buffer."""
import ctypes

import pytest
import torch

from oracle import slope_oracle as so
from paper_2405_16325_amd import binding as sl
from paper_2405_16325_amd import inputs
from tests.parity_util import check_product

pytestmark = pytest.mark.gpu

# (b, d_out, d_in, r) in call order: split over K with partial sums + adapters; the same layer with fewer
# tokens (small-batch kernel, T = X L from partial sums); many tokens (copy of L in the buffer); a smaller
# layer without adapters that still takes the split over K; few tokens on a short matrix with a long contraction
# (row-split small-batch kernel, slices' partial sums in the buffer); a single token
SEQUENCE = [(100, 768, 4096, 128), (16, 768, 4096, 128), (700, 512, 768, 64), (48, 512, 8192, 0),
            (16, 2056, 16384, 64), (1, 256, 512, 32)]


def test_static_scratch_matches_the_workspace_call_on_successive_shrinking_calls():
    lib = sl.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for call, (b, d_out, d_in, r) in enumerate(SEQUENCE):
        print(f"no-alloc call {call}: b={b} d_out={d_out} d_in={d_in} r={r}", flush=True)
        t = inputs.layer_inputs(b, d_out, d_in, r, seed=40 + call)
        d = {k: sl.bf16_to_device(v) for k, v in t.items()}
        vals, meta, _ = sl.slope_prune_rows(d["W"])
        L, R = (d["L"], d["R"]) if r else (None, None)
        need = sl.slope_spmm_fwd_workspace_bytes(b, d_in, d_out, r)
        assert 0 < need <= sl.SLOPE_STATIC_SCRATCH_BYTES
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        want_y = torch.empty((b, d_out), dtype=torch.bfloat16, device="cuda")
        got_y = torch.full((b, d_out), float("nan"), dtype=torch.bfloat16, device="cuda")
        p = lambda x: None if x is None else ctypes.c_void_p(x.data_ptr())
        assert lib.slope_spmm_fwd(p(d["X"]), b, p(vals), p(meta), d_out, d_in, p(L), p(R), r, p(want_y), p(ws),
                                  stream) == sl.SLOPE_OK
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        assert lib.slope_spmm_fwd_static(p(d["X"]), b, p(vals), p(meta), d_out, d_in, p(L), p(R), r, p(got_y),
                                         stream) == sl.SLOPE_OK
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert (sl.bf16_to_host(got_y) == sl.bf16_to_host(want_y)).all()
        check_product(sl.bf16_to_host(got_y), so.spmm_fwd(t["X"], t["W"], so.prune_rows(t["W"]), t.get("L"), t.get("R")),
                      "Y", two_stage=bool(r))
