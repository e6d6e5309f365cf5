"""The C-ABI library loads, exports every symbol the header declares, and rejects bad arguments
on the host (no GPU needed: argument errors are found before anything is launched); host logic:
the workgroup -> tile order of the tile kernels covers every tile once and balances the XCDs."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2405_16325_amd import binding
from paper_2405_16325_amd import binding as sl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "slope.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(slope_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 12
    handle = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(handle, n), n
    assert set(names) == set(binding.SIGNATURES), "binding and header disagree"


def test_size_queries():
    lib = binding.lib()
    assert lib.slope_version() >= 100
    # 2 x 16 bits of values + 4 bits of index per group of four
    assert lib.slope_packed_vals_bytes(3072, 768) == 3072 * 768
    assert lib.slope_packed_meta_bytes(3072, 768) == 3072 * 768 // 8
    assert lib.slope_mask_bytes(3072, 768) == 3072 * 768 // 8
    assert lib.slope_packed_vals_bytes(16, 12) == 0
    assert lib.slope_spmm_fwd_workspace_bytes(2048, 768, 3072, 0) == 0
    ws = lib.slope_spmm_fwd_workspace_bytes(2048, 768, 3072, 64)
    assert ws >= 2 * 64 * (2048 + 768 + 3072) and ws % 256 == 0


def test_argument_errors_are_reported_before_launch():
    lib = binding.lib()
    p = ctypes.c_void_p(0x1000)       # aligned, never dereferenced: every call below must fail first
    odd = ctypes.c_void_p(0x1008)
    big = 1 << 40
    E = binding
    assert lib.slope_prune_rows(None, 64, 64, 2, 4, p, p, None, None) == E.SLOPE_ERR_NULL
    assert lib.slope_prune_rows(p, 64, 64, 1, 2, p, p, None, None) == E.SLOPE_ERR_UNSUPPORTED
    assert lib.slope_prune_rows(p, 64, 60, 2, 4, p, p, None, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_prune_rows(p, 0, 64, 2, 4, p, p, None, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_prune_rows(p, 64, 64, 2, 4, odd, p, None, None) == E.SLOPE_ERR_ALIGN
    assert lib.slope_double_prune(p, p, 64, 100, p, p, None, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_double_prune(p, p, 68, 64, p, p, None, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_double_prune(p, p, 64, (1 << 23) + 8, p, p, None, None) == E.SLOPE_ERR_SHAPE   # 2^23 at most
    assert lib.slope_double_prune(p, p, (1 << 23) + 8, 64, p, p, None, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_double_prune(p, None, 64, 64, p, p, None, None) == E.SLOPE_ERR_NULL
    assert lib.slope_spmm_fwd(p, 0, p, p, 64, 64, None, None, 0, p, None, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_spmm_fwd(p, 8, p, p, 64, 64, p, p, 48, p, p, None) == E.SLOPE_ERR_UNSUPPORTED
    assert lib.slope_spmm_fwd(p, 8, p, p, 64, 64, p, None, 32, p, p, None) == E.SLOPE_ERR_NULL
    assert lib.slope_spmm_fwd(p, 8, p, p, 64, 64, p, p, 32, p, None, None) == E.SLOPE_ERR_NULL
    assert lib.slope_spmm_fwd(p, 8, p, p, 64, 1 << 31, None, None, 0, p, None, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_spmm_fwd(p, 8, p, p, 64, 68, None, None, 0, p, None, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_spmm_fwd(p, 8, p, p, 64, 64, None, None, 0, p, odd, None) == E.SLOPE_ERR_ALIGN
    # the sized form refuses a workspace that is too small (here: adapters need T, a copy of L, partial sums)
    need = lib.slope_workspace_bytes(E.SLOPE_CALL_SPMM_FWD, 8, 64, 64, 32)
    assert need > 0 and need == lib.slope_spmm_fwd_workspace_bytes(8, 64, 64, 32)
    assert lib.slope_spmm_fwd_ws(p, 8, p, p, 64, 64, p, p, 32, p, p, need - 1, None) == E.SLOPE_ERR_WORKSPACE
    assert lib.slope_spmm_fwd_ws(p, 8, p, p, 64, 64, p, p, 32, p, None, big, None) == E.SLOPE_ERR_NULL
    assert lib.slope_spmm_bwd_x(p, 8, p, p, 64, 76, p, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_spmm_bwd_x(odd, 8, p, p, 64, 64, p, None) == E.SLOPE_ERR_ALIGN
    assert lib.slope_wgrad_masked(p, p, 8, None, 64, 64, p, None) == E.SLOPE_ERR_NULL
    assert lib.slope_wgrad_masked(p, p, -1, p, 64, 64, p, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_wgrad_masked(p, odd, 8, p, 64, 64, p, None) == E.SLOPE_ERR_ALIGN
    need = lib.slope_workspace_bytes(E.SLOPE_CALL_WGRAD_MASKED_WS, 100, 64, 128, 0)
    assert need == lib.slope_wgrad_workspace_bytes(100, 64, 128) >= (64 + 128) * 128 * 2
    assert need == lib.slope_token_copy_bytes(100, 64) + lib.slope_token_copy_bytes(100, 128)
    assert lib.slope_wgrad_masked_ws(p, p, 100, p, 128, 64, p, None, big, None) == E.SLOPE_ERR_NULL
    assert lib.slope_wgrad_masked_ws(p, p, 100, p, 128, 64, p, odd, big, None) == E.SLOPE_ERR_ALIGN
    assert lib.slope_wgrad_masked_ws(p, p, 100, p, 128, 64, p, p, need - 1, None) == E.SLOPE_ERR_WORKSPACE
    assert lib.slope_transpose_tokens(p, 100, 64, p, lib.slope_token_copy_bytes(100, 64) - 1, None) == E.SLOPE_ERR_WORKSPACE
    assert lib.slope_transpose_tokens(p, 100, 60, p, big, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_transpose_tokens(None, 100, 64, p, big, None) == E.SLOPE_ERR_NULL
    assert lib.slope_wgrad_masked_t(p, p, 100, p, 128, 72, p, None, 0, None) == E.SLOPE_ERR_SHAPE   # d_in % 32 for this form
    assert lib.slope_wgrad_masked_t(p, None, 100, p, 128, 64, p, None, 0, None) == E.SLOPE_ERR_NULL
    assert lib.slope_wgrad_masked_t(odd, p, 100, p, 128, 64, p, None, 0, None) == E.SLOPE_ERR_ALIGN
    assert lib.slope_wgrad_masked_t(p, p, 100, p, 128, 64, p, odd, big, None) == E.SLOPE_ERR_ALIGN
    # a 9216 x 9216 layer is 1296 tiles of 256 x 256: the 16 left over after five rounds are cut into 16 slabs
    tail = lib.slope_workspace_bytes(E.SLOPE_CALL_WGRAD_MASKED_T, 16384, 9216, 9216, 0)
    assert tail == 16 * 16 * 256 * 256 * 4
    assert lib.slope_wgrad_masked_t(p, p, 16384, p, 9216, 9216, p, p, tail - 1, None) == E.SLOPE_ERR_WORKSPACE
    assert lib.slope_workspace_bytes(E.SLOPE_CALL_WGRAD_MASKED_WS, 16384, 9216, 9216, 0) == \
        lib.slope_token_copy_bytes(16384, 9216) * 2 + tail
    # whole rounds (36864 x 9216 at 128 x ... no: 4096 x 4096 is exactly 256 tiles), narrow grids and few tokens: no cut
    assert lib.slope_workspace_bytes(E.SLOPE_CALL_WGRAD_MASKED_T, 16384, 4096, 4096, 0) == 0
    assert lib.slope_workspace_bytes(E.SLOPE_CALL_WGRAD_MASKED_T, 16384, 2560, 2560, 0) == 0
    assert lib.slope_workspace_bytes(E.SLOPE_CALL_WGRAD_MASKED_T, 512, 9216, 9216, 0) == 0
    assert lib.slope_spmm_bwd_x_adapter(p, 8, p, p, 64, 64, p, None, 32, p, p, big, None) == E.SLOPE_ERR_NULL
    assert lib.slope_spmm_bwd_x_adapter(p, 8, p, p, 64, 64, p, p, 48, p, p, big, None) == E.SLOPE_ERR_UNSUPPORTED
    assert lib.slope_spmm_bwd_x_adapter(p, 8, p, p, 64, 64, p, p, 32, p, odd, big, None) == E.SLOPE_ERR_ALIGN
    need = lib.slope_workspace_bytes(E.SLOPE_CALL_SPMM_BWD_X_ADAPTER, 8, 64, 64, 32)
    assert need == lib.slope_spmm_bwd_x_adapter_workspace_bytes(8, 32) > 0
    assert lib.slope_spmm_bwd_x_adapter(p, 8, p, p, 64, 64, p, p, 32, p, p, need - 1, None) == E.SLOPE_ERR_WORKSPACE
    assert lib.slope_wgrad_adapter(p, p, 8, p, 64, 64, p, p, 32, p, p, p, None, big, None) == E.SLOPE_ERR_NULL
    assert lib.slope_wgrad_adapter(p, p, 8, p, 64, 76, p, p, 32, p, p, p, p, big, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_wgrad_adapter(p, p, 8, p, 64, 64, p, p, 1024, p, p, p, p, big, None) == E.SLOPE_ERR_UNSUPPORTED
    need = lib.slope_workspace_bytes(E.SLOPE_CALL_WGRAD_ADAPTER, 100, 64, 128, 32)
    assert need == lib.slope_wgrad_adapter_workspace_bytes(100, 64, 128, 32) > lib.slope_wgrad_workspace_bytes(100, 64, 128)
    assert lib.slope_wgrad_adapter(p, p, 100, p, 128, 64, p, p, 32, p, p, p, p, need - 1, None) == E.SLOPE_ERR_WORKSPACE
    for call in (E.SLOPE_CALL_PRUNE_ROWS, E.SLOPE_CALL_DOUBLE_PRUNE, E.SLOPE_CALL_SPMM_BWD_X, E.SLOPE_CALL_WGRAD_MASKED, 0, 99):
        assert lib.slope_workspace_bytes(call, 100, 64, 128, 32) == 0
    assert lib.slope_prune_mask(p, 8, 64, 1, 3, 0, None, p, None, None, None) == E.SLOPE_ERR_UNSUPPORTED
    assert lib.slope_prune_mask(p, 8, 64, 5, 4, 0, None, p, None, None, None) == E.SLOPE_ERR_UNSUPPORTED
    assert lib.slope_prune_mask(p, 6, 64, 2, 4, 1, None, p, None, None, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_prune_mask(p, 8, 60, 2, 4, 0, None, p, None, None, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_prune_mask(p, 8, 64, 2, 4, 0, None, None, None, None, None) == E.SLOPE_ERR_NULL
    assert lib.slope_prune_mask(p, 8, 64, 2, 4, 0, None, odd, None, None, None) == E.SLOPE_ERR_ALIGN
    assert lib.slope_prune_mask(p, 8, 64, 2, 4, 0, odd, p, None, None, None) == E.SLOPE_ERR_ALIGN
    assert lib.slope_gemm_tn(p, 8, p, 64, 100, p, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_gemm_tn(p, 8, None, 64, 128, p, None) == E.SLOPE_ERR_NULL
    assert lib.slope_sparse_add(p, None, 4, 64, 1.0, 1.0, p, None) == E.SLOPE_ERR_NULL
    assert lib.slope_sparse_add(p, p, 4, 20, 1.0, 1.0, p, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_sparse_add(p, p, 4, 64, 1.0, 1.0, odd, None) == E.SLOPE_ERR_ALIGN
    assert lib.slope_update_sparse(p, p, 64, 64, p, None, p, None) == E.SLOPE_ERR_NULL
    assert lib.slope_update_sparse(p, p, 64, 100, p, p, p, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_update_sparse(p, p, 64, (1 << 23) + 8, p, p, p, None) == E.SLOPE_ERR_SHAPE
    assert lib.slope_update_sparse(p, p, 64, 64, p, p, odd, None) == E.SLOPE_ERR_ALIGN
    assert b"NULL" in lib.slope_status_string(E.SLOPE_ERR_NULL)


def test_binding_checks_dtypes_and_shapes_before_the_call():
    """The library sees raw pointers only; the binding refuses tensors of the wrong dtype, shape or size."""
    import torch

    class Fake:
        """Stands in for a device tensor (there is no GPU here): only what the checks look at."""
        def __init__(self, shape, dtype, cuda=True, contiguous=True):
            self.shape, self.dtype, self.is_cuda, self._c = tuple(shape), dtype, cuda, contiguous
            self.device = "cuda:0"
        def dim(self): return len(self.shape)
        def is_contiguous(self): return self._c
        def numel(self):
            n = 1
            for e in self.shape: n *= e
            return n
        def data_ptr(self): raise AssertionError("the call must be refused before a pointer is taken")

    bf, u8 = torch.bfloat16, torch.uint8
    vals, meta = Fake((64, 32), bf), Fake((64, 8), u8)
    with pytest.raises(ValueError, match="bfloat16"):
        binding.slope_spmm_fwd(Fake((8, 64), torch.float16), vals, meta)
    with pytest.raises(ValueError, match="shape"):
        binding.slope_spmm_fwd(Fake((8, 72), bf), vals, meta)
    with pytest.raises(ValueError, match="shape"):
        binding.slope_spmm_fwd(Fake((8, 64), bf), vals, Fake((64, 16), u8))
    with pytest.raises(ValueError, match="shape"):
        binding.slope_spmm_fwd(Fake((8, 64), bf), vals, meta, out=Fake((8, 32), bf))
    with pytest.raises(ValueError, match="shape"):
        binding.slope_spmm_fwd(Fake((8, 64), bf), vals, meta, Fake((64, 32), bf), Fake((16, 64), bf))
    with pytest.raises(ValueError, match="bytes"):
        binding.slope_spmm_fwd(Fake((8, 64), bf), vals, meta, Fake((64, 32), bf), Fake((32, 64), bf),
                               workspace=Fake((256,), u8))
    with pytest.raises(ValueError, match="shape"):
        binding.slope_wgrad_masked(Fake((8, 64), bf), Fake((9, 64), bf), meta)
    with pytest.raises(ValueError, match="contiguous"):
        binding.slope_spmm_bwd_x(Fake((8, 64), bf, contiguous=False), vals, meta)
    with pytest.raises(ValueError, match="device"):
        binding.slope_prune_rows(Fake((8, 8), bf, cuda=False))


def test_static_scratch_rejects_a_shape_beyond_its_buffer():
    lib = binding.lib()
    b, d_out, d_in, r = 512, 9216, 36864, 128
    assert binding.slope_spmm_fwd_workspace_bytes(b, d_in, d_out, r) > binding.SLOPE_STATIC_SCRATCH_BYTES
    p = ctypes.c_void_p(0x1000)            # never dereferenced: the size is refused on the host, before any launch
    assert lib.slope_spmm_fwd_static(p, b, p, p, d_out, d_in, p, p, r, p, None) == binding.SLOPE_ERR_WORKSPACE
    assert lib.slope_spmm_fwd_static(p, b, p, p, d_out, d_in + 4, p, p, r, p, None) == binding.SLOPE_ERR_SHAPE
    assert lib.slope_spmm_fwd_static(p, 8, p, p, 64, 64, p, None, 32, p, None) == binding.SLOPE_ERR_NULL
    text = open(os.path.join(ROOT, "include", "slope.h")).read()
    assert "#define SLOPE_STATIC_SCRATCH_BYTES (%du << 20)" % (binding.SLOPE_STATIC_SCRATCH_BYTES >> 20) in text
    assert b"scratch" in lib.slope_status_string(binding.SLOPE_ERR_WORKSPACE)


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(ValueError):
        binding.slope_prune_rows(torch.zeros((8, 8), dtype=torch.bfloat16))


# ---- host logic: the XCD-aware workgroup -> tile order of the tile kernels -----------------------
TILE_GRIDS = [(1, 1), (1, 128), (128, 1), (3, 7), (15, 400), (16, 16), (17, 16), (16, 19), (36, 36), (36, 144),
              (144, 36), (64, 144), (64, 36), (100, 100), (33, 47), (2, 2000), (250, 15)]


@pytest.mark.parametrize("tiles_m,tiles_n", TILE_GRIDS)
def test_tile_order_covers_every_tile_once(tiles_m, tiles_n):
    tm, tn = sl.slope_tile_order(tiles_m, tiles_n)
    live = tm >= 0
    assert np.array_equal(live, tn >= 0)
    assert (tm[live] < tiles_m).all() and (tn[live] < tiles_n).all()
    flat = tm[live].astype(np.int64) * tiles_n + tn[live]
    assert flat.size == tiles_m * tiles_n
    assert np.array_equal(np.sort(flat), np.arange(tiles_m * tiles_n))


@pytest.mark.parametrize("tiles_m,tiles_n", [g for g in TILE_GRIDS if g[0] * g[1] >= 256])
def test_tile_order_balances_the_xcds(tiles_m, tiles_n):
    # workgroups are dealt round-robin to 8 XCDs: no XCD may get much more than its share
    tm, _ = sl.slope_tile_order(tiles_m, tiles_n)
    per_xcd = np.array([(tm[x::8] >= 0).sum() for x in range(8)])
    assert per_xcd.sum() == tiles_m * tiles_n
    assert per_xcd.max() - per_xcd.min() <= 32          # one chunk of 8 x 4 tiles


def test_tile_order_keeps_chunks_together():
    # wide grids: the 32 tiles an XCD holds at a time share few operand panels: an 8 x 4 chunk where whole chunks
    # cover the grid (here 32 of the 36 rows), 4 rows x 8 columns in the rows below that
    tm, tn = sl.slope_tile_order(36, 144)
    assert tm.size == 36 * 144                                # 20 whole rounds and 64 tiles more: 8 per XCD
    for start in range(0, 36 * 144 // 256 * 256, 256):
        for x in range(8):
            a, b = tm[start + x:start + 256:8], tn[start + x:start + 256:8]
            a, b = a[a >= 0], b[b >= 0]
            if a.size == 0:
                continue
            if a.max() < 32:
                assert a.max() - a.min() < 8 and b.max() - b.min() < 4 and a.min() % 8 == 0 and b.min() % 4 == 0
            else:
                assert a.min() >= 32 and b.max() - b.min() < 8


@pytest.mark.parametrize("tiles_m,tiles_n", [(16, 16), (36, 36), (36, 144), (17, 19), (33, 47), (100, 100), (36, 8), (8, 32)])
def test_tile_order_of_wide_grids_has_no_gaps(tiles_m, tiles_n):
    # whole rounds of 256 workgroups hold one tile each (the first launch of a cut weight gradient is exactly
    # these); what is left over is dealt to the 8 XCDs in equal runs
    tm, _ = sl.slope_tile_order(tiles_m, tiles_n)
    tiles = tiles_m * tiles_n
    whole = tiles // 256 * 256
    assert (tm[:whole] >= 0).all()
    last = tm[whole:]
    assert last.size == -(-(tiles - whole) // 8) * 8
    per_xcd = np.array([(last[x::8] >= 0).sum() for x in range(8)])
    assert per_xcd.sum() == tiles - whole and per_xcd.max() - per_xcd.min() <= per_xcd.max() and per_xcd.max() <= -(-(tiles - whole) // 8)
