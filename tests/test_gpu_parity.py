"""HIP path vs CPU oracle through the C ABI (needs an MI355X).

Integer outputs (kept values, metadata, masks) must match bit for bit.  Products must satisfy
||gpu - oracle||_F / ||oracle||_F <= 1e-2 (bf16 operands, fp32 accumulation, bf16 result: the
output rounding alone contributes about 2^-9 / sqrt(3) ~ 1.1e-3, fp32 accumulation order far less)
and, element by element, the bound of tests/parity_util.py.
"""
import numpy as np
import pytest
import torch

from oracle import slope_oracle as so
from paper_2405_16325_amd import binding as sl
from paper_2405_16325_amd import inputs
from tests.parity_util import TOL, check_product

pytestmark = pytest.mark.gpu


def dev(bits):
    return sl.bf16_to_device(bits)


def host(t):
    return sl.bf16_to_host(t)


def u8(t):
    return t.cpu().numpy()


def say(msg):
    print(msg, flush=True)


def special_weights():
    """Rows full of ties, zeros, infinities and NaNs."""
    f = np.float32
    rows = [
        [1, 1, 1, 1, -1, 1, -1, 1], [0, 0, 0, 0, -0.0, 0.0, 0.0, -0.0], [0, 0, 0, 7, 7, 0, 0, 0],
        [np.inf, 1, -np.inf, 2, np.nan, np.inf, 5, 1], [1e-40, -1e-40, 0, 1e-39, 3, -3, 3, -3],
        [2, 1, 2, 1, 1, 2, 1, 2], [-5, 4, -3, 2, 2, -3, 4, -5], [0.5, 0.25, -0.5, 0.25, 1, 1, 2, 1],
    ]
    w = inputs.f32_to_bf16_bits(np.array(rows, dtype=f))
    return np.tile(w, (8, 8))            # 64 x 64


PRUNE_CASES = [
    ("cfg1_fc1", lambda: inputs.gaussian_bf16((3072, 768), 0.02, 0, 2)),
    ("one_row", lambda: inputs.gaussian_bf16((1, 8), 0.02, 1, 2)),
    ("ragged_rows", lambda: inputs.gaussian_bf16((101, 72), 0.02, 2, 2)),
    ("odd_chunks", lambda: inputs.gaussian_bf16((3, 40), 0.02, 3, 2)),
    ("ties", lambda: inputs.coarse_weights(320, 192, 4)),
    ("special", special_weights),
]


@pytest.mark.parametrize("name,make", PRUNE_CASES, ids=[c[0] for c in PRUNE_CASES])
def test_prune_rows_bit_exact(name, make):
    w = make()
    say(f"prune_rows {name} {w.shape}")
    vals, meta, mask = sl.slope_prune_rows(dev(w), want_mask=True)
    torch.cuda.synchronize()
    ov, om, ob = so.prune_rows_packed(w)
    assert (host(vals) == ov).all()
    assert (u8(meta) == om).all()
    assert (u8(mask) == ob).all()
    vals2, meta2, none = sl.slope_prune_rows(dev(w), want_mask=False)
    assert none is None and (host(vals2) == ov).all() and (u8(meta2) == om).all()


DP_CASES = [
    ("cfg1_fc1", lambda: inputs.gaussian_bf16((3072, 768), 0.02, 0, 2)),
    ("one_tile_part", lambda: inputs.gaussian_bf16((64, 64), 0.02, 5, 2)),
    ("ragged_tiles", lambda: inputs.gaussian_bf16((192, 320), 0.02, 6, 2)),
    # more than one chunk of 8 x 8 tiles in both directions, the last chunks partly outside the matrix
    ("many_chunks", lambda: inputs.gaussian_bf16((1312, 1160), 0.02, 8, 2)),
    ("many_chunks_byte_rows", lambda: inputs.gaussian_bf16((1160, 1288), 0.02, 9, 2)),
    ("ties", lambda: inputs.coarse_weights(320, 192, 7)),
    ("zeros", lambda: np.zeros((128, 64), dtype=np.uint16)),
    ("special", special_weights),
]


@pytest.mark.parametrize("name,make", DP_CASES, ids=[c[0] for c in DP_CASES])
def test_double_prune_bit_exact(name, make):
    w = make()
    say(f"double_prune {name} {w.shape}")
    ov, om, _ = so.prune_rows_packed(w)
    vt, mt, mrc = sl.slope_double_prune(dev(ov), torch.from_numpy(om).cuda(), want_mask=True)
    torch.cuda.synchronize()
    evt, emt, emrc = so.double_prune_packed(ov, om)
    assert (host(vt) == evt).all()
    assert (u8(mt) == emt).all()
    assert (u8(mrc) == emrc).all()
    vt2, mt2, none = sl.slope_double_prune(dev(ov), torch.from_numpy(om).cuda())
    assert none is None and (host(vt2) == evt).all() and (u8(mt2) == emt).all()


def layer_on_device(b, d_out, d_in, rank, seed):
    t = inputs.layer_inputs(b, d_out, d_in, rank, seed)
    d = {k: dev(v) for k, v in t.items()}
    vals, meta, _ = sl.slope_prune_rows(d["W"])
    vals_t, meta_t, _ = sl.slope_double_prune(vals, meta)
    d.update(vals=vals, meta=meta, vals_t=vals_t, meta_t=meta_t)
    mask_r = so.prune_rows(t["W"])
    mask_rc = so.double_prune(t["W"], mask_r)
    return t, d, mask_r, mask_rc


# (b, d_out, d_in): the first is the OPT-125m FC1 layer; the others cover ragged token counts,
# partial tiles of the small and the large tile of the fast kernels (contraction length a multiple
# of 256), the generic kernels (other multiples of 64) and a single k-step
PRODUCT_SHAPES = [
    (2048, 3072, 768), (300, 448, 320), (1, 64, 64), (17, 192, 64),
    (4100, 4160, 256), (4096, 4096, 128), (1000, 1024, 1280), (4100, 4224, 512), (777, 256, 256),
    (4100, 768, 4160), (4000, 4032, 512), (4000, 512, 4032),   # the last two: 256 x 256 tiles, ragged both ways
]


# few tokens (inference): the narrow-token tiles, with few and with many weight tiles
SKINNY_SHAPES = [(1, 512, 512), (7, 25600, 256), (100, 512, 768), (128, 25600, 256), (16, 256, 25600),
                 (32, 2112, 4160), (17, 4160, 2112), (33, 512, 512),
                 (8, 8320, 256), (16, 13696, 256), (3, 256, 8320),   # 48- and 64-row workgroups of the small-batch kernel
                 (24, 8320, 256),                                      # 17-32 tokens, 48-row workgroups
                 (100, 768, 4096), (200, 4160, 2048), (48, 512, 8192)]   # split over K with partial sums (forward)


# few tokens and a contraction that is a multiple of 1024: the row-split small-batch kernel.  Tall matrices in one
# slice (the last workgroup's rows partly outside); short ones cut along the contraction into equal and unequal slices
# (slices only for contractions of 16384 or more; 17 to 32 tokens take the kernel only with four slices or more)
ROWS_SHAPES = [(5, 24584, 1024), (1, 36864, 2048), (16, 2056, 16384), (17, 4104, 16384), (32, 4104, 17408),
               (3, 9600, 16384)]


@pytest.mark.parametrize("b,d_out,d_in", PRODUCT_SHAPES + SKINNY_SHAPES + ROWS_SHAPES)
def test_spmm_fwd(b, d_out, d_in):
    say(f"spmm_fwd b={b} d_out={d_out} d_in={d_in}")
    t, d, mask_r, _ = layer_on_device(b, d_out, d_in, 0, seed=b + d_out)
    y = sl.slope_spmm_fwd(d["X"], d["vals"], d["meta"])
    torch.cuda.synchronize()
    want = so.spmm_fwd(t["X"], t["W"], mask_r)
    err = check_product(host(y), want, "Y")
    say(f"  rel_fro {err:.3e}")


# (the input gradient has no scratch: the row-split kernel only where the transposed weight is tall enough)
@pytest.mark.parametrize("b,d_out,d_in", PRODUCT_SHAPES + SKINNY_SHAPES + [(5, 1024, 24584), (16, 2048, 36872)])
def test_spmm_bwd_x(b, d_out, d_in):
    say(f"spmm_bwd_x b={b} d_out={d_out} d_in={d_in}")
    t, d, _, mask_rc = layer_on_device(b, d_out, d_in, 0, seed=b + d_in)
    dx = sl.slope_spmm_bwd_x(d["dY"], d["vals_t"], d["meta_t"])
    torch.cuda.synchronize()
    want = so.spmm_bwd_x(t["dY"], t["W"], mask_rc)
    err = check_product(host(dx), want, "dX")
    say(f"  rel_fro {err:.3e}")


# the last three are large enough for the workspace path (256 x 256 tiles of token-contiguous
# copies): full tiles, ragged tiles in both dimensions, a token count that is not a multiple of 64
WGRAD_SHAPES = PRODUCT_SHAPES + [(1000, 320, 448), (200, 4096, 2048), (1000, 4160, 2112), (77, 2048, 4096)]


@pytest.mark.parametrize("ws", ["auto", None], ids=["workspace", "in_place"])
@pytest.mark.parametrize("b,d_out,d_in", WGRAD_SHAPES)
def test_wgrad_masked(b, d_out, d_in, ws):
    say(f"wgrad_masked b={b} d_out={d_out} d_in={d_in} workspace={ws}")
    t, d, _, _ = layer_on_device(b, d_out, d_in, 0, seed=b + 7)
    g = sl.slope_wgrad_masked(d["dY"], d["X"], d["meta"], workspace=ws)
    torch.cuda.synchronize()
    want = so.wgrad_masked(t["dY"], t["X"], u8(d["meta"]))
    err = check_product(host(g), want, "dW")
    say(f"  rel_fro {err:.3e}")


@pytest.mark.parametrize("b,d_out,d_in,r", [(2048, 3072, 768, 64), (300, 448, 320, 32), (4100, 4160, 256, 128), (4000, 4032, 256, 128),
                                            (4000, 4032, 256, 160),   # 256 x 256 tiles, two chunks of R, the second 32 rows
                                            (16, 512, 768, 64), (1, 1280, 256, 32), (32, 4160, 1024, 128), (7, 448, 320, 288),
                                            (16, 8320, 256, 64), (5, 13696, 256, 512),
                                            (200, 4160, 2048, 64), (100, 768, 4096, 128), (48, 512, 8192, 32), (32, 8320, 256, 64),
                                            (50, 128, 192, 160),
                                            # the MFMA split of X L: several column groups of the rank, token groups of 128
                                            (130, 512, 768, 288), (500, 1024, 1024, 512), (40, 768, 512, 160), (20, 4160, 640, 96),
                                            # the row-split small-batch kernel: one slice, several slices
                                            (12, 24584, 1024, 160), (16, 2056, 16384, 64), (3, 9600, 16384, 32),
                                            (20, 4104, 16384, 160), (4, 24584, 1024, 512), (1, 36872, 2048, 32)])
def test_spmm_fwd_with_adapter(b, d_out, d_in, r):
    say(f"spmm_fwd adapter b={b} d_out={d_out} d_in={d_in} r={r}")
    t, d, mask_r, _ = layer_on_device(b, d_out, d_in, r, seed=r + b)
    y = sl.slope_spmm_fwd(d["X"], d["vals"], d["meta"], d["L"], d["R"])
    torch.cuda.synchronize()
    want = so.spmm_fwd(t["X"], t["W"], mask_r, t["L"], t["R"])
    err = check_product(host(y), want, "Y with adapters", two_stage=True)
    base = so.spmm_fwd(t["X"], t["W"], mask_r)
    say(f"  rel_fro {err:.3e} (adapter share of the norm {np.linalg.norm(want - base) / np.linalg.norm(want):.3f})")
    # the low-rank term itself, isolated by subtracting the plain sparse product computed on the GPU
    y0 = sl.slope_spmm_fwd(d["X"], d["vals"], d["meta"])
    low = so.bf16_to_f64(host(y)) - so.bf16_to_f64(host(y0))
    assert so.rel_fro(low, want - base) <= 5e-2


def test_runs_are_bit_identical():
    t, d, _, _ = layer_on_device(512, 256, 384, 32, seed=99)
    a = [sl.slope_spmm_fwd(d["X"], d["vals"], d["meta"], d["L"], d["R"]),
         sl.slope_spmm_bwd_x(d["dY"], d["vals_t"], d["meta_t"]),
         sl.slope_wgrad_masked(d["dY"], d["X"], d["meta"])]
    b = [sl.slope_spmm_fwd(d["X"], d["vals"], d["meta"], d["L"], d["R"]),
         sl.slope_spmm_bwd_x(d["dY"], d["vals_t"], d["meta_t"]),
         sl.slope_wgrad_masked(d["dY"], d["X"], d["meta"])]
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert (host(x) == host(y)).all()


def test_error_status_raises():
    w = dev(inputs.gaussian_bf16((64, 60), 0.02, 1, 2))
    with pytest.raises(sl.SlopeError) as e:
        sl.slope_prune_rows(w)
    assert e.value.status == sl.SLOPE_ERR_SHAPE


@pytest.mark.parametrize("b,d_out,d_in", [(2048, 3072, 768), (1000, 320, 448), (4100, 4160, 256), (77, 2048, 4096), (1, 64, 64)])
def test_wgrad_from_prepared_token_copies(b, d_out, d_in):
    """slope_transpose_tokens + slope_wgrad_masked_t (copies made once, reusable by layers that share an operand)
    give what slope_wgrad_masked_ws gives, bit for bit, and the oracle's result within the bar."""
    say(f"wgrad from prepared copies b={b} d_out={d_out} d_in={d_in}")
    t, d, _, _ = layer_on_device(b, d_out, d_in, 0, seed=b + 11)
    xt, dyt = sl.slope_transpose_tokens(d["X"]), sl.slope_transpose_tokens(d["dY"])
    g = sl.slope_wgrad_masked_t(dyt, xt, b, d["meta"])
    g_ws = sl.slope_wgrad_masked(d["dY"], d["X"], d["meta"], workspace="auto")
    # a second layer with the same input: the copy of X is used again
    w2 = dev(inputs.gaussian_bf16((d_out, d_in), 0.02, b + 12, 2))
    _, meta2, _ = sl.slope_prune_rows(w2)
    g2 = sl.slope_wgrad_masked_t(dyt, xt, b, meta2)
    torch.cuda.synchronize()
    assert (host(g) == host(g_ws)).all()
    check_product(host(g), so.wgrad_masked(t["dY"], t["X"], u8(d["meta"])), "dW")
    check_product(host(g2), so.wgrad_masked(t["dY"], t["X"], u8(meta2)), "dW of the second layer")


@pytest.mark.parametrize("b,d_out,d_in", [(1536, 4096, 4352), (1100, 4360, 4320), (4096, 4608, 4096)])
def test_wgrad_cuts_the_tiles_of_a_last_partial_round(b, d_out, d_in):
    """Grids of 256 x 256 tiles that leave a few tiles after the last full round of 256 (272, 306, 288 here):
    with scratch memory those tiles are cut along the tokens and summed in a second pass.  Both forms must meet
    the oracle; the cut one is also what slope_wgrad_masked gives with its workspace, bit for bit."""
    say(f"wgrad with a cut last round b={b} d_out={d_out} d_in={d_in}")
    need = sl.slope_workspace_bytes(sl.SLOPE_CALL_WGRAD_MASKED_T, b, d_in, d_out)
    assert need > 0
    t, d, _, _ = layer_on_device(b, d_out, d_in, 0, seed=b + 31)
    xt, dyt = sl.slope_transpose_tokens(d["X"]), sl.slope_transpose_tokens(d["dY"])
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")     # stale bytes (NaNs) must not leak
    g_cut = sl.slope_wgrad_masked_t(dyt, xt, b, d["meta"], workspace=ws)
    g_plain = sl.slope_wgrad_masked_t(dyt, xt, b, d["meta"], workspace=None)
    g_ws = sl.slope_wgrad_masked(d["dY"], d["X"], d["meta"], workspace="auto")
    torch.cuda.synchronize()
    want = so.wgrad_masked(t["dY"], t["X"], u8(d["meta"]))
    check_product(host(g_cut), want, "dW, last round cut")
    check_product(host(g_plain), want, "dW, last round whole")
    assert (host(g_cut) == host(g_ws)).all()
    with pytest.raises(ValueError):
        sl.slope_wgrad_masked_t(dyt, xt, b, d["meta"], workspace=ws[:need - 256])


def test_sized_workspaces_are_checked():
    t, d, _, _ = layer_on_device(300, 256, 512, 32, seed=5)
    need = sl.slope_spmm_fwd_workspace_bytes(300, 512, 256, 32)
    small = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(ValueError):
        sl.slope_spmm_fwd(d["X"], d["vals"], d["meta"], d["L"], d["R"], workspace=small)
    import ctypes
    p = lambda x: ctypes.c_void_p(x.data_ptr())
    y = torch.empty((300, 256), dtype=torch.bfloat16, device="cuda")
    st = sl.lib().slope_spmm_fwd_ws(p(d["X"]), 300, p(d["vals"]), p(d["meta"]), 256, 512, p(d["L"]), p(d["R"]), 32, p(y),
                                    p(small), small.numel(), None)
    assert st == sl.SLOPE_ERR_WORKSPACE


def test_ceiling_micro_benchmarks_run():
    buf = torch.zeros(64 << 20, dtype=torch.uint8, device="cuda")
    for kind in (sl.SLOPE_CEILING_SPARSE_MFMA, sl.SLOPE_CEILING_DENSE_MFMA, sl.SLOPE_CEILING_READ, sl.SLOPE_CEILING_COPY):
        assert sl.slope_ceiling(kind, buf, 4) > 0
    torch.cuda.synchronize()
    with pytest.raises(sl.SlopeError):
        sl.slope_ceiling(7, buf, 4)
    with pytest.raises(sl.SlopeError):
        sl.slope_ceiling(sl.SLOPE_CEILING_READ, buf[:1 << 20], 4)
