"""Parity at the benchmark's full layer sizes, in the launch configuration bench.py times: every
distinct layer shape of the OPT-2.7B, OPT-13B (rank 64) and OPT-66B (rank 128) layer sets at
16384 tokens, and the OPT-66B layers at inference batch sizes.

The oracle cannot evaluate 11 TFLOP products, so it computes seeded samples of the outputs:

  * prune_rows is local to a row: sampled rows of W are pruned by the oracle and compared bit for
    bit with the same rows of the GPU's packed W^R;
  * double_prune is local to a group of four columns of W: for sampled column groups the oracle
    prunes W[:, group] along rows, then along d_out, and the GPU's packed (W^{R,C})^T rows of those
    columns must match bit for bit;
  * Y, dX, dW (and, with adapters, the backward pass through them: dX, dL, dR) are compared on
    (sampled tokens x sampled features) blocks whose operands the oracle derives from those same
    sampled rows / column groups of W.  The samples are contiguous runs of 16 that include the first
    and the last rows, columns and tokens, so that whole MFMA fragments at the tile edges are covered,
    and each block meets the norm and the element-wise bound of tests/parity_util.py.

What the samples cannot see is covered by a property that holds at any size (Eq. 4-6: the sparse
products equal dense products with the masked weight): EVERY element of Y, dX and dW is compared
with fp32 library GEMMs (torch.matmul) on the weight masked by the bit masks the two prune calls
emit, under the same element-wise bound; the masks themselves are tied to the oracle by the samples
and by the packed metadata naming exactly the masks' positions.
"""
import numpy as np
import pytest
import torch

from oracle import slope_oracle as so
from paper_2405_16325_amd import binding as sl
from paper_2405_16325_amd import inputs
from tests.parity_util import ABS_ONE_ROUNDING, ABS_TWO_STAGE, REL, check_product

pytestmark = pytest.mark.gpu


def host(t):
    return sl.bf16_to_host(t)


def say(msg):
    print(msg, flush=True)


def runs_of_16(extent, rng, random_runs=2):
    """Indices of the first and last 16 of range(extent) plus `random_runs` aligned runs of 16."""
    starts = {0, extent - 16}
    while len(starts) < 2 + random_runs and extent >= 64:
        starts.add(int(rng.integers(1, extent // 16 - 1)) * 16)
    return np.unique(np.concatenate([np.arange(s, s + 16) for s in sorted(starts)]))


def unpack_bits(mask_u8):
    """u8[rows, cols/8] bit mask -> bool[rows, cols] on the device."""
    shifts = torch.arange(8, device=mask_u8.device, dtype=torch.uint8)
    return ((mask_u8[:, :, None] >> shifts) & 1).bool().reshape(mask_u8.shape[0], -1)


def assert_all_close(got_bf16, ref_f32, what, two_stage=False, chunk=2048):
    """Every element of a device result against a device fp32 reference, under the element-wise bound."""
    rms = float(ref_f32.double().pow(2).mean().sqrt())
    a = (ABS_TWO_STAGE if two_stage else ABS_ONE_ROUNDING) * rms
    bad, worst = 0, 0.0
    for r0 in range(0, got_bf16.shape[0], chunk):
        g = got_bf16[r0:r0 + chunk].float()
        w = ref_f32[r0:r0 + chunk]
        assert bool(torch.isfinite(g).all()), f"{what}: non-finite values"
        excess = (g - w).abs() - (REL * w.abs() + a)
        bad += int((excess > 0).sum())
        worst = max(worst, float(excess.max()))
    assert bad == 0, f"{what}: {bad} of {got_bf16.numel()} elements outside the element-wise bound (worst excess {worst:.3g})"


# name -> (d_out, d_in, adapter rank): the distinct layer shapes of the three training layer sets
LAYERS = {
    "opt2.7b_attn": (2560, 2560, 0), "opt2.7b_fc1": (10240, 2560, 0), "opt2.7b_fc2": (2560, 10240, 0),
    "opt13b_attn": (5120, 5120, 64), "opt13b_fc1": (20480, 5120, 64), "opt13b_fc2": (5120, 20480, 64),
    "opt66b_attn": (9216, 9216, 128), "opt66b_fc1": (36864, 9216, 128), "opt66b_fc2": (9216, 36864, 128),
    # a token count that is no multiple of a tile (65 token tiles, the last with 40 tokens): the strips of the tile
    # order, wrapped rows in the loaders and in the scalar-cache prefetch, a padded token-contiguous copy
    "opt66b_attn_ragged_tokens": (9216, 9216, 128, 16424),
}


@pytest.mark.parametrize("name", list(LAYERS))
def test_training_layer_full_size(name):
    d_out, d_in, rank = LAYERS[name][:3]
    b = LAYERS[name][3] if len(LAYERS[name]) > 3 else 16384
    say(f"full-size {name}: b={b} d_out={d_out} d_in={d_in} rank={rank}")
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_BASE + d_out + 3 * d_in)

    def gauss(shape, std):
        return (torch.randn(shape, generator=gen, device=dev, dtype=torch.float32) * std).to(torch.bfloat16)

    X, W, dY = gauss((b, d_in), 1.0), gauss((d_out, d_in), 0.02), gauss((b, d_out), 1e-3)
    L = R = None
    if rank:
        L, R = gauss((d_in, rank), 0.02), gauss((rank, d_out), 0.02)
    vals, meta, mask_bits = sl.slope_prune_rows(W, want_mask=True)
    vals_t, meta_t, maskrc_bits = sl.slope_double_prune(vals, meta, want_mask=True)
    Y = sl.slope_spmm_fwd(X, vals, meta, L, R)
    dX = sl.slope_spmm_bwd_x(dY, vals_t, meta_t)
    G = sl.slope_wgrad_masked(dY, X, meta)
    if rank:
        dXa = sl.slope_spmm_bwd_x_adapter(dY, vals_t, meta_t, L, R)
        Ga, dL, dR = sl.slope_wgrad_adapter(dY, X, meta, L, R)
    torch.cuda.synchronize()

    rng = np.random.default_rng(d_out * 7 + d_in)
    rows = runs_of_16(d_out, rng)                                   # sampled rows of W (features of Y)
    cols = runs_of_16(d_in, rng)                                    # sampled columns of W, whole groups of 4
    toks = runs_of_16(b, rng)
    groups = cols[::4] // 4
    rows_t, cols_t, toks_t = (torch.from_numpy(a).to(dev) for a in (rows, cols, toks))

    # ---- prune_rows on sampled rows
    w_rows = host(W[rows_t])
    ov, om, ob = so.prune_rows_packed(w_rows)
    assert (host(vals[rows_t]) == ov).all()
    assert (meta[rows_t].cpu().numpy() == om).all()
    assert (mask_bits[rows_t].cpu().numpy() == ob).all()

    # ---- double_prune on sampled column groups: W[:, cols] is a complete set of row-prune groups
    w_cols = host(W[:, cols_t].contiguous())
    cv, cm, _ = so.prune_rows_packed(w_cols)
    evt, emt, emrc = so.double_prune_packed(cv, cm)                 # rows = the sampled columns, along d_out
    assert (host(vals_t[cols_t]) == evt).all()
    assert (meta_t[cols_t].cpu().numpy() == emt).all()
    got_mrc = unpack_bits(maskrc_bits)[:, cols_t].cpu().numpy()
    assert (got_mrc == np.unpackbits(emrc, axis=1, bitorder="little").astype(bool)).all()

    # ---- oracle blocks
    mask_rows = so.prune_rows(w_rows)
    l_host = host(L) if rank else None
    r_rows = host(R[:, rows_t].contiguous()) if rank else None
    errs = {}
    errs["fwd"] = check_product(host(Y[toks_t][:, rows_t].contiguous()),
                                so.spmm_fwd(host(X[toks_t]), w_rows, mask_rows, l_host, r_rows), "Y block",
                                two_stage=bool(rank))
    mask_cols_r = so.prune_rows(w_cols)
    mask_cols_rc = so.double_prune(w_cols, mask_cols_r)
    errs["bwd_x"] = check_product(host(dX[toks_t][:, cols_t].contiguous()),
                                  so.spmm_bwd_x(host(dY[toks_t]), w_cols, mask_cols_rc), "dX block")
    sub_meta = om.reshape(len(rows), d_in // 8)
    nib = np.where((groups % 2) == 0, sub_meta[:, groups // 2] & 0xF, sub_meta[:, groups // 2] >> 4)
    pairs = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)   # metadata of the sampled groups, re-packed
    dy_rows, x_cols = host(dY[:, rows_t].contiguous()), host(X[:, cols_t].contiguous())
    gidx = torch.from_numpy((groups[:, None] * 2 + np.arange(2)).ravel()).to(dev)
    want_g = so.wgrad_masked(dy_rows, x_cols, pairs)
    errs["wgrad"] = check_product(host(G[rows_t][:, gidx].contiguous()), want_g, "dW block")
    if rank:
        # backward pass through the adapters (chain rule of Eq. 11) on the same blocks
        r_full, l_cols = host(R), host(L[cols_t].contiguous())
        want_dxa = so.spmm_bwd_x(host(dY[toks_t]), w_cols, mask_cols_rc) \
            + (so.bf16_to_f64(host(dY[toks_t])) @ so.bf16_to_f64(r_full).T) @ so.bf16_to_f64(l_cols).T
        errs["bwd_x(adapter)"] = check_product(host(dXa[toks_t][:, cols_t].contiguous()), want_dxa,
                                               "dX block with adapters", two_stage=True)
        assert bool((Ga == G).all())                                # same kernel on the same copies
        # dL rows = sampled columns of W need all of dY R^T; dR columns = sampled rows need all of X L
        t2 = (dY.float() @ R.float().T).double().cpu().numpy()      # [b, r] (library GEMM as a step, fp32)
        t1 = (X.float() @ L.float()).double().cpu().numpy()
        want_dl = so.bf16_to_f64(x_cols).T @ t2
        want_dr = t1.T @ so.bf16_to_f64(dy_rows)
        errs["dL"] = check_product(host(dL[cols_t].contiguous()), want_dl, "dL block", two_stage=True)
        errs["dR"] = check_product(host(dR[:, rows_t].contiguous()), want_dr, "dR block", two_stage=True)
    say("  " + "  ".join(f"{k} {v:.2e}" for k, v in errs.items()))

    # ---- every group of the full-size packed outputs names two distinct ascending positions, and
    #      W^R's metadata names exactly the positions of the emitted bit mask
    for m in (meta, meta_t):
        lo, hi = m & 3, (m >> 2) & 3
        lo2, hi2 = (m >> 4) & 3, m >> 6
        assert bool((lo < hi).all()) and bool((lo2 < hi2).all())
    mask_r = unpack_bits(mask_bits)
    mask_rc = unpack_bits(maskrc_bits)
    assert bool((mask_r.view(d_out, d_in // 4, 4).sum(-1) == 2).all())
    assert bool((mask_rc & ~mask_r).sum() == 0)
    assert bool((mask_rc.view(d_out // 4, 4, d_in).sum(1) <= 2).all())
    nibs = torch.stack([meta & 0xF, meta >> 4], dim=-1).reshape(d_out, d_in // 4).long()
    named = torch.zeros((d_out, d_in // 4, 4), dtype=torch.bool, device=dev)
    named.scatter_(2, (nibs & 3)[..., None], True)
    named.scatter_(2, ((nibs >> 2) & 3)[..., None], True)
    assert bool((named.view(d_out, d_in) == mask_r).all())
    del named, nibs

    # ---- every element against fp32 library GEMMs on the masked weight
    Wf = W.float()
    Xf, dYf = X.float(), dY.float()
    ref = Xf @ (Wf * mask_r).T
    if rank:
        ref += (Xf @ L.float()) @ R.float()
    assert_all_close(Y, ref, "Y (all elements)", two_stage=bool(rank))
    del ref
    ref = dYf @ (Wf * mask_rc)
    assert_all_close(dX, ref, "dX (all elements)")
    if rank:
        ref += (dYf @ R.float().T) @ L.float().T
        assert_all_close(dXa, ref, "dX with adapters (all elements)", two_stage=True)
    del ref
    ref = (dYf.T @ Xf)[mask_r].view(d_out, d_in // 2)               # kept positions, ascending inside each row
    assert_all_close(G, ref, "dW (all elements)")
    del ref
    if rank:
        assert_all_close(dL, Xf.T @ (dYf @ R.float().T), "dL (all elements)", two_stage=True)
        assert_all_close(dR, (Xf @ L.float()).T @ dYf, "dR (all elements)", two_stage=True)


@pytest.mark.parametrize("name,d_out,d_in", [("fc1", 36864, 9216), ("fc2", 9216, 36864), ("attn", 9216, 9216)])
def test_opt66b_inference_sampled(name, d_out, d_in):
    """The same layers at the inference benchmark's batch sizes (1, 16, 128 tokens and two in between),
    rank-128 adapters included: every token, sampled rows of W against the oracle, and every element
    against the fp32 library GEMM on the masked weight."""
    rank = 128
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_BASE + 67)

    def gauss(shape, std):
        return (torch.randn(shape, generator=gen, device=dev, dtype=torch.float32) * std).to(torch.bfloat16)

    W = gauss((d_out, d_in), 0.02)
    L, R = gauss((d_in, rank), 0.02), gauss((rank, d_out), 0.02)
    vals, meta, mask_bits = sl.slope_prune_rows(W, want_mask=True)
    rng = np.random.default_rng(67)
    rows = runs_of_16(d_out, rng)
    rows_t = torch.from_numpy(rows).to(dev)
    w_rows = host(W[rows_t])
    mask_rows = so.prune_rows(w_rows)
    assert (mask_bits[rows_t].cpu().numpy() == so.mask_to_bits(mask_rows)).all()
    l_host, r_host = host(L), host(R[:, rows_t].contiguous())
    Wm = W.float() * unpack_bits(mask_bits)
    for b in (1, 16, 24, 128, 300):
        say(f"full-size inference {name}: b={b} d_out={d_out} d_in={d_in} rank={rank}")
        X = gauss((b, d_in), 1.0)
        for with_adapter in (False, True):
            Y = sl.slope_spmm_fwd(X, vals, meta, L, R) if with_adapter else sl.slope_spmm_fwd(X, vals, meta)
            torch.cuda.synchronize()
            want = so.spmm_fwd(host(X), w_rows, mask_rows, l_host, r_host) if with_adapter \
                else so.spmm_fwd(host(X), w_rows, mask_rows)
            err = check_product(host(Y[:, rows_t].contiguous()), want, "Y block", two_stage=with_adapter)
            say(f"  adapter={with_adapter} rel_fro {err:.3e}")
            ref = X.float() @ Wm.T
            if with_adapter:
                ref += (X.float() @ L.float()) @ R.float()
            assert_all_close(Y, ref, "Y (all elements)", two_stage=with_adapter)
