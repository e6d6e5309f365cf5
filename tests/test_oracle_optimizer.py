"""Pins for the oracle's optimizer-side packed operations (Alg. 1 lines 15-18; CPU only)."""
import numpy as np
import pytest

from oracle import slope_oracle as so
from paper_2405_16325_amd import inputs


def bf(x):
    return inputs.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def packed_layer(d_out=32, d_in=48, seed=5):
    w = inputs.gaussian_bf16((d_out, d_in), 0.02, seed, 0)
    vals, meta, _ = so.prune_rows_packed(w)
    vt, mt, mask_rc_bits = so.double_prune_packed(vals, meta)
    return w, vals, meta, vt, mt


# ---------------------------------------------------------------- sparse_add
def test_sparse_add_hand_values():
    # exactly representable operands: 1/gamma = 0.25, alpha = 0.5
    a = bf([[8.0, -4.0, 0.0, 2.0]])
    b = bf([[1.0, 1.0, -3.0, 0.5]])
    got = so.sparse_add(a, b, 0.25, 0.5)
    assert (got == np.array([[2.5, -0.5, -1.5, 0.75]])).all()


def test_sparse_add_special_cases():
    _, vals, meta, _, _ = packed_layer()
    g = inputs.gaussian_bf16(vals.shape, 1e-3, 9, 1)
    assert (so.sparse_add(g, vals, 1.0, 0.0) == so.bf16_to_f64(g)).all()
    assert (so.sparse_add(g, vals, 0.0, 1.0) == so.bf16_to_f64(vals)).all()
    assert (so.sparse_add(g, g, 3.0, -3.0) == 0.0).all()
    # symmetric in its two (matrix, scalar) pairs
    assert (so.sparse_add(g, vals, 0.5, 0.125) == so.sparse_add(vals, g, 0.125, 0.5)).all()


def test_sparse_add_equals_dense_combination_on_the_mask():
    """Packing commutes with the linear combination: unpack(beta A + gamma B) is the dense
    beta (A * mask) + gamma (B * mask)."""
    w, vals, meta, _, _ = packed_layer()
    mask = so.meta_to_mask(meta)
    gd = inputs.gaussian_bf16(w.shape, 1e-3, 9, 2)                   # a dense "gradient"
    g_vals, g_meta = so.pack_2to4(gd, mask)
    assert (g_meta == meta).all()
    beta, gamma = 1.0 / 1024.0, 0.01
    got = so.sparse_add(g_vals, vals, beta, gamma)                   # packed, fp64
    want_dense = float(np.float32(beta)) * so.masked_weight(gd, mask) + float(np.float32(gamma)) * so.masked_weight(w, mask)
    # scatter the packed result back with the metadata, position by position
    d_out, d_in = w.shape
    dense = np.zeros((d_out, d_in))
    for o in range(d_out):
        for gi in range(d_in // 4):
            nib = (int(meta[o, gi // 2]) >> (4 * (gi & 1))) & 0xF
            dense[o, 4 * gi + (nib & 3)] = got[o, 2 * gi]
            dense[o, 4 * gi + (nib >> 2)] = got[o, 2 * gi + 1]
    assert (dense == want_dense).all()


def test_sparse_add_rounds_scalars_to_fp32():
    a = bf([[1.0]])
    b = bf([[0.0]])
    assert so.sparse_add(a, b, 0.1, 0.0)[0, 0] == float(np.float32(0.1))


# ---------------------------------------------------------------- update_sparse
def test_update_with_unchanged_values_reproduces_the_double_prune():
    _, vals, meta, vt, mt = packed_layer()
    new_vals, new_vt = so.update_sparse(vals, meta, mt)
    assert (new_vals == vals).all()
    assert (new_vt == vt).all()                                      # padding slots included


def test_update_carries_new_values_and_keeps_padding_zero():
    w, vals, meta, vt, mt = packed_layer(d_out=64, d_in=40, seed=11)
    mask_r = so.meta_to_mask(meta)
    mask_rc = so.double_prune(so.unpack_2to4(vals, meta), mask_r)
    fresh = inputs.gaussian_bf16(w.shape, 0.02, 12, 3)               # new dense weights
    fresh = np.where(fresh == 0, np.uint16(0x3F80), fresh)           # no zeros: padding must stand out
    wnew_vals, wnew_meta = so.pack_2to4(fresh, mask_r)
    assert (wnew_meta == meta).all()
    out_vals, out_vt = so.update_sparse(wnew_vals, meta, mt)
    assert (out_vals == wnew_vals).all()
    # the transposed copy, decompressed, is exactly (W_new * mask_RC)^T ...
    want_t = np.where(mask_rc, fresh, np.uint16(0)).T
    assert (so.unpack_2to4(out_vt, mt) == want_t).all()
    # ... and slot by slot: a slot holds a value iff the position it names is in mask_RC
    d_in, half = out_vt.shape
    for i in range(d_in):
        for g in range(half // 2):
            nib = (int(mt[i, g // 2]) >> (4 * (g & 1))) & 0xF
            for k, pos in enumerate((nib & 3, nib >> 2)):
                o = 4 * g + pos
                want = fresh[o, i] if mask_rc[o, i] else 0
                assert out_vt[i, 2 * g + k] == want


def test_update_padding_slots_exist_in_the_case_above():
    """The case must contain groups with fewer than two survivors, else the padding rule is untested."""
    w, vals, meta, vt, mt = packed_layer(d_out=64, d_in=40, seed=11)
    mask_rc = so.double_prune(so.unpack_2to4(vals, meta), so.meta_to_mask(meta))
    per_group = mask_rc.T.reshape(40, 16, 4).sum(-1)
    assert (per_group < 2).any() and (per_group == 2).any()


def test_update_then_products_use_new_weights():
    """After the update the backward operand is W_new restricted to mask_RC (Eq. 6 with new values)."""
    t = inputs.layer_inputs(6, 16, 24, 0, 31)
    vals, meta, _ = so.prune_rows_packed(t["W"])
    vt, mt, _ = so.double_prune_packed(vals, meta)
    mask_r = so.meta_to_mask(meta)
    mask_rc = so.double_prune(so.unpack_2to4(vals, meta), mask_r)
    fresh = inputs.gaussian_bf16(t["W"].shape, 0.02, 32, 1)
    nv, _ = so.pack_2to4(fresh, mask_r)
    _, nvt = so.update_sparse(nv, meta, mt)
    dx_from_packed = so.bf16_to_f64(t["dY"]) @ so.bf16_to_f64(so.unpack_2to4(nvt, mt)).T
    assert np.allclose(dx_from_packed, so.spmm_bwd_x(t["dY"], fresh, mask_rc), rtol=1e-13, atol=1e-18)
