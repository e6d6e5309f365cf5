"""Pins for the oracle's N:M pruning, double pruning and packed form (CPU only)."""
import itertools
from math import comb

import numpy as np
import pytest

from oracle import slope_oracle as so
from paper_2405_16325_amd import inputs
from tests.golden_io import read_lemma_table, read_sections


def bf(x):
    return inputs.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


# ---------------------------------------------------------------- row prune
@pytest.mark.parametrize("n,m", [(2, 4), (1, 2), (2, 8), (1, 4)])
def test_prune_rows_structure_and_dominance(n, m):
    w = inputs.gaussian_bf16((64, 256), 0.02, seed=11, stream=2)
    mask = so.prune_rows(w, n, m)
    g = mask.reshape(64, -1, m)
    assert (g.sum(-1) == n).all()
    mag = np.abs(so.bf16_to_f64(w)).reshape(64, -1, m)
    kept_min = np.where(g, mag, np.inf).min(-1)
    drop_max = np.where(~g, mag, -np.inf).max(-1)
    assert (drop_max <= kept_min).all()


def brute_force_group(mag, cand, n):
    """Best subset of candidates of size min(n, #cand): maximal kept magnitude sum, and among
    equal sums the lexicographically smallest index tuple."""
    idx = [i for i in range(len(mag)) if cand[i]]
    k = min(n, len(idx))
    best, best_sum = None, None
    for sub in itertools.combinations(idx, k):
        s = sum(mag[i] for i in sub)
        if best is None or s > best_sum:
            best, best_sum = sub, s
    return set(best)


@pytest.mark.parametrize("maker", ["gauss", "coarse"])
def test_prune_rows_brute_force_all_masks(maker):
    if maker == "gauss":
        w = inputs.gaussian_bf16((4, 8), 0.02, seed=3, stream=2)
    else:
        w = inputs.coarse_weights(16, 16, seed=4)
    mask = so.prune_rows(w, 2, 4)
    mag = np.abs(so.bf16_to_f64(w))
    for r in range(w.shape[0]):
        for g0 in range(0, w.shape[1], 4):
            want = brute_force_group(list(mag[r, g0:g0 + 4]), [True] * 4, 2)
            got = {i for i in range(4) if mask[r, g0 + i]}
            assert got == want, (r, g0, mag[r, g0:g0 + 4])


def test_prune_rows_hand_built_groups():
    # (values, kept indices): ties go to the lower index, sign is ignored, +-0 are equal,
    # Inf beats finite, NaN ranks above Inf (its bit pattern is larger)
    cases = [
        ([1, 1, 1, 1], (0, 1)),
        ([0, 0, 0, 0], (0, 1)),
        ([-0.0, 0.0, 0.0, -0.0], (0, 1)),
        ([1, -2, 2, -1], (1, 2)),
        ([-3, 1, 1, 3], (0, 3)),
        ([0.5, 0.25, -0.5, 0.25], (0, 2)),
        ([1, 2, 3, 4], (2, 3)),
        ([4, 3, 2, 1], (0, 1)),
        ([0, 0, 0, 7], (0, 3)),
        ([1, np.inf, 2, -np.inf], (1, 3)),
        ([np.nan, np.inf, 5, 1], (0, 1)),
        ([1, 1, 2, 1], (0, 2)),
    ]
    w = bf(np.array([c[0] for c in cases], dtype=np.float32))
    w = np.concatenate([w, w], axis=1)  # two groups per row so that it also packs
    mask = so.prune_rows(w, 2, 4)
    for r, (_, keep) in enumerate(cases):
        assert tuple(np.flatnonzero(mask[r, :4])) == keep, cases[r]
        assert tuple(np.flatnonzero(mask[r, 4:])) == keep


def test_magnitude_key_is_monotone_in_abs_value():
    vals = np.array([0, 1e-30, 1e-3, 0.5, 1, 1.5, 2, 1e30, np.inf], dtype=np.float32)
    k = so.magnitude_key(bf(vals))
    assert (np.diff(k) > 0).all()
    assert (so.magnitude_key(bf(-vals)) == k).all()


# ---------------------------------------------------------------- double prune
def test_double_prune_structure_and_subset():
    w = inputs.gaussian_bf16((128, 96), 0.02, seed=5, stream=2)
    mr = so.prune_rows(w)
    mrc = so.double_prune(w, mr)
    assert not (mrc & ~mr).any()                                   # only adds zeros
    assert (mrc.reshape(128, -1, 4).sum(-1) <= 2).all()            # along rows
    assert (mrc.T.reshape(96, -1, 4).sum(-1) <= 2).all()           # along columns
    cand = mr.T.reshape(96, -1, 4).sum(-1)
    kept = mrc.T.reshape(96, -1, 4).sum(-1)
    assert (kept == np.minimum(cand, 2)).all()                     # never drops more than needed


@pytest.mark.parametrize("maker", ["gauss", "coarse"])
def test_double_prune_brute_force(maker):
    w = inputs.gaussian_bf16((8, 8), 0.02, seed=6, stream=2) if maker == "gauss" \
        else inputs.coarse_weights(16, 8, seed=7)
    mr = so.prune_rows(w)
    mrc = so.double_prune(w, mr)
    mag = np.abs(so.bf16_to_f64(w))
    for c in range(w.shape[1]):
        for g0 in range(0, w.shape[0], 4):
            want = brute_force_group(list(mag[g0:g0 + 4, c]), list(mr[g0:g0 + 4, c]), 2)
            got = {i for i in range(4) if mrc[g0 + i, c]}
            assert got == want


def test_double_prune_idempotent_on_transposable_pattern():
    # a pattern that is 2:4 along rows and columns already: nothing may change
    tile = np.array([[1, 1, 0, 0], [0, 0, 1, 1], [1, 1, 0, 0], [0, 0, 1, 1]], dtype=bool)
    mask = np.tile(tile, (4, 4))
    w = inputs.gaussian_bf16((16, 16), 0.02, seed=8, stream=2)
    w = np.where(mask, w | 0x0080, 0).astype(np.uint16)            # kept values are non-zero
    mr = so.prune_rows(w)
    assert (mr == mask).all()
    assert (so.double_prune(w, mr) == mask).all()


def eq8(n, m):
    s = n / m
    return sum(comb(m, j) * s**j * (1 - s) ** (m - j) * (j - n) / m for j in range(n + 1, m + 1))


def test_eq8_reproduces_printed_values():
    for n, m, printed, disagrees in read_lemma_table():
        if disagrees:
            assert abs(eq8(n, m) - printed) > 0.01      # the paper's 2:8 figure is not Eq. 8
        else:
            assert eq8(n, m) == pytest.approx(printed, abs=1e-12)


@pytest.mark.parametrize("n,m", [(2, 4), (1, 2), (2, 8)])
def test_lemma_extra_sparsity_on_iid_matrix(n, m):
    d_out, d_in = 2048, 1024
    w = inputs.gaussian_bf16((d_out, d_in), 0.02, seed=9, stream=2)
    mr = so.prune_rows(w, n, m)
    mrc = so.double_prune(w, mr, n, m)
    drop = mr.mean() - mrc.mean()
    want = eq8(n, m)
    printed = {(a, b): p for a, b, p, bad in read_lemma_table() if not bad}
    if (n, m) in printed:
        assert want == pytest.approx(printed[(n, m)], abs=1e-12)
    groups = d_out * d_in / m
    assert abs(drop - want) < 6.0 / np.sqrt(groups)
    # candidates per column group are Binomial(M, N/M) (proof of Lemma 2.1)
    cnt = mr.T.reshape(d_in, -1, m).sum(-1).ravel()
    hist = np.bincount(cnt, minlength=m + 1) / cnt.size
    s = n / m
    pmf = np.array([comb(m, j) * s**j * (1 - s) ** (m - j) for j in range(m + 1)])
    assert np.abs(hist - pmf).max() < 6.0 / np.sqrt(cnt.size)


# ---------------------------------------------------------------- packed form
def test_pack_roundtrip_and_sizes():
    w = inputs.gaussian_bf16((32, 64), 0.02, seed=10, stream=2)
    vals, meta, mbits = so.prune_rows_packed(w)
    mr = so.prune_rows(w)
    assert vals.shape == (32, 32) and vals.dtype == np.uint16
    assert meta.shape == (32, 8) and meta.dtype == np.uint8
    assert mbits.shape == (32, 8)
    # 2 x 16 bits of values + 4 bits of index per group of four (Sec. 2.1 memory analysis,
    # with two 2-bit indices in place of the 3-bit minimum of Eq. 7)
    assert (vals.nbytes + meta.nbytes) * 8 == (32 * 64 // 4) * (2 * 16 + 4)
    assert (so.unpack_2to4(vals, meta) == np.where(mr, w, 0)).all()
    assert (so.meta_to_mask(meta) == mr).all()
    assert (np.unpackbits(mbits, axis=1, bitorder="little").astype(bool) == mr).all()
    lo, hi = meta & 3, (meta >> 2) & 3
    assert (lo < hi).all() and (((meta >> 4) & 3) < (meta >> 6)).all()


def test_pack_canonical_padding():
    # kept sets with fewer than two members are padded with the lowest free positions
    cases = [((), (0, 1)), ((0,), (0, 1)), ((1,), (0, 1)), ((2,), (0, 2)), ((3,), (0, 3)),
             ((1, 3), (1, 3)), ((2, 3), (2, 3))]
    bits = bf(np.arange(1, 9, dtype=np.float32).reshape(1, 8).repeat(len(cases), 0))
    mask = np.zeros((len(cases), 8), dtype=bool)
    for r, (kept, _) in enumerate(cases):
        for i in kept:
            mask[r, i] = True
            mask[r, 4 + i] = True
    vals, meta = so.pack_2to4(bits, mask)
    for r, (kept, slots) in enumerate(cases):
        nib = slots[0] | (slots[1] << 2)
        assert meta[r, 0] == nib | (nib << 4)
        for half in range(2):
            for s, pos in enumerate(slots):
                want = bits[r, 4 * half + pos] if pos in kept else 0
                assert vals[r, 2 * half + s] == want
    assert (so.unpack_2to4(vals, meta) == np.where(mask, bits, 0)).all()
    with pytest.raises(ValueError):
        so.pack_2to4(bits, np.ones_like(mask))


def test_double_prune_packed_matches_dense_definition():
    w = inputs.coarse_weights(64, 48, seed=12)
    vals, meta, _ = so.prune_rows_packed(w)
    vt, mt, mrc_bits = so.double_prune_packed(vals, meta)
    mr = so.prune_rows(w)
    mrc = so.double_prune(w, mr)
    assert vt.shape == (48, 32) and mt.shape == (48, 8)
    assert (so.unpack_2to4(vt, mt) == np.where(mrc, w, 0).T).all()
    assert (np.unpackbits(mrc_bits, axis=1, bitorder="little").astype(bool) == mrc).all()
    # every named slot is either a kept position or a zero-valued pad
    named = so.meta_to_mask(mt)
    assert not (mrc.T & ~named).any()
    assert (so.unpack_2to4(vt, mt)[named & ~mrc.T] == 0).all()


def test_worked_example_masks_and_packing():
    gold = read_sections("worked_4x8.txt")
    w = bf(gold["W"])
    mr = so.prune_rows(w)
    assert (mr == gold["mask_R"].astype(bool)).all()
    mrc = so.double_prune(w, mr)
    assert (mrc == gold["mask_RC"].astype(bool)).all()
    vals, meta, mbits = so.prune_rows_packed(w)
    assert (vals == bf(gold["Wr_vals"])).all()
    assert (meta.ravel() == gold["Wr_meta"].ravel().astype(np.uint8)).all()
    assert (mbits.ravel() == gold["mask_R_bits"].ravel().astype(np.uint8)).all()
    assert (so.mask_to_bits(mrc).ravel() == gold["mask_RC_bits"].ravel().astype(np.uint8)).all()
