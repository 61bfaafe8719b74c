"""Pins for the oracle's pattern selection and masking (Section IV.C Algorithm 2,
Section IV.D Algorithm 3)."""
import os

import numpy as np
import pytest

import oracle


def _rng(seed):
    return np.random.default_rng(seed)


def _taps(m):
    return [t for t in range(9) if m >> t & 1]


@pytest.mark.parametrize("k,rule", [(2, 2), (3, 2), (4, 2), (3, 0), (5, 3)])
def test_winner_is_exhaustive_argmax(k, rule):
    masks = oracle.pattern_dict(k, rule)
    w = _rng(k * 10 + rule).standard_normal((40, 7, 3, 3))
    idx = oracle.select(w, masks)
    assert idx.shape == (280,)
    flat = w.reshape(-1, 9)
    for g in range(flat.shape[0]):
        scores = [float(np.sum(flat[g, _taps(m)] ** 2)) for m in masks.tolist()]
        # retained norm of the winner >= every other pattern's (random reals: no ties)
        assert scores[idx[g]] >= max(scores) - 1e-15
        assert int(np.argmax(scores)) == idx[g]


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 8])
def test_unfiltered_dictionary_is_magnitude_pruning(k):
    # With every k-subset allowed, the best pattern keeps the k largest |w| of each kernel:
    # textbook magnitude pruning, checked against a sort.
    masks = oracle.pattern_dict(k, oracle.RULE_ALL)
    w = _rng(100 + k).standard_normal((300, 9))
    idx = oracle.select(w, masks)
    for g in range(300):
        keep = set(np.argsort(-np.abs(w[g]))[:k].tolist())
        assert set(_taps(int(masks[idx[g]]))) == keep


def test_ties_go_to_lowest_index():
    masks = oracle.pattern_dict(3)
    # all weights equal: every pattern scores the same -> index 0
    assert oracle.select(np.full(9, 0.5), masks).tolist() == [0]
    assert oracle.select(np.zeros(18), masks).tolist() == [0, 0]
    # two disjoint patterns get identical energy, all others less: lower index wins
    m = masks.tolist()
    a, b = 5, 17
    ta, tb = _taps(m[a]), _taps(m[b])
    w = np.zeros(9)
    for t in set(ta) | set(tb):
        w[t] = 1.0
    scores = [sum(w[t] ** 2 for t in _taps(x)) for x in m]
    first_best = int(np.argmax(scores))  # numpy argmax returns the first maximum
    assert oracle.select(w, masks).tolist() == [first_best]
    # low-precision weights: few distinct magnitudes, so ties are frequent
    w16 = _rng(7).standard_normal((2000, 9)).astype(np.float16).astype(np.float64)
    w16 = np.round(w16 * 4) / 4
    idx = oracle.select(w16, masks)
    for g in range(2000):
        scores = [sum(w16[g, t] * w16[g, t] for t in _taps(x)) for x in m]
        assert idx[g] == int(np.argmax(scores))


def test_nan_and_inf():
    masks = oracle.pattern_dict(2)  # pattern 0 = taps {0,1}, pattern 1 = taps {0,3}, pattern 2 = {1,2}
    m = masks.tolist()
    assert _taps(m[0]) == [0, 1] and _taps(m[2]) == [1, 2]
    w = np.zeros(9)
    w[0] = np.nan  # poisons patterns 0 and 1 only
    w[4], w[5] = 1.0, 1.0
    want = m.index((1 << 4) | (1 << 5))
    assert oracle.select(w, masks).tolist() == [want]
    assert oracle.select(np.full(9, np.nan), masks).tolist() == [0]  # all-NaN -> 0
    w = np.ones(9)
    w[8] = np.inf
    first_with_8 = min(i for i, x in enumerate(m) if x >> 8 & 1)
    assert oracle.select(w, masks).tolist() == [first_with_8]
    w[0] = -np.inf  # +inf scores tie -> lowest index among patterns that touch tap 0 or 8
    first_inf = min(i for i, x in enumerate(m) if (x >> 8 & 1) or (x & 1))
    assert oracle.select(w, masks).tolist() == [first_inf]


def _apply_sym(t, rot, flip):
    r, c = divmod(t, 3)
    if flip:
        c = 2 - c
    for _ in range(rot):
        r, c = c, 2 - r
    return 3 * r + c


@pytest.mark.parametrize("rot,flip", [(1, False), (2, False), (0, True), (3, True)])
def test_grid_symmetry_covariance(rot, flip):
    # Rotating / reflecting every kernel moves the winning mask the same way.
    masks = oracle.pattern_dict(3)
    m = masks.tolist()
    w = _rng(5).standard_normal((500, 9))
    perm = [_apply_sym(t, rot, flip) for t in range(9)]
    w2 = np.empty_like(w)
    w2[:, perm] = w
    i1, i2 = oracle.select(w, masks), oracle.select(w2, masks)
    for g in range(500):
        moved = sum(1 << perm[t] for t in _taps(m[i1[g]]))
        assert m[i2[g]] == moved


def test_mask_invariants_3x3(golden_dir):
    printed = {}
    for line in open(os.path.join(golden_dir, "table3_reduction_ratio.txt")):
        if line.strip() and not line.startswith("#"):
            k, r = line.split()
            printed[int(k)] = float(r)
    w = _rng(11).standard_normal((16, 24, 3, 3)) + 3.0  # shifted: no weight is zero
    for k in (2, 3, 4, 5):
        masks = oracle.pattern_dict(k)
        idx = oracle.select(w, masks)
        wm = oracle.mask(w, masks, idx)
        nz = wm.reshape(-1, 9) != 0
        assert (nz.sum(axis=1) == k).all()  # exactly k survivors in every kernel
        assert np.array_equal(wm[wm != 0], w[wm != 0])  # survivors are untouched
        # Table 3 reduction ratios are ~ 9/k, i.e. total / surviving parameters
        assert abs(w.size / nz.sum() - printed[k]) < 0.11


def test_mask_1x1_flat_view_and_tail():
    # Section IV.D: flatten the whole [Co, Ci] tensor row-major, chunks of 9 that may cross
    # rows, left-over (< 9) weights pruned.  256 x 256 -> 7281 groups + 7 left over.
    masks = oracle.pattern_dict(2)
    w = _rng(3).standard_normal((256, 256, 1, 1)) + 2.0
    idx = oracle.select(w, masks)
    assert idx.size == 7281
    wm = oracle.mask(w, masks, idx)
    flat, flatm = w.reshape(-1), wm.reshape(-1)
    assert np.count_nonzero(flatm) == 14562
    assert (flatm[-7:] == 0).all()
    assert np.array_equal(flatm[flatm != 0], flat[flatm != 0])
    # group 28 starts at flat offset 252 and straddles rows 0 and 1
    g = 28
    chunk = flat[9 * g:9 * g + 9]
    scores = [sum(chunk[t] ** 2 for t in _taps(m)) for m in masks.tolist()]
    assert idx[g] == int(np.argmax(scores))
    # flat view of a 3x3 tensor is the per-kernel view
    w3 = _rng(4).standard_normal((5, 6, 3, 3))
    assert np.array_equal(oracle.select(w3, masks), oracle.select(w3.reshape(-1), masks))
