"""Pins for the oracle's usage count and dictionary reduction (Section IV.B, second narrowing
criterion: keep the patterns that win most often over random kernels)."""
import numpy as np
import pytest

import oracle
from paper_2303_02191_amd import workloads as wl


def test_histogram_is_a_count():
    idx = np.array([0, 3, 3, 1, 250, 3, 0], dtype=np.uint8)
    assert oracle.histogram(idx, 4).tolist() == [2, 1, 0, 3]  # 250 is outside the dictionary
    # brute force on random data, and the counts add up to the number of groups
    rng = np.random.default_rng(0)
    idx = rng.integers(0, 22, 5000).astype(np.uint8)
    h = oracle.histogram(idx, 22)
    assert h.sum() == 5000
    for p in range(22):
        assert h[p] == sum(1 for v in idx.tolist() if v == p)


def test_reduce_keeps_most_used_in_dictionary_order():
    masks = np.array([0b11, 0b110, 0b1001, 0b10010, 0b100100], dtype=np.uint16)
    counts = np.array([5, 9, 5, 1, 7])
    out, kept = oracle.reduce_dict(masks, counts, 3)
    # ranking 1 (9), 4 (7), then the tie 0 vs 2 at 5 goes to the lower index; original order restored
    assert kept.tolist() == [0, 1, 4]
    assert out.tolist() == [0b11, 0b110, 0b100100]
    out, kept = oracle.reduce_dict(masks, counts, 5)
    assert kept.tolist() == [0, 1, 2, 3, 4] and out.tolist() == masks.tolist()
    out, kept = oracle.reduce_dict(masks, counts, 1)
    assert kept.tolist() == [1]


def test_unfiltered_dictionary_is_used_uniformly():
    # With every k-subset in the dictionary and iid weights, all patterns are exchangeable: each
    # wins with probability 1 / C(9, k) (Eq. 1 count).  Pins select + histogram against a closed form.
    k, n = 2, 180000
    masks = oracle.pattern_dict(k, oracle.RULE_ALL)
    assert len(masks) == 36
    _, w = wl.draw_random_kernels(11, n, wl.F32)
    h = oracle.histogram(oracle.select(w, masks), len(masks))
    p = 1.0 / 36
    sigma = np.sqrt(n * p * (1 - p))
    assert h.sum() == n
    assert np.all(np.abs(h - n * p) < 5 * sigma), h


def test_connected_dictionary_prefers_nothing_by_symmetry():
    # The 3x3 grid's 8 symmetries permute the connected patterns, and iid weights are invariant under
    # them: patterns in one orbit are used equally often.
    n = 120000
    masks = oracle.pattern_dict(2, oracle.RULE_CONNECTED4)
    assert len(masks) == 12
    _, w = wl.draw_random_kernels(12, n, wl.F32)
    h = oracle.histogram(oracle.select(w, masks), 12)
    # two orbits: dominoes touching the centre (4) and dominoes along the border (8)
    centre = [i for i, m in enumerate(masks.tolist()) if m >> 4 & 1]
    border = [i for i in range(12) if i not in centre]
    assert len(centre) == 4 and len(border) == 8
    for orbit in (centre, border):
        mean = h[orbit].mean()
        sigma = np.sqrt(mean * (1 - mean / n))
        assert np.all(np.abs(h[orbit] - mean) < 5 * sigma), (orbit, h)


def test_reduced_dictionary_reselects_consistently():
    # Kernels whose winner survives the reduction keep the same pattern (same mask) afterwards.
    masks = oracle.pattern_dict(3, oracle.RULE_CONNECTED4)
    _, w = wl.draw_random_kernels(13, 20000, wl.F16)
    idx = oracle.select(w, masks)
    h = oracle.histogram(idx, len(masks))
    red, kept = oracle.reduce_dict(masks, h, 10)
    idx2 = oracle.select(w, red)
    survived = np.isin(idx, kept)
    assert survived.any() and (~survived).any()
    assert np.array_equal(red[idx2[survived]], masks[idx[survived]])
