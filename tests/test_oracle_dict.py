"""Pins for the oracle's pattern dictionary (Section IV.B, Eq. 1 and the adjacency filter)."""
import itertools
import os
from math import comb

import numpy as np
import pytest

import oracle


def _read_pairs(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a, b = line.split()
        out[a] = b
    return out


def test_eq1_counts_golden(golden_dir):
    g = _read_pairs(os.path.join(golden_dir, "eq1_candidate_counts.txt"))
    for k in range(1, 9):
        assert int(g[str(k)]) == comb(9, k)  # the fixture is Eq. 1 evaluated
        masks = oracle.pattern_dict(k, oracle.RULE_ALL)
        assert len(masks) == int(g[str(k)])
        assert len(set(masks.tolist())) == len(masks)
        assert all(bin(m).count("1") == k for m in masks.tolist())


def _components(taps, eight):
    """Independent connectivity check: union-find over coordinate pairs."""
    parent = {t: t for t in taps}

    def find(a):
        while parent[a] != a:
            a = parent[a]
        return a

    for a, b in itertools.combinations(taps, 2):
        (ra, ca), (rb, cb) = divmod(a, 3), divmod(b, 3)
        adj = max(abs(ra - rb), abs(ca - cb)) == 1 if eight else abs(ra - rb) + abs(ca - cb) == 1
        if adj:
            parent[find(a)] = find(b)
    return len({find(t) for t in taps})


def _has_pair4(taps):
    if len(taps) == 1:
        return True
    return any(abs(a // 3 - b // 3) + abs(a % 3 - b % 3) == 1 for a, b in itertools.combinations(taps, 2))


@pytest.mark.parametrize("k", range(1, 9))
def test_rules_against_independent_search(k):
    expect = {oracle.RULE_ALL: [], oracle.RULE_ANYPAIR4: [], oracle.RULE_CONNECTED4: [], oracle.RULE_CONNECTED8: []}
    for taps in itertools.combinations(range(9), k):  # ascending tuples, lexicographic order
        m = sum(1 << t for t in taps)
        expect[oracle.RULE_ALL].append(m)
        if _has_pair4(taps):
            expect[oracle.RULE_ANYPAIR4].append(m)
        if _components(taps, False) == 1:
            expect[oracle.RULE_CONNECTED4].append(m)
        if _components(taps, True) == 1:
            expect[oracle.RULE_CONNECTED8].append(m)
    for rule, want in expect.items():
        got = oracle.pattern_dict(k, rule).tolist()
        assert got == want  # same members AND same order (pattern index = rank)


def test_two_entry_patterns_are_grid_edges():
    # closed form: the 3x3 grid graph has 2 * 3 * 2 = 12 edges
    masks = oracle.pattern_dict(2, oracle.RULE_CONNECTED4).tolist()
    assert len(masks) == 12
    assert masks == oracle.pattern_dict(2, oracle.RULE_ANYPAIR4).tolist()
    # each edge joins one odd-numbered tap (edge midpoint) and one even-numbered tap
    for m in masks:
        taps = [t for t in range(9) if m >> t & 1]
        assert sorted(t % 2 for t in taps) == [0, 1]


def test_three_entry_connected_count_closed_form():
    # 3 rows + 3 columns (straight) + 4 corners-of-a-2x2-block x 4 blocks (L shapes) = 22
    assert len(oracle.pattern_dict(3, oracle.RULE_CONNECTED4)) == 6 + 16


def _sym_images(m):
    out = set()
    for rot in range(4):
        for flip in (False, True):
            mm = 0
            for t in range(9):
                if not m >> t & 1:
                    continue
                r, c = divmod(t, 3)
                if flip:
                    c = 2 - c
                for _ in range(rot):
                    r, c = c, 2 - r
                mm |= 1 << (3 * r + c)
            out.add(mm)
    return out


@pytest.mark.parametrize("rule", [0, 1, 2, 3])
@pytest.mark.parametrize("k", [2, 3, 4, 5])
def test_dictionary_closed_under_grid_symmetries(k, rule):
    s = set(oracle.pattern_dict(k, rule).tolist())
    for m in s:
        assert _sym_images(m) <= s


def test_bad_arguments():
    with pytest.raises(ValueError):
        oracle.pattern_dict(0)
    with pytest.raises(ValueError):
        oracle.pattern_dict(3, 7)
    assert oracle.pattern_dict(9, oracle.RULE_ALL).tolist() == [0x1FF]
