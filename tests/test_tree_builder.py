"""Drafting-tree construction (Algorithm 3): the oracle against brute force and closed forms, and the library's
host function against the oracle.  No GPU."""
import itertools

import numpy as np
import pytest

from oracle import tree_builder as tb


def _lib():
    from paper_2504_15475_amd import race
    race.lib()
    return race


def _is_tree(vertices, nr):
    seen = {()}
    for idx in vertices:
        assert idx not in seen
        assert idx[:-1] in seen, f"{idx}: parent missing"
        assert 0 <= idx[-1] < nr
        assert idx[-1] == 0 or idx[:-1] + (idx[-1] - 1,) in seen, f"{idx}: earlier sibling missing"
        seen.add(idx)


# ----------------------------------------------------------------------------- oracle pins
@pytest.mark.parametrize("r", [(0.6, 0.25, 0.1), (0.9, 0.05), (0.5, 0.5, 0.3, 0.2), (0.33,)], ids=str)
@pytest.mark.parametrize("k", [1, 2, 5, 7])
def test_oracle_tree_is_the_best_k_vertex_set_by_brute_force(r, k):
    # Section 4: the optimal tree consists of the k vertices with the largest acceptance probability
    every = [idx for d in range(1, k + 1) for idx in itertools.product(range(len(r)), repeat=d)]
    best = sorted((tb.acceptance(r, idx) for idx in every), reverse=True)[:k]
    tree = tb.optimal_tree(r, k)
    assert len(tree) == k
    _is_tree(tree, len(r))
    assert sum(tb.acceptance(r, idx) for idx in tree) == pytest.approx(sum(best), rel=1e-13)


def test_oracle_special_cases():
    # one arrival per context: a chain, expected accepted tokens a + a^2 + ... (geometric)
    a = 0.7
    tree = tb.optimal_tree((a,), 6)
    assert tree == [(0,) * d for d in range(1, 7)]
    assert sum(tb.acceptance((a,), i) for i in tree) == pytest.approx(a * (1 - a**6) / (1 - a))
    # a hopeless continuation (r0^2 < every r_j): all k vertices are alternatives at the root (the batch strategy)
    r = (0.3, 0.25, 0.2, 0.15)
    assert tb.optimal_tree(r, 4) == [(0,), (1,), (2,), (3,)]
    # vertices join in order of decreasing R
    vals = [tb.acceptance((0.6, 0.3, 0.1), i) for i in tb.optimal_tree((0.6, 0.3, 0.1), 40)]
    assert all(x >= y for x, y in zip(vals, vals[1:]))
    # flat layout
    par, rk = tb.flat([(0,), (1,), (0, 0), (1, 0), (0, 0, 1)][:4])
    assert par == [-1, -1, 0, 1] and rk == [0, 1, 0, 0]


def test_oracle_specinfer_tree_shape():
    t = tb.specinfer_tree(11)
    assert t[:2] == [(0,), (0, 0)]
    assert t[2:5] == [(0, 0, 0), (0, 0, 1), (0, 0, 2)]
    assert t[5:8] == [(0, 0, 0, 0), (0, 0, 1, 0), (0, 0, 2, 0)]
    assert len(t) == 11 and len(set(t)) == 11
    assert tb.specinfer_tree(1) == [(0,)]
    assert tb.specinfer_tree(4, shared=0, branches=2) == [(0,), (1,), (0, 0), (1, 0)]


# ----------------------------------------------------------------------------- library against the oracle
def test_library_tree_equals_oracle_tree():
    race = _lib()
    rng = np.random.default_rng(12)
    for trial in range(40):
        nr = int(rng.integers(1, 9))
        r = np.sort(rng.random(nr))[::-1] * rng.uniform(0.3, 1.0)
        if trial % 5 == 0:
            r = np.round(r, 1)  # equal values: depth, then index tuple, decide
        k = int(rng.integers(1, 200))
        parent, rank, acc, total = race.tree_build_optimal(r, k)
        ref = tb.optimal_tree(tuple(r), k)
        rp, rr = tb.flat(ref)
        assert parent.tolist() == rp and rank.tolist() == rr
        assert acc.tolist() == [tb.acceptance(tuple(r), i) for i in ref]
        assert total == pytest.approx(sum(acc), rel=1e-12)
        assert race.arrival_tree_validate_host(parent, rank)


def test_library_tree_large_and_argument_errors():
    race = _lib()
    parent, rank, acc, total = race.tree_build_optimal([0.8, 0.1, 0.05], 8192)
    assert race.arrival_tree_validate_host(parent, rank)
    assert np.all(np.diff(acc) <= 0) and total == pytest.approx(acc.sum())
    for bad in ([], [1.5], [float("nan")], [-0.1], [0.3, 0.5]):   # the last: acceptance must not increase with the rank
        with pytest.raises(race.ErsdError):
            race.tree_build_optimal(bad, 4)
    with pytest.raises(race.ErsdError):
        race.tree_build_optimal([0.5], 0)


def test_library_specinfer_tree_equals_oracle():
    race = _lib()
    for k, shared, branches in [(1, 2, 3), (2, 2, 3), (11, 2, 3), (64, 2, 3), (9, 0, 2), (20, 5, 4)]:
        parent, rank = race.tree_build_specinfer(k, shared, branches)
        rp, rr = tb.flat(tb.specinfer_tree(k, shared, branches))
        assert parent.tolist() == rp and rank.tolist() == rr
        assert race.arrival_tree_validate_host(parent, rank)
    with pytest.raises(race.ErsdError):
        race.tree_build_specinfer(0)
