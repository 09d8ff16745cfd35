"""Data-driven draft tree (paper Sec. 4.3, appendix "Initial tree for optimization"): pins of the
oracle's two functions, and the library's host-side versions against them (no GPU needed)."""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _depths(parent):
    d = np.zeros(len(parent), int)
    for u in range(1, len(parent)):
        d[u] = d[parent[u]] + 1
    return d


def _children(parent):
    ch = [[] for _ in parent]
    for u in range(1, len(parent)):
        ch[parent[u]].append(u)
    return ch


def test_initial_tree_matches_the_paper():
    want = dict(l.split() for l in open(os.path.join(GOLD, "initial_tree_paper.txt")) if not l.startswith("#"))
    p = oracle.tree_initial(20)
    d = _depths(p)
    assert len(p) == int(want["nodes"]) and d.max() == int(want["depth"])
    ch = _children(p)
    # the rules the appendix states, checked on the result
    assert len(ch[0]) == 8
    assert [len(ch[u]) for u in ch[0]] == [8, 6, 4, 2, 1, 1, 1, 1]       # max(8 - 2 rank, 1); the first already has >= 3
    for u in range(len(p)):
        if 2 <= d[u] <= 3:
            assert len(ch[u]) >= 2
    for lv in range(20):
        first = min(u for u in range(len(p)) if d[u] == lv)
        assert len(ch[first]) >= 3                                       # leftmost node of every level
    # layout: breadth first, children contiguous in rank order
    assert all(p[u] < u for u in range(1, len(p))) and np.all(np.diff(p[1:]) >= 0) and np.all(np.diff(d) >= 0)
    # fewer levels give a prefix of the same tree
    p5 = oracle.tree_initial(5)
    assert np.array_equal(p5, p[: len(p5)]) and _depths(p5).max() == 5


def _closed_subsets(parent, size):
    n = len(parent)
    for comb in itertools.combinations(range(1, n), size - 1):
        s = {0, *comb}
        if all(parent[u] in s for u in comb):
            yield s


def test_select_is_the_best_closed_subtree():
    """Brute force on small trees: among all parent-closed node sets of the given size, the
    selected one has the largest total count when the counts come from paths (a node is never
    counted more often than its parent), and it is parent-closed for any counts."""
    rng = np.random.default_rng(3)
    parent = np.array([-1, 0, 0, 0, 1, 1, 2, 4, 4, 6], np.int32)
    ch = _children(parent)
    for trial in range(20):
        counts = np.zeros(len(parent), np.uint64)
        for _ in range(200):
            u = 0
            counts[0] += 1
            while ch[u] and rng.random() < 0.75:
                u = ch[u][int(rng.integers(len(ch[u])))]
                counts[u] += 1
        for keep in (1, 3, 5, 8, 10):
            newp, old = oracle.tree_select(parent, counts, keep)
            got = set(int(x) for x in old)
            assert len(got) == keep and all(u == 0 or parent[u] in got for u in got)
            best = max(sum(int(counts[u]) for u in s) for s in _closed_subsets(parent, keep))
            assert sum(int(counts[u]) for u in got) == best
            # re-packed tree: same shape as the kept nodes, breadth first, siblings in old order
            assert newp[0] == -1 and all(old[newp[i]] == parent[old[i]] for i in range(1, keep))
            assert np.all(np.diff(newp[1:]) >= 0)
            assert list(old) == sorted(old, key=lambda u: (_depths(parent)[u], u))
    # arbitrary counts: still closed under parents; a high count below a low one does not help
    counts = np.array([9, 1, 5, 0, 8, 0, 7, 9, 0, 9], np.uint64)
    newp, old = oracle.tree_select(parent, counts, 4)
    assert set(old) == {0, 2, 6, 9}          # usable counts: 2 -> 5, 6 -> 5, 9 -> 5; 1 -> 1 and its subtree -> 1
    assert list(newp) == [-1, 0, 1, 2]


def test_library_tree_functions_equal_the_oracle():
    binding = pytest.importorskip("paper_2506_04708_amd.binding")
    for levels in (1, 3, 7, 20):
        assert np.array_equal(binding.tree_initial(levels), oracle.tree_initial(levels))
    p = oracle.tree_initial(20)
    rng = np.random.default_rng(8)
    ch = _children(p)
    counts = np.zeros(len(p), np.uint64)
    for _ in range(4000):
        u = 0
        counts[0] += 1
        while ch[u] and rng.random() < 0.8:
            u = ch[u][min(int(rng.geometric(0.45)) - 1, len(ch[u]) - 1)]
            counts[u] += 1
    for keep in (1, 2, 16, 80, 300, 625):
        a, ao = oracle.tree_select(p, counts, keep)
        b, bo = binding.tree_select(p, counts, keep)
        assert np.array_equal(a, b) and np.array_equal(ao, bo)
    arbitrary = rng.integers(0, 30, len(p)).astype(np.uint64)                # many ties, not monotone
    for keep in (5, 64, 128):
        a, ao = oracle.tree_select(p, arbitrary, keep)
        b, bo = binding.tree_select(p, arbitrary, keep)
        assert np.array_equal(a, b) and np.array_equal(ao, bo)
    with pytest.raises(RuntimeError):
        binding.tree_select(np.array([-1, 0, 1, 0], np.int32), np.ones(4, np.uint64), 2)   # children not contiguous
