"""Pins for the oracle's ancestor masks, depths, positions and leaf paths (no GPU)."""
import os

import numpy as np
import pytest

import inputs
import oracle
from _golden import GOLDEN, groups, ints, read_fixture


def bits(words):
    return [j for j in range(128) if (int(words[j // 64]) >> (j % 64)) & 1]


def test_golden_small():
    fx = read_fixture("tree_small.txt")
    parent = np.array([ints(fx["parent"])], np.int32)
    n = parent.shape[1]
    r = oracle.build_tree_mask(parent, [n], [10], n_leaf_max=4, depth_cap=3)
    assert [bits(r["mask"][0, i]) for i in range(n)] == groups(fx["mask"])
    assert r["depth"][0].tolist() == ints(fx["depth"])
    assert r["pos"][0].tolist() == ints(fx["pos"])
    want = groups(fx["paths"])
    for row, p in enumerate(want):
        assert r["paths"][0, row, :len(p)].tolist() == p
        assert (r["paths"][0, row, len(p):] == -1).all()
    assert (r["paths"][0, len(want):] == -1).all()
    assert r["status"][0] == 0


def test_chain_closed_form():
    n = 100                                      # spans both mask words
    parent = np.arange(-1, n - 1, dtype=np.int32)[None, :]
    r = oracle.build_tree_mask(parent, [n], [7], n_leaf_max=2, depth_cap=n)
    for i in range(n):
        assert bits(r["mask"][0, i]) == list(range(i + 1))   # lower triangle
        assert r["depth"][0, i] == i and r["pos"][0, i] == 7 + i
    assert r["paths"][0, 0, :n].tolist() == list(range(n))
    assert (r["paths"][0, 1] == -1).all()


def test_star_closed_form():
    n = 128
    parent = np.zeros((1, n), np.int32)
    parent[0, 0] = -1
    r = oracle.build_tree_mask(parent, [n], [0], n_leaf_max=n, depth_cap=1)
    assert bits(r["mask"][0, 0]) == [0]
    for i in range(1, n):
        assert bits(r["mask"][0, i]) == [0, i] and r["depth"][0, i] == 1
        assert r["paths"][0, i - 1].tolist() == [0, i]
    assert (r["paths"][0, n - 1] == -1).all()


@pytest.mark.parametrize("seed", range(8))
def test_invariants_and_python_walk(seed):
    rng = np.random.default_rng(seed)
    B, K = 3, int(rng.integers(2, 129))
    parent = np.stack([inputs.random_recursive_tree(rng, K, 64) for _ in range(B)])
    n_nodes = rng.integers(1, K + 1, size=B).astype(np.int32)
    prefix = rng.integers(0, 5000, size=B).astype(np.int32)
    r = oracle.build_tree_mask(parent, n_nodes, prefix, n_leaf_max=K, depth_cap=K)
    for b in range(B):
        n = int(n_nodes[b])
        leaves = []
        for i in range(K):
            m = r["mask"][b, i]
            if i >= n:
                assert int(m[0]) == 0 and int(m[1]) == 0 and r["pos"][b, i] == -1 and r["depth"][b, i] == -1
                continue
            anc, j = [], i
            while j != -1:
                anc.append(j)
                j = int(parent[b, j])
            assert bits(m) == sorted(anc)
            assert len(bits(m)) == r["depth"][b, i] + 1
            assert r["pos"][b, i] == prefix[b] + len(anc) - 1
            if i > 0:
                pm = r["mask"][b, parent[b, i]]
                want = [int(pm[0]), int(pm[1])]
                want[i // 64] |= 1 << (i % 64)
                assert [int(m[0]), int(m[1])] == want
            if not any(parent[b, c] == i for c in range(i + 1, n)):
                leaves.append(anc[::-1])
        for row, p in enumerate(leaves):
            assert r["paths"][b, row, :len(p)].tolist() == p
        assert (r["paths"][b, len(leaves):] == -1).all()


def test_workload_trees_fill_the_budget():
    """Budgets the paper prints (Sec. 3.2; App. A.1 table): 8+52 = 24+36 = 40+20 = 60."""
    rows = {}
    with open(os.path.join(GOLDEN, "budget_split.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) == 4:
                rows[line[0]] = line[1:]
    for stage in ("d0", "d1", "d5"):
        keep, ret, dist = rows[stage]
        assert int(keep) + int(ret) == 60
        assert sum(int(x) for x in dist.split("+")) == int(ret)
    assert sum(int(x) for x in rows["full"][2].split("+")) == 80
    # the generators' trees: draft nodes retained per the d1 / d5 stages, the rest grafted
    for name, keep in (("c2", 24), ("c3", 40)):
        w = inputs.get_workload(name)
        s = inputs.make_step_inputs(w)
        assert int((s["kind"][0] == 0).sum()) == keep and s["n_nodes"][0] == w.K
        r = oracle.build_tree_mask(s["parent"], s["n_nodes"], s["prefix_len"])
        assert r["status"][0] == 0 and (r["pos"][0] >= w.P).all()


def test_bad_trees_flagged():
    parent = np.array([[-1, 0, 2, 1], [0, 0, 1, 1], [-1, 0, -1, 1], [-1, 0, 1, 2]], np.int32)
    r = oracle.build_tree_mask(parent, [4, 4, 4, 5], [3, 3, 3, 3], n_leaf_max=2, depth_cap=2)
    assert r["status"].tolist() == [oracle.ST_BAD_TREE] * 4
    assert (r["mask"] == 0).all() and (r["pos"] == -1).all() and (r["paths"] == -1).all()


def test_path_overflow_flag():
    parent = np.array([[-1, 0, 1, 2, 0, 0]], np.int32)      # leaves 3 (depth 3), 4, 5
    r = oracle.build_tree_mask(parent, [6], [0], n_leaf_max=2, depth_cap=2)
    assert r["status"][0] == oracle.ST_PATH_OVERFLOW
    assert (r["paths"][0, 0] == -1).all()                    # too deep: blank row
    assert r["paths"][0, 1].tolist() == [0, 4, -1]           # third leaf dropped
