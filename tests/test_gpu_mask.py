"""GPU parity: graft_build_tree_mask vs the CPU oracle, bit-exact (MI355X only)."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2605_20104_amd as graft
from gpu_util import assert_same, dev, host_dict

pytestmark = pytest.mark.gpu
KEYS = ("mask", "pos", "depth", "status")


def both(parent, n_nodes, prefix, n_leaf_max=0, depth_cap=0):
    ref = oracle.build_tree_mask(parent, n_nodes, prefix, n_leaf_max, depth_cap)
    out = graft.graft_build_tree_mask(dev(parent), dev(n_nodes), dev(prefix), n_leaf_max, depth_cap)
    return host_dict(out), ref


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_workloads(name):
    w = inputs.get_workload(name)
    s = inputs.make_step_inputs(w)
    gpu, ref = both(s["parent"], s["n_nodes"], s["prefix_len"], n_leaf_max=w.K, depth_cap=40)
    assert_same(gpu, ref, KEYS + ("paths",))
    assert (gpu["status"] == 0).all()


@pytest.mark.parametrize("seed", range(8))
def test_random_trees(seed):
    rng = np.random.default_rng(seed)
    B = 7
    K = [1, 2, 63, 64, 65, 127, 128, 100][seed]
    parent = np.stack([inputs.random_recursive_tree(rng, K, int(rng.integers(1, 130))) for _ in range(B)])
    n_nodes = rng.integers(1, K + 1, size=B).astype(np.int32)
    n_nodes[0] = K
    prefix = rng.integers(0, 100000, size=B).astype(np.int32)
    n_leaf_max = int(rng.integers(1, K + 1))
    depth_cap = int(rng.integers(0, min(K, 127)))
    gpu, ref = both(parent, n_nodes, prefix, n_leaf_max, depth_cap)
    assert_same(gpu, ref, KEYS + ("paths",))
    gpu, ref = both(parent, n_nodes, prefix)              # without the path table
    assert_same(gpu, ref, KEYS)


def test_chain_and_star_128():
    chain = np.arange(-1, 127, dtype=np.int32)
    star = np.zeros(128, np.int32)
    star[0] = -1
    gpu, ref = both(np.stack([chain, star]), [128, 128], [5, 6], n_leaf_max=128, depth_cap=127)
    assert_same(gpu, ref, KEYS + ("paths",))


def test_bad_trees_and_dirty_outputs():
    parent = np.array([[-1, 0, 2, 1], [0, 0, 1, 1], [-1, 0, -1, 1], [-1, 0, 1, 2], [-1, 0, 0, 2]], np.int32)
    n_nodes = np.array([4, 4, 4, 5, 4], np.int32)
    prefix = np.array([3, 3, 3, 3, 3], np.int32)
    ref = oracle.build_tree_mask(parent, n_nodes, prefix, 3, 2)
    out = {"mask": torch.full((5, 4, 2), -7, dtype=torch.int64, device="cuda"),
           "pos": torch.full((5, 4), 99, dtype=torch.int32, device="cuda"),
           "depth": torch.full((5, 4), 99, dtype=torch.int32, device="cuda"),
           "paths": torch.full((5, 3, 3), 99, dtype=torch.int32, device="cuda"),
           "status": torch.full((5,), 99, dtype=torch.int32, device="cuda")}
    graft.graft_build_tree_mask(dev(parent), dev(n_nodes), dev(prefix), 3, 2, out=out)
    gpu = host_dict(out)
    assert_same(gpu, ref, KEYS + ("paths",))
    assert gpu["status"].tolist() == [2, 2, 2, 2, 0]
