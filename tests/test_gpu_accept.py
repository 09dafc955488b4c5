"""GPU parity: graft_accept vs the CPU oracle, bit-exact in both modes (MI355X only)."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2605_20104_amd as graft
from gpu_util import assert_same, dev, host_dict

pytestmark = pytest.mark.gpu
KEYS = ("accept_len", "best_node", "path", "out_tokens", "status")


def both(parent, tokens, n_nodes, depth_cap, target_ids=None, logits=None):
    ref = oracle.accept(parent, tokens, n_nodes, depth_cap, target_ids=target_ids, logits=logits)
    out = graft.graft_accept(dev(parent), dev(tokens), dev(n_nodes), depth_cap,
                             target_ids=dev(target_ids), logits=dev(logits, "f32"))
    return host_dict(out), ref


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_workloads_target_ids(name):
    w = inputs.get_workload(name)
    s = inputs.make_step_inputs(w)
    gpu, ref = both(s["parent"], s["tokens"], s["n_nodes"], 48, target_ids=s["target_ids"])
    assert_same(gpu, ref, KEYS)
    assert (gpu["status"] == 0).all()


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_workloads_logits(name):
    w = inputs.get_workload(name)
    s = inputs.make_step_inputs(w, with_logits=True)
    gpu, ref = both(s["parent"], s["tokens"], s["n_nodes"], 48, logits=s["logits"])
    assert_same(gpu, ref, KEYS + ("target_ids",))
    assert (gpu["target_ids"][:, :w.K] == s["target_ids"]).all()
    if name == "c1":                                        # plain random logits as well
        rng = np.random.default_rng(1)
        logits = rng.standard_normal((1, w.K, w.vocab)).astype(np.float32)
        gpu, ref = both(s["parent"], s["tokens"], s["n_nodes"], 48, logits=logits)
        assert_same(gpu, ref, KEYS + ("target_ids",))


@pytest.mark.parametrize("seed", range(8))
def test_random_small_vocab(seed):
    """Tiny vocabularies: many matches, duplicate siblings, ties in depth."""
    rng = np.random.default_rng(seed)
    B = 6
    K = [1, 2, 17, 64, 65, 128, 100, 33][seed]
    parent = np.stack([inputs.random_recursive_tree(rng, K, int(rng.integers(1, 40))) for _ in range(B)])
    tokens = rng.integers(0, 3, size=(B, K)).astype(np.int32)
    target = rng.integers(0, 3, size=(B, K)).astype(np.int32)
    n_nodes = rng.integers(1, K + 1, size=B).astype(np.int32)
    depth_cap = int(rng.integers(0, 12))
    gpu, ref = both(parent, tokens, n_nodes, depth_cap, target_ids=target)
    assert_same(gpu, ref, KEYS)


@pytest.mark.parametrize("V", [1, 3, 1003, 4096, 50001])
def test_argmax_first_maximum(V):
    rng = np.random.default_rng(V)
    B, K = 2, 9
    parent = np.stack([inputs.random_recursive_tree(rng, K, 4) for _ in range(B)])
    tokens = rng.integers(0, min(V, 5), size=(B, K)).astype(np.int32)
    logits = rng.integers(-3, 4, size=(B, K, V)).astype(np.float32)      # few distinct values: many ties
    logits[0, 1, :] = -np.inf
    logits[0, 2, V - 1] = 100.0
    gpu, ref = both(parent, tokens, [K, K - 1], 8, logits=logits)
    assert_same(gpu, ref, KEYS + ("target_ids",))


def test_bad_tree_and_overflow():
    parent = np.array([[-1, 1, 0], [-1, 0, 1]], np.int32)
    tokens = np.array([[5, 6, 7], [5, 6, 7]], np.int32)
    target = np.array([[6, 7, 8], [6, 7, 8]], np.int32)
    gpu, ref = both(parent, tokens, [3, 3], 1, target_ids=target)
    assert_same(gpu, ref, KEYS)
    assert gpu["status"].tolist() == [graft.GRAFT_STATUS_BAD_TREE, graft.GRAFT_STATUS_PATH_OVERFLOW]
    logits = np.zeros((2, 3, 10), np.float32)
    gpu, ref = both(parent, tokens, [3, 3], 1, logits=logits)
    assert_same(gpu, ref, KEYS + ("target_ids",))
