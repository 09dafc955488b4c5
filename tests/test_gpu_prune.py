"""GPU parity of graft_prune_select against the CPU oracle (bit-exact: the fp32 scores decide integers
and both sides accumulate them in the same order)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_20104_amd as graft
from gpu_util import dev, host

pytestmark = pytest.mark.gpu
KEYS = ("parent", "tokens", "index", "n_nodes", "stage", "n_ret", "status")


def _both(parent, tokens, logq, n_nodes, chk_depth, log_tau, keep, ret):
    ref = oracle.prune_select(parent, tokens, logq, n_nodes, chk_depth, log_tau, keep, ret)
    out = graft.graft_prune_select(dev(parent), dev(tokens), dev(logq, "f32"), dev(n_nodes), dev(chk_depth),
                                   dev(log_tau, "f32"), dev(keep), dev(ret))
    torch.cuda.synchronize()
    for k in KEYS:
        assert (host(out[k]) == ref[k]).all(), (k, host(out[k]), ref[k])
    return ref


def _trees(rng, B, K, n_nodes, max_depth=None):
    parent = np.full((B, K), -1, np.int32)
    for b in range(B):
        depth = [0]
        for i in range(1, n_nodes[b]):
            while True:
                p = int(rng.integers(0, i))
                if max_depth is None or depth[p] < max_depth:
                    break
            parent[b, i] = p
            depth.append(depth[p] + 1)
    return parent


@pytest.mark.parametrize("B,K,seed", [(1, 16, 0), (4, 60, 1), (8, 128, 2), (3, 7, 3), (2, 1, 4)])
def test_prune_select_random(B, K, seed):
    rng = np.random.default_rng(seed)
    n_nodes = rng.integers(1, K + 1, B).astype(np.int32)
    n_nodes[0] = K
    parent = _trees(rng, B, K, n_nodes, max_depth=9)
    tokens = rng.integers(0, 150000, (B, K)).astype(np.int32)
    logq = np.log(rng.random((B, K)).astype(np.float32) * 0.98 + 0.01).astype(np.float32)   # inexact sums
    logq[:, : K // 3] = -np.round(rng.random((B, K // 3)) * 8).astype(np.float32) / 4            # and exact ties
    chk = ([1, 2, 6], [8, 24, 40], [52, 36, 20])
    for log_tau in ([-0.7, -1.5, -4.0], [-20.0, -1.0, -3.0], [-50.0, -50.0, -50.0], [0.5, 0.0, 0.0],
                    [-0.2, -50.0, -50.0]):
        _both(parent, tokens, logq, n_nodes, chk[0], log_tau, chk[1], chk[2])
    # no checkpoint at all, and the maximum number of them
    _both(parent, tokens, logq, n_nodes, np.zeros(0, np.int32), np.zeros(0, np.float32), np.zeros(0, np.int32),
          np.zeros(0, np.int32))
    n16 = graft.GRAFT_MAX_CHECKPOINTS
    _both(parent, tokens, logq, n_nodes, np.arange(1, n16 + 1), np.linspace(-30, -1, n16), np.arange(1, n16 + 1) * 3,
          np.arange(n16))


def test_prune_select_deep_chain_and_star():
    K = 128
    chain = np.arange(-1, K - 1, dtype=np.int32)[None]
    star = np.concatenate([[-1], np.zeros(K - 1, np.int32)])[None].astype(np.int32)
    parent = np.concatenate([chain, star])
    tokens = np.tile(np.arange(K, dtype=np.int32), (2, 1))
    logq = np.full((2, K), np.log(0.9), np.float32)
    _both(parent, tokens, logq, [K, K], [1, 64, 127], [-0.05, -6.0, -13.0], [10, 70, 100], [5, 6, 7])
    _both(parent, tokens, logq, [K, K], [127], [-13.4], [100], [28])


def test_prune_select_error_paths():
    parent = np.array([[-1, 0, 3, 1], [-1, 0, 1, 2], [-1, 0, 0, 0], [0, 0, 0, 0]], np.int32)
    logq = np.array([[0, -1, -1, -1], [0, -5, 4, -1], [0, -1, -1, -1], [0, -1, -1, -1]], np.float32)
    # (checkpoint at depth 2, so that the node whose positive log q lifts it above its parent is a candidate)
    ref = _both(parent, np.zeros((4, 4), np.int32), logq, [4, 4, 5, 4], [2], [0.0], [2], [7])
    assert ref["status"].tolist() == [graft.GRAFT_STATUS_BAD_TREE] * 4
