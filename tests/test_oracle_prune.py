"""Pins of the oracle's confidence gates and draft-node selection (Sec. 3.1; App. A Alg. 2; App. E)."""
import math

import numpy as np

import inputs
import oracle
from _golden import ints, read_fixture


def _fix(g, key):
    return np.array(ints(g[key]), np.float32) / 8.0


def test_hand_worked_gates_and_selection():
    g = read_fixture("prune_small.txt")
    parent, tokens = [ints(g["parent"])], [ints(g["tokens"])]
    logq = _fix(g, "logq8")[None]
    r = oracle.prune_select(parent, tokens, logq, [7], ints(g["chk_depth"]), _fix(g, "chk_log_tau8"),
                            ints(g["chk_keep"]), ints(g["chk_ret"]))
    assert r["status"].tolist() == [0] and r["stage"].tolist() == [int(g["stage"])]
    assert r["n_nodes"].tolist() == [4] and r["n_ret"].tolist() == [int(g["n_ret"])]
    assert r["index"][0, :4].tolist() == ints(g["out_index"]) and (r["index"][0, 4:] == -1).all()
    assert r["tokens"][0, :4].tolist() == ints(g["out_tokens"])
    assert r["parent"][0, :4].tolist() == ints(g["out_parent"])
    r = oracle.prune_select(parent, tokens, logq, [7], ints(g["chk_depth"]), _fix(g, "chk_log_tau8_b"),
                            ints(g["chk_keep"]), ints(g["chk_ret"]))
    assert r["stage"].tolist() == [int(g["stage_b"])] and r["n_ret"].tolist() == [int(g["n_ret_b"])]
    assert r["index"][0, :2].tolist() == ints(g["out_index_b"]) and r["parent"][0, :2].tolist() == ints(g["out_parent_b"])
    r = oracle.prune_select(parent, tokens, logq, [7], ints(g["chk_depth"]), _fix(g, "chk_log_tau8_c"),
                            ints(g["chk_keep"]), ints(g["chk_ret"]))
    assert r["stage"].tolist() == [int(g["stage_c"])] and r["n_nodes"].tolist() == [7] and r["n_ret"].tolist() == [0]
    assert r["parent"][0].tolist() == ints(g["parent"]) and r["index"][0].tolist() == list(range(7))


def _random_tree(rng, K, n):
    parent = np.full(K, -1, np.int32)
    for i in range(1, n):
        parent[i] = rng.integers(0, i)
    return parent


def test_selection_against_a_sort_and_closed_under_parents():
    rng = np.random.default_rng(8)
    B, K = 16, 64
    n_nodes = rng.integers(1, K + 1, B).astype(np.int32)
    parent = np.stack([_random_tree(rng, K, n_nodes[b]) for b in range(B)])
    tokens = rng.integers(0, 1000, (B, K)).astype(np.int32)
    logq = -np.round(rng.random((B, K)) * 16).astype(np.float32) / 4          # exact sums, many ties
    chk_depth, chk_keep, chk_ret = [1, 2, 4], [8, 24, 40], [52, 36, 20]
    for log_tau in ([-0.5, -1.0, -2.0], [-9.0, -9.0, -1.0], [-99.0, -99.0, -99.0], [0.0, 0.0, 0.0]):
        r = oracle.prune_select(parent, tokens, logq, n_nodes, chk_depth, log_tau, chk_keep, chk_ret)
        assert (r["status"] == 0).all()
        for b in range(B):
            n = int(n_nodes[b])
            S, dp = np.zeros(n, np.float32), np.zeros(n, np.int64)
            for i in range(1, n):
                S[i] = np.float32(S[parent[b, i]] + logq[b, i])
                dp[i] = dp[parent[b, i]] + 1
            stage = 3
            for c in range(3):
                at = S[dp == chk_depth[c]]
                if at.size == 0 or not (at.max() > np.float32(log_tau[c])):
                    stage = c
                    break
            assert r["stage"][b] == stage
            # a closed gate ends the tree at its depth: deeper nodes are no candidates (Sec. 3.1; Alg. 2)
            cand = [i for i in range(n) if stage == 3 or dp[i] <= chk_depth[stage]]
            keep = n if stage == 3 else min(chk_keep[stage], len(cand))
            order = sorted(cand, key=lambda i: (-S[i], i))[:keep]
            kept = sorted(order)
            assert r["n_nodes"][b] == keep and r["index"][b, :keep].tolist() == kept
            assert r["n_ret"][b] == (0 if stage == 3 else chk_ret[stage])
            pos = {old: new for new, old in enumerate(kept)}
            for new, old in enumerate(kept):
                assert r["tokens"][b, new] == tokens[b, old]
                assert r["parent"][b, new] == (-1 if old == 0 else pos[int(parent[b, old])])   # parent kept too
            # what is left is a valid input of the rebuild step
            m = oracle.build_tree_mask(r["parent"][b:b + 1], r["n_nodes"][b:b + 1], [10])
            assert m["status"].tolist() == [0]


def test_chain_closed_form():
    """A chain with constant probability p per step: c_d = p^d, so the gate at depth d closes iff p^d <= tau."""
    K = 12
    parent = np.arange(-1, K - 1, dtype=np.int32)[None]
    tokens = np.arange(K, dtype=np.int32)[None]
    for p, tau, d in ((0.5, 0.2, 2), (0.5, 0.3, 2), (0.9, 0.5, 6), (0.9, 0.55, 6), (0.25, 0.25, 1)):
        logq = np.full((1, K), math.log(p), np.float32)
        r = oracle.prune_select(parent, tokens, logq, [K], [d], [math.log(tau)], [3], [9])
        S_d = np.float32(0)
        for _ in range(d):
            S_d = np.float32(S_d + np.float32(math.log(p)))
        closed = not (S_d > np.float32(math.log(tau)))
        assert closed == (p ** d <= tau * (1 + 1e-6))                     # the fp32 gate agrees with the real one here
        assert r["stage"].tolist() == [0 if closed else 1]
        kept = min(3, d + 1)                                              # the pruned chain has d + 1 nodes left
        assert r["n_nodes"].tolist() == [kept if closed else K]
        if closed:
            assert r["index"][0, :kept].tolist() == list(range(kept))     # the best-scoring nodes of a chain are its top


def test_nodes_below_the_closed_checkpoint_are_not_candidates():
    """Sec. 3.1: a closed gate prunes the draft tree at its checkpoint and nothing deeper is expanded (Alg. 2
    prunes at the stage's depth, then keeps the best K_draft of what is left).  On a finished static tree
    (App. E) a confident chain below the checkpoint must therefore not displace a shallow sibling."""
    #        0
    #      /   \
    #     1     2        depth 1: scores -1/8 and -3
    #     |
    #     3              depth 2: -2/8
    #     |
    #     4              depth 3: -3/8
    parent = np.array([[-1, 0, 0, 1, 3]], np.int32)
    tokens = np.array([[9, 10, 20, 11, 12]], np.int32)
    logq = np.array([[0, -0.125, -3.0, -0.125, -0.125]], np.float32)
    # the gate at depth 1 is closed (-1/8 > 0 is false): stage 0 keeps 3 of the nodes of depth <= 1
    r = oracle.prune_select(parent, tokens, logq, [5], [1, 2], [0.0, -9.0], [3, 4], [2, 1])
    assert r["stage"].tolist() == [0] and r["n_nodes"].tolist() == [3] and r["n_ret"].tolist() == [2]
    assert r["index"][0, :3].tolist() == [0, 1, 2]            # not {0, 1, 3}: node 3 scores higher than node 2 but is deeper
    assert r["parent"][0, :3].tolist() == [-1, 0, 0] and r["tokens"][0, :3].tolist() == [9, 10, 20]
    # fewer candidates than the stage would keep: all of them stay
    r = oracle.prune_select(parent, tokens, logq, [5], [1, 2], [0.0, -9.0], [4, 4], [2, 1])
    assert r["n_nodes"].tolist() == [3] and r["index"][0, :3].tolist() == [0, 1, 2]
    # the gate at depth 2 closes instead (depth 1 open): candidates are depths 0..2, node 4 stays out
    r = oracle.prune_select(parent, tokens, logq, [5], [1, 2], [-1.0, -0.125], [3, 4], [2, 1])
    assert r["stage"].tolist() == [1] and r["index"][0, :4].tolist() == [0, 1, 2, 3] and r["n_nodes"].tolist() == [4]
    # every gate open: the whole tree stays
    r = oracle.prune_select(parent, tokens, logq, [5], [1, 2], [-1.0, -1.0], [3, 4], [2, 1])
    assert r["stage"].tolist() == [2] and r["n_nodes"].tolist() == [5]


def test_budget_identity_with_the_paper_s_stages():
    """Retained + retrieved = the 60-node verification budget at every stage (Sec. 3.2)."""
    rng = np.random.default_rng(1)
    K = 60
    # a top-10 draft tree: ten children per expanded node, so that every stage has enough candidates
    parent = np.array([[-1] + [(i - 1) // 10 for i in range(1, K)]], np.int32)
    logq = -rng.random((1, K)).astype(np.float32)
    for stage, (keep, ret) in enumerate(((8, 52), (24, 36), (40, 20))):
        log_tau = [-99.0] * 3
        log_tau[stage] = 0.0                                               # closes exactly this gate
        r = oracle.prune_select(parent, np.zeros((1, K), np.int32), logq, [K], [1, 2, 3], log_tau,
                                [8, 24, 40], [52, 36, 20])
        assert r["stage"].tolist() == [stage]
        assert int(r["n_nodes"][0]) + int(r["n_ret"][0]) == keep + ret == 60


def test_gates_are_monotone_in_the_thresholds():
    rng = np.random.default_rng(4)
    K = 40
    parent = _random_tree(rng, K, K)[None]
    logq = -rng.random((1, K)).astype(np.float32)
    prev = None
    for t in np.linspace(-6.0, 0.0, 25):
        r = oracle.prune_select(parent, np.zeros((1, K), np.int32), logq, [K], [1, 2, 3], [t, t, t],
                                [8, 24, 32], [1, 1, 1])
        if prev is not None:
            assert r["stage"][0] <= prev                                   # a stricter threshold never prunes later
        prev = int(r["stage"][0])


def test_bad_trees_and_positive_scores():
    parent = np.array([[-1, 0, 3, 1], [-1, 0, 1, 2]], np.int32)           # node 2's parent has a larger index
    logq = np.array([[0, -1, -1, -1], [0, -5, 4, -1]], np.float32)        # positive log q lifts node 2 above its parent
    # (checkpoint at depth 2, so that node 2 is a candidate: the best two of {0, 1, 2} are 0 and 2)
    r = oracle.prune_select(parent, np.zeros((2, 4), np.int32), logq, [4, 4], [2], [0.0], [2], [7])
    assert r["status"].tolist() == [oracle.ST_BAD_TREE, oracle.ST_BAD_TREE]
    assert r["n_nodes"].tolist() == [0, 0] and r["stage"].tolist() == [-1, -1] and (r["index"] == -1).all()
