"""Pins for the oracle's greedy acceptance walk (no GPU)."""
import itertools

import numpy as np
import pytest

import inputs
import oracle
from _golden import ints, read_fixture


def greedy_decode(ctx_tail, vocab, seed, n):
    """Plain autoregressive greedy decoding with the toy target."""
    seq = [int(t) for t in ctx_tail]
    out = []
    for _ in range(n):
        t = inputs.toy_target(seq[-3:], vocab, seed)
        out.append(t)
        seq.append(t)
    return out


def test_golden_small():
    fx = read_fixture("accept_small.txt")
    parent = np.array([ints(fx["parent"])], np.int32)
    tokens = np.array([ints(fx["tokens"])], np.int32)
    target = np.array([ints(fx["target"])], np.int32)
    r = oracle.accept(parent, tokens, [parent.shape[1]], depth_cap=5, target_ids=target)
    assert r["accept_len"][0] == int(fx["accept_len"]) and r["best_node"][0] == int(fx["best_node"])
    p, t = ints(fx["path"]), ints(fx["out_tokens"])
    assert r["path"][0, :len(p)].tolist() == p and (r["path"][0, len(p):] == -1).all()
    assert r["out_tokens"][0, :len(t)].tolist() == t and (r["out_tokens"][0, len(t):] == -1).all()


def random_tree_with_tokens(rng, K, vocab, ctx_tail4, seed, p_right):
    parent = inputs.random_recursive_tree(rng, K, 12)
    tokens = np.zeros(K, np.int32)
    tokens[0] = ctx_tail4[-1]
    for i in range(1, K):
        path = []
        j = int(parent[i])
        while j != -1:
            path.append(int(tokens[j]))
            j = int(parent[j])
        seq = [int(t) for t in ctx_tail4[:3]] + path[::-1]
        right = inputs.toy_target(seq[-3:], vocab, seed)
        tokens[i] = right if rng.random() < p_right else int(rng.integers(0, vocab))
    return parent, tokens


@pytest.mark.parametrize("seed", range(10))
def test_lossless_against_greedy_decoding(seed):
    """App. B.4 (lossless): emitted tokens are a prefix of plain greedy decoding, for any tree."""
    rng = np.random.default_rng(seed)
    vocab, K = 50, int(rng.integers(1, 65))
    ctx_tail4 = rng.integers(0, vocab, size=4)
    parent, tokens = random_tree_with_tokens(rng, K, vocab, ctx_tail4, seed, 0.7)
    target = inputs.toy_target_for_nodes(ctx_tail4[:3], parent, tokens, K, vocab, seed)
    r = oracle.accept(parent[None], tokens[None], [K], depth_cap=K, target_ids=target[None])
    n = int(r["accept_len"][0])
    ref = greedy_decode(ctx_tail4, vocab, seed, n + 1)
    assert r["out_tokens"][0, :n + 1].tolist() == ref
    # and it is the longest: no child of the best node carries the next greedy token's... (maximality)
    best = int(r["best_node"][0])
    kids = [c for c in range(K) if parent[c] == best]
    assert all(tokens[c] != target[best] for c in kids)
    # logits mode gives the same result when the row maximum sits at the target id
    logits = rng.standard_normal((1, K, vocab)).astype(np.float32)
    for i in range(K):
        logits[0, i, target[i]] = 9.0
    r2 = oracle.accept(parent[None], tokens[None], [K], depth_cap=K, logits=logits)
    for k in ("accept_len", "best_node", "path", "out_tokens"):
        assert (r[k] == r2[k]).all()
    assert r2["target_ids"][0].tolist() == target.tolist()


def accepted_by_enumeration(parent, tokens, target, n):
    """Brute force: try every node's root path, keep the deepest fully matching one."""
    best, best_depth = 0, 0
    for i in range(n):
        path, j = [], i
        while j != -1:
            path.append(j)
            j = int(parent[j])
        path = path[::-1]
        if all(tokens[path[k]] == target[path[k - 1]] for k in range(1, len(path))):
            if len(path) - 1 > best_depth:
                best, best_depth = i, len(path) - 1
    return best, best_depth


@pytest.mark.parametrize("seed", range(10))
def test_enumeration_and_monotonicity(seed):
    """Brute force over all paths; App. B.1 Prop. 1 / B.2 Prop. 2: more nodes never accept less."""
    rng = np.random.default_rng(100 + seed)
    K, vocab = int(rng.integers(2, 40)), 3            # tiny vocabulary: many matches and ties
    parent = inputs.random_recursive_tree(rng, K, 10)
    tokens = rng.integers(0, vocab, size=K).astype(np.int32)
    target = rng.integers(0, vocab, size=K).astype(np.int32)
    full = oracle.accept(parent[None], tokens[None], [K], depth_cap=K, target_ids=target[None])
    assert (int(full["best_node"][0]), int(full["accept_len"][0])) == \
        accepted_by_enumeration(parent, tokens, target, K)
    prev = -1
    for n in range(1, K + 1):                         # prefixes of the node list are sub-trees
        r = oracle.accept(parent[None], tokens[None], [n], depth_cap=K, target_ids=target[None])
        assert r["accept_len"][0] >= prev
        prev = int(r["accept_len"][0])
    assert prev == full["accept_len"][0]


def test_first_maximum_and_duplicate_siblings():
    parent = np.array([[-1, 0, 0, 1, 2]], np.int32)
    tokens = np.array([[9, 4, 4, 7, 7]], np.int32)     # duplicate siblings 1 and 2, both match
    logits = np.zeros((1, 5, 10), np.float32)
    logits[0, 0, 4] = logits[0, 0, 6] = 3.0            # tie: first maximum (4) wins
    logits[0, 1, 7] = 1.0
    logits[0, 2, 7] = 1.0
    logits[0, 3, 2] = 1.0
    logits[0, 4, 5] = 1.0
    r = oracle.accept(parent, tokens, [5], depth_cap=4, logits=logits)
    assert r["target_ids"][0].tolist() == [4, 7, 7, 2, 5]
    assert r["accept_len"][0] == 2 and r["best_node"][0] == 3      # deepest, smallest index on ties
    assert r["path"][0].tolist() == [0, 1, 3, -1, -1]
    assert r["out_tokens"][0].tolist() == [4, 7, 2, -1, -1]


def test_root_only_and_bad_tree_and_depth_cap():
    r = oracle.accept(np.array([[-1]], np.int32), np.array([[3]], np.int32), [1], 2,
                      target_ids=np.array([[8]], np.int32))
    assert r["accept_len"][0] == 0 and r["best_node"][0] == 0 and r["out_tokens"][0].tolist() == [8, -1, -1]
    r = oracle.accept(np.array([[-1, 1]], np.int32), np.array([[3, 3]], np.int32), [2], 2,
                      target_ids=np.array([[3, 3]], np.int32))
    assert r["status"][0] == oracle.ST_BAD_TREE and r["best_node"][0] == -1 and r["accept_len"][0] == 0
    parent = np.arange(-1, 5, dtype=np.int32)[None]                      # chain of 6, all matching
    tok = np.array([[0, 1, 2, 3, 4, 5]], np.int32)
    tgt = np.array([[1, 2, 3, 4, 5, 6]], np.int32)
    r = oracle.accept(parent, tok, [6], depth_cap=3, target_ids=tgt)
    assert r["status"][0] == oracle.ST_PATH_OVERFLOW and r["accept_len"][0] == 3
    assert r["out_tokens"][0].tolist() == [1, 2, 3, 4]


def test_toy_loop_is_lossless_end_to_end():
    """50 steps of retrieve -> graft -> mask -> accept reproduce plain greedy decoding (App. B.4)."""
    rng = np.random.default_rng(7)
    vocab, seed, m, C = 12, 3, 4, 2
    ctx = [int(t) for t in rng.integers(0, vocab, size=40)]
    start = len(ctx)
    steps = 50
    emitted = 0
    for _ in range(steps):
        arr = np.array([ctx], np.int32)
        ret = oracle.retrieve(arr, [len(ctx)], 1, 3, C, m)
        # hybrid tree: root + a 3-node random "draft" part + the retrieved chains under the root
        parent, tokens = [-1], [ctx[-1]]
        for _ in range(3):
            parent.append(int(rng.integers(0, len(parent))))
            tokens.append(int(rng.integers(0, vocab)))
        for c in range(C):
            prev = 0
            for j in range(int(ret["chain_len"][0, c])):
                parent.append(prev)
                tokens.append(int(ret["chain_tok"][0, c, j]))
                prev = len(parent) - 1
        K = len(parent)
        P = np.array([parent], np.int32)
        T = np.array([tokens], np.int32)
        mk = oracle.build_tree_mask(P, [K], [len(ctx) - 1])
        assert mk["status"][0] == 0
        tgt = inputs.toy_target_for_nodes(ctx[-4:-1], P[0], T[0], K, vocab, seed)
        acc = oracle.accept(P, T, [K], depth_cap=K, target_ids=tgt[None])
        n = int(acc["accept_len"][0])
        ctx += acc["out_tokens"][0, :n + 1].tolist()
        emitted += n + 1
    ref = greedy_decode(ctx[:start], vocab, seed, emitted)
    assert ctx[start:] == ref
    assert emitted > steps            # retrieval got something accepted along the way
