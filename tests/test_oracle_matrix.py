"""Pins of the oracle's matrix retrieval and matrix refresh (Sec. 3.2, Sec. 3.3, App. A.1)."""
import collections

import numpy as np
import pytest

import inputs
import oracle
from inputs import templates
from _golden import groups, ints, read_fixture


# ---------------------------------------------------------------- templates (input structure)
def test_templates_have_the_paper_s_depth_counts():
    tp, tr, td, sizes = templates.retrieval_envelope()
    paths = templates.rank_paths(tp, tr)
    with open(__import__("os").path.join(__import__("_golden").GOLDEN, "budget_split.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for stage, draft, n_ret, counts in rows:
        want = [int(x) for x in counts.split("+")]
        n = sizes[stage]
        assert n == int(n_ret) == sum(want)
        got = collections.Counter(len(p) for p in paths[:n])
        assert [got[d] for d in range(1, 10)] == want
        if draft != "-":
            assert templates.STAGE_DRAFT_NODES[stage] == int(draft) and int(draft) + n == 60


def test_templates_are_well_formed_and_follow_the_design_principle():
    tp, tr, td, sizes = templates.retrieval_envelope()
    paths = templates.rank_paths(tp, tr)
    assert len(set(paths)) == len(paths) == 80
    for u in range(80):
        assert -1 <= tp[u] < u                                   # parents come first: every prefix is a tree
        assert td[u] == len(paths[u]) == (1 if tp[u] < 0 else td[tp[u]] + 1)
    for stage, n in sizes.items():
        kids = collections.defaultdict(list)
        for p in paths[:n]:
            kids[p[:-1]].append(p[-1])
        for par, ranks in kids.items():
            assert sorted(ranks) == list(range(len(ranks)))      # ranks 0..c-1, no gaps
        # higher-ranked successors receive at least as many children as lower-ranked siblings
        for par, ranks in kids.items():
            n_child = [len(kids.get(par + (r,), [])) for r in range(len(ranks))]
            assert n_child == sorted(n_child, reverse=True)
        assert (0,) * 9 in paths[:n]                             # the greedy chain reaches depth 9
        assert max(len(p) for p in paths[:n]) == 9


# ---------------------------------------------------------------- retrieval from the matrix
def test_hand_worked_lookup():
    g = read_fixture("matrix_small.txt")
    M = np.array(groups(g["M"]), np.int32)
    tokens = np.full((1, 8), -7, np.int32)
    parent = np.full((1, 8), -7, np.int32)
    tokens[0, :2], parent[0, :2] = ints(g["tokens_in"]), ints(g["parent_in"])
    r = oracle.matrix_retrieve(M, ints(g["tpl_parent"]), ints(g["tpl_rank"]), [5], tokens, parent, [2])
    assert r["n_nodes"].tolist() == [7] and r["status"].tolist() == [0]
    assert r["tokens"][0, :7].tolist() == ints(g["tokens_out"])
    assert r["parent"][0, :7].tolist() == ints(g["parent_out"])
    assert r["tokens"][0, 7] == -7 and r["parent"][0, 7] == -7          # nothing past the new end is touched
    tokens[0, 0] = 4
    r = oracle.matrix_retrieve(M, ints(g["tpl_parent"]), ints(g["tpl_rank"]), [5], tokens, parent, [2])
    assert r["tokens"][0, :7].tolist() == ints(g["tokens_out_root4"])
    # a prefix of the template
    r = oracle.matrix_retrieve(M, ints(g["tpl_parent"]), ints(g["tpl_rank"]), [2], tokens, parent, [2])
    assert r["n_nodes"].tolist() == [4] and r["tokens"][0, :4].tolist() == ints(g["tokens_out_root4"])[:4]


def test_chain_template_is_repeated_successor():
    """A template that is one greedy chain walks x -> M[x][0] -> ... : iterate a dict instead."""
    rng = np.random.default_rng(5)
    V, k = 50, 4
    M = rng.integers(0, V, (V, k), dtype=np.int32)
    succ = {x: int(M[x, 0]) for x in range(V)}
    tp, tr = np.arange(-1, 8, dtype=np.int32), np.zeros(9, np.int32)
    for root in range(V):
        tokens = np.zeros((1, 10), np.int32)
        tokens[0, 0] = root
        r = oracle.matrix_retrieve(M, tp, tr, [9], tokens, np.full((1, 10), -1, np.int32), [1])
        want, x = [], root
        for _ in range(9):
            x = succ[x]
            want.append(x)
        assert r["tokens"][0, 1:].tolist() == want
        assert r["parent"][0].tolist() == [-1] + list(range(9))


def test_envelope_fill_equals_enumeration_of_rank_paths():
    """With M[x][r] = f(x, r) for an explicit f, node [r1..rd] must hold f(...f(f(root, r1), r2)..., rd)."""
    V, k = 97, 8
    f = lambda x, r: (x * 31 + r * 7 + 3) % V
    M = np.array([[f(x, r) for r in range(k)] for x in range(V)], np.int32)
    tp, tr, td, sizes = templates.retrieval_envelope()
    paths = templates.rank_paths(tp, tr)
    B, K = 3, 128
    roots, n_draft = [5, 60, 96], [8, 24, 40]
    stages = ["d0", "d1", "d5"]
    tokens = np.zeros((B, K), np.int32)
    parent = np.full((B, K), -1, np.int32)
    for b in range(B):
        tokens[b, 0] = roots[b]
        parent[b, 1:n_draft[b]] = 0
    n_ret = [sizes[s] for s in stages]
    r = oracle.matrix_retrieve(M, tp, tr, n_ret, tokens, parent, n_draft)
    assert r["n_nodes"].tolist() == [60, 60, 60]                         # the verification budget (Sec. 3.2)
    for b in range(B):
        for u in range(n_ret[b]):
            x = roots[b]
            for rk in paths[u]:
                x = f(x, rk)
            assert r["tokens"][b, n_draft[b] + u] == x
            # the merged parent is the merged position of the path without its last rank
            pu = r["parent"][b, n_draft[b] + u]
            assert pu == (0 if len(paths[u]) == 1 else n_draft[b] + paths.index(paths[u][:-1]))
        # the merged tree is a valid input of the rebuild step
        m = oracle.build_tree_mask(r["parent"][b:b + 1], r["n_nodes"][b:b + 1], [100])
        assert m["status"].tolist() == [0]
        assert m["depth"][0, n_draft[b]:60].tolist() == td[:n_ret[b]].tolist()


def test_retrieve_rejects_what_does_not_fit():
    M = np.zeros((4, 2), np.int32)
    tokens, parent = np.zeros((3, 6), np.int32), np.full((3, 6), -1, np.int32)
    r = oracle.matrix_retrieve(M, [-1, 0, 1], [0, 0, 0], [3, 4, 2], tokens, parent, [4, 1, 0])
    assert r["status"].tolist() == [oracle.ST_BAD_LENGTH] * 3            # 4+3 > 6; 4 > N; no root
    assert r["n_nodes"].tolist() == [4, 1, 0] and (r["tokens"] == 0).all()
    # ill-formed templates: a parent that is not an earlier node, a rank outside [0, k)
    tokens = np.zeros((2, 6), np.int32)
    for tp, tr in (([-1, 1, 0], [0, 0, 0]), ([-1, 0, 1], [0, 2, 0]), ([-2, 0, 1], [0, 0, 0])):
        r = oracle.matrix_retrieve(M, tp, tr, [3, 1], tokens, np.full((2, 6), -1, np.int32), [1, 1])
        assert r["status"].tolist() == [oracle.ST_BAD_TREE, oracle.ST_BAD_TREE if tp[0] < -1 else 0]
        assert r["n_nodes"].tolist() == [1, 1 if tp[0] < -1 else 2]


# ---------------------------------------------------------------- refresh of the matrix
def test_hand_worked_refresh():
    g = read_fixture("matrix_small.txt")
    M = np.array(groups(g["M"]), np.int32)
    logits = np.array([[float(x) for x in g["logits%d" % i].split()] for i in range(3)], np.float32)[None]
    r = oracle.matrix_update(M, [ints(g["upd_tokens"])], [3], logits)
    assert r["M"].tolist() == groups(g["M_after"])
    assert r["target_ids"].tolist() == [ints(g["target_ids"])]


def test_refresh_against_a_stable_sort_and_the_acceptance_argmax():
    rng = np.random.default_rng(11)
    B, K, V, k = 2, 12, 300, 8
    logits = np.round(rng.standard_normal((B, K, V)) * 4).astype(np.float32) / 4      # many exact ties
    tokens = rng.permutation(V)[:B * K].reshape(B, K).astype(np.int32)               # all distinct
    n_nodes = np.array([12, 7], np.int32)
    M0 = rng.integers(0, V, (V, k), dtype=np.int32)
    r = oracle.matrix_update(M0, tokens, n_nodes, logits)
    want = M0.copy()
    for b in range(B):
        for i in range(n_nodes[b]):
            want[tokens[b, i]] = np.argsort(-logits[b, i], kind="stable")[:k]
    assert (r["M"] == want).all()
    # first column = the greedy token of the acceptance step
    a = oracle.accept(np.tile(np.arange(-1, K - 1, dtype=np.int32), (B, 1)), tokens, n_nodes, K, logits=logits)
    for b in range(B):
        assert r["target_ids"][b, :n_nodes[b]].tolist() == a["target_ids"][b, :n_nodes[b]].tolist()
        assert (r["target_ids"][b, n_nodes[b]:] == -1).all()


def test_refresh_duplicates_and_out_of_range_tokens():
    rng = np.random.default_rng(3)
    B, K, V, k = 3, 6, 40, 3
    logits = rng.standard_normal((B, K, V)).astype(np.float32)
    tokens = rng.integers(0, 5, (B, K)).astype(np.int32)                 # heavy repetition
    tokens[1, 2], tokens[2, 0] = -1, V                                   # skipped
    n_nodes = np.array([6, 6, 4], np.int32)
    M0 = np.full((V, k), -1, np.int32)
    r = oracle.matrix_update(M0, tokens, n_nodes, logits)
    last = {}
    for b in range(B):
        for i in range(n_nodes[b]):
            if 0 <= tokens[b, i] < V:
                last[int(tokens[b, i])] = (b, i)
    for x in range(V):
        if x in last:
            b, i = last[x]
            assert r["M"][x].tolist() == np.argsort(-logits[b, i], kind="stable")[:k].tolist()
        else:
            assert (r["M"][x] == -1).all()


def test_refresh_then_lookup_round_trip():
    """What the refresh writes for a token is what the next lookup from that token returns."""
    V, k = 64, 8
    rng = np.random.default_rng(2)
    logits = rng.standard_normal((1, 1, V)).astype(np.float32)
    M = oracle.matrix_update(np.full((V, k), -1, np.int32), [[17]], [1], logits)["M"]
    tp, tr = np.full(8, -1, np.int32), np.arange(8, dtype=np.int32)     # eight children of the root, ranks 0..7
    tokens = np.zeros((1, 9), np.int32)
    tokens[0, 0] = 17
    r = oracle.matrix_retrieve(M, tp, tr, [8], tokens, np.full((1, 9), -1, np.int32), [1])
    assert r["tokens"][0, 1:].tolist() == np.argsort(-logits[0, 0], kind="stable")[:8].tolist()
