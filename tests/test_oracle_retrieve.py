"""Pins for the oracle's suffix n-gram retrieval (no GPU).

The oracle is the brute-force scan written in C; these tests pin it to things
other than itself: a hand-worked fixture, an independent pure-Python
enumeration using slice comparison, the planted-span closed form of the
workload generators, and structural invariants.
"""
import numpy as np
import pytest

import inputs
import oracle
from _golden import groups, ints, read_fixture


def brute_force(ctx, L, tail, n_min, n_max):
    """All hits as (match_len, e), best first.  Independent formulation: string slices."""
    ctx = [int(t) for t in ctx[:L]]
    q = ctx + [int(t) for t in tail]
    hits = []
    for e in range(1, L):
        best = 0
        for l in range(1, min(n_max, e) + 1):
            if ctx[e - l:e] == q[len(q) - l:]:
                best = l            # matches are suffix-nested, so the last success is the longest
        if best >= n_min:
            hits.append((best, e))
    hits.sort(reverse=True)
    return hits


def test_golden_small():
    fx = read_fixture("retrieve_small.txt")
    ctx = np.array([ints(fx["ctx"])], np.int32)
    r = oracle.retrieve(ctx, [ctx.shape[1]], n_min=1, n_max=3, C=4, m=3)
    assert r["n_hits"][0] == int(fx["n_hits"])
    assert r["chain_pos"][0].tolist() == ints(fx["chain_pos"])
    assert r["chain_match"][0].tolist() == ints(fx["chain_match"])
    assert r["chain_len"][0].tolist() == ints(fx["chain_len"])
    assert r["chain_tok"][0].tolist() == groups(fx["chain_tok"])


@pytest.mark.parametrize("seed", range(12))
def test_brute_force_tiny_alphabet(seed):
    rng = np.random.default_rng(seed)
    B, L_max = 3, 64
    vocab = int(rng.integers(2, 5))
    ctx = rng.integers(0, vocab, size=(B, L_max)).astype(np.int32)
    ctx_len = rng.integers(0, L_max + 1, size=B).astype(np.int32)
    ctx_len[0] = L_max
    use_tail = seed % 2 == 1
    tail_max = 5
    tail = rng.integers(0, vocab, size=(B, tail_max)).astype(np.int32)
    tail_len = rng.integers(0, tail_max + 1, size=B).astype(np.int32)
    n_min, n_max = int(rng.integers(1, 4)), int(rng.integers(4, 9))
    C, m = L_max, 6          # C = L: every hit comes back, so the full ranking is compared
    r = oracle.retrieve(ctx, ctx_len, n_min, n_max, C, m,
                        tail if use_tail else None, tail_len if use_tail else None)
    for b in range(B):
        L = int(ctx_len[b])
        t = tail[b, :tail_len[b]] if use_tail else []
        hits = brute_force(ctx[b], L, t, n_min, n_max)
        assert r["n_hits"][b] == len(hits)
        for c in range(C):
            if c < len(hits):
                l, e = hits[c]
                assert (r["chain_match"][b, c], r["chain_pos"][b, c]) == (l, e)
                cl = min(m, L - e)
                assert r["chain_len"][b, c] == cl
                assert r["chain_tok"][b, c, :cl].tolist() == ctx[b, e:e + cl].tolist()
                assert (r["chain_tok"][b, c, cl:] == -1).all()
            else:
                assert r["chain_len"][b, c] == 0 and r["chain_pos"][b, c] == -1
                assert r["chain_match"][b, c] == 0 and (r["chain_tok"][b, c] == -1).all()


def test_top_c_is_prefix_of_full_ranking():
    rng = np.random.default_rng(5)
    ctx = rng.integers(0, 3, size=(1, 200)).astype(np.int32)
    full = oracle.retrieve(ctx, [200], 2, 6, 200, 4)
    top = oracle.retrieve(ctx, [200], 2, 6, 3, 4)
    assert top["n_hits"][0] == full["n_hits"][0] > 3
    assert top["chain_pos"][0].tolist() == full["chain_pos"][0, :3].tolist()
    assert top["chain_tok"][0].tolist() == full["chain_tok"][0, :3].tolist()


def test_planted_closed_form_c1():
    """Tiny config: one 4-gram planted three times + the query itself => exactly 3 hits."""
    w = inputs.get_workload("c1")
    s = inputs.make_step_inputs(w)
    r = oracle.retrieve(s["ctx"], s["ctx_len"], w.n_min, w.n_max, 3, w.m, s["tail"], s["tail_len"])
    assert r["n_hits"][0] == 3
    assert r["chain_pos"][0].tolist() == s["planted_pos"][0]          # most recent first
    assert r["chain_match"][0].tolist() == [4, 4, 4]
    assert r["chain_tok"][0].tolist() == s["planted_tok"][0]
    firsts = {c[0] for c in s["planted_tok"][0]}
    assert len(firsts) == 3                                            # distinct continuations


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_planted_closed_form_workloads(name):
    """The generator plants the query n-gram at known places: those must be the top hits."""
    w = inputs.get_workload(name)
    s = inputs.make_step_inputs(w)
    r = oracle.retrieve(s["ctx"], s["ctx_len"], w.n_min, w.n_max, w.C, w.m, s["tail"], s["tail_len"])
    for b in range(w.B):
        assert r["chain_pos"][b].tolist() == s["planted_pos"][b][:w.C]
        assert (r["chain_match"][b] == w.n_max).all()
        assert r["chain_tok"][b].tolist() == s["planted_tok"][b][:w.C]
        assert r["n_hits"][b] >= len(s["planted_pos"][b])
        for c, slot in enumerate(s["ret_slots"][b]):
            assert s["tokens"][b, slot:slot + w.m].tolist() == r["chain_tok"][b, c].tolist()


def test_invariants_and_edges():
    rng = np.random.default_rng(11)
    ctx = rng.integers(0, 6, size=(4, 300)).astype(np.int32)
    ctx_len = np.array([300, 1, 0, 17], np.int32)
    n_min, n_max, C, m = 2, 5, 8, 7
    r = oracle.retrieve(ctx, ctx_len, n_min, n_max, C, m)
    assert r["n_hits"][1] == 0 and r["n_hits"][2] == 0
    for b in range(4):
        L = int(ctx_len[b])
        keys = []
        for c in range(C):
            e, l = int(r["chain_pos"][b, c]), int(r["chain_match"][b, c])
            if e < 0:
                continue
            assert 1 <= e <= L - 1 and n_min <= l <= min(n_max, e)
            assert ctx[b, e - l:e].tolist() == ctx[b, L - l:L].tolist()
            if l < min(n_max, e):                                   # l is maximal
                assert ctx[b, e - l - 1] != ctx[b, L - l - 1]
            keys.append((l, e))
        assert keys == sorted(keys, reverse=True) and len(set(keys)) == len(keys)


def test_no_hit_and_end_of_buffer_truncation():
    ctx = np.arange(100, dtype=np.int32)[None, :].copy()              # all distinct: no hit
    r = oracle.retrieve(ctx, [100], 1, 4, 2, 4)
    assert r["n_hits"][0] == 0 and (r["chain_tok"] == -1).all() and (r["chain_pos"] == -1).all()
    ctx = np.array([[7, 8, 9, 1, 2, 7, 8]], np.int32)                  # match at e=2, then 5 tokens left
    r = oracle.retrieve(ctx, [7], 2, 2, 1, 8)
    assert r["chain_pos"][0, 0] == 2 and r["chain_len"][0, 0] == 5
    assert r["chain_tok"][0, 0].tolist() == [9, 1, 2, 7, 8, -1, -1, -1]
    ctx = np.array([[1, 2, 3, 1, 2]], np.int32)                        # continuation cut by the end
    r = oracle.retrieve(ctx, [5], 2, 2, 1, 4)
    assert r["chain_pos"][0, 0] == 2 and r["chain_len"][0, 0] == 3


def test_periodic_text_overlapping_matches():
    ctx = np.array([[4] * 10], np.int32)                               # aaaa...: every e matches
    r = oracle.retrieve(ctx, [10], 1, 3, 10, 2)
    assert r["n_hits"][0] == 9
    # l = min(3, e): e=9..3 have l=3, then e=2 (l=2), e=1 (l=1)
    assert r["chain_pos"][0].tolist() == [9, 8, 7, 6, 5, 4, 3, 2, 1, -1]
    assert r["chain_match"][0].tolist() == [3] * 7 + [2, 1, 0]


def test_tail_extends_query():
    # context ... 5 6 | tail 7 : query tail "6 7" only occurs where ctx has 6 7
    ctx = np.array([[5, 6, 7, 9, 9, 5, 6]], np.int32)
    r = oracle.retrieve(ctx, [7], 2, 3, 2, 2, tail=np.array([[7]], np.int32), tail_len=[1])
    assert r["n_hits"][0] == 1 and r["chain_pos"][0, 0] == 3 and r["chain_match"][0, 0] == 3
    assert r["chain_tok"][0, 0].tolist() == [9, 9]


def test_bad_lengths_flagged():
    ctx = np.zeros((2, 8), np.int32)
    r = oracle.retrieve(ctx, [9, 8], 1, 2, 1, 2)
    assert r["status"].tolist() == [oracle.ST_BAD_LENGTH, 0]
    assert r["n_hits"][0] == 0 and (r["chain_tok"][0] == -1).all()
