"""GPU parity of graft_matrix_retrieve / graft_matrix_update against the CPU oracle (bit-exact)."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2605_20104_amd as graft
from gpu_util import dev, host
from inputs import templates

pytestmark = pytest.mark.gpu


def _retrieve_both(M, tp, tr, n_ret, tokens, parent, n_nodes):
    ref = oracle.matrix_retrieve(M, tp, tr, n_ret, tokens, parent, n_nodes)
    t, p, n = dev(tokens), dev(parent), dev(n_nodes)
    st = graft.graft_matrix_retrieve(dev(M), dev(tp), dev(tr), dev(n_ret), t, p, n)
    torch.cuda.synchronize()
    got = {"tokens": host(t), "parent": host(p), "n_nodes": host(n), "status": host(st)}
    for key in ("tokens", "parent", "n_nodes", "status"):
        assert (got[key] == ref[key]).all(), (key, got[key], ref[key])
    return ref


@pytest.mark.parametrize("V,k,seed", [(1000, 8, 0), (128256, 8, 1), (151936, 16, 2), (50, 1, 3)])
def test_retrieve_envelope_stages(V, k, seed):
    rng = np.random.default_rng(seed)
    M = rng.integers(0, V, (V, k), dtype=np.int32)
    M[rng.random((V, k)) < 0.05] = -1                                    # some empty entries
    tp, tr, td, sizes = templates.retrieval_envelope()
    if k < 8:
        tp, tr = np.arange(-1, 8, dtype=np.int32), np.zeros(9, np.int32)   # a chain fits any k
        sizes = {"d5": 3, "d1": 5, "d0": 7, "full": 9}
    B, K = 6, 128
    tokens = rng.integers(0, V, (B, K)).astype(np.int32)
    parent = np.full((B, K), -1, np.int32)
    n_draft = np.array([40, 24, 8, 1, 48, 1], np.int32)
    for b in range(B):
        for i in range(1, n_draft[b]):
            parent[b, i] = rng.integers(0, i)
    n_ret = np.array([sizes["d5"], sizes["d1"], sizes["d0"], sizes["full"], 0, 1], np.int32)
    tokens[5, 0] = V + 3                                                 # a root outside the vocabulary
    ref = _retrieve_both(M, tp, tr, n_ret, tokens, parent, n_draft)
    assert ref["status"].tolist() == [0] * B
    assert (ref["tokens"][5, 1:2] == -1).all()


def test_retrieve_error_paths_leave_the_tree_alone():
    M = np.arange(40, dtype=np.int32).reshape(10, 4) % 10
    tokens = np.arange(24, dtype=np.int32).reshape(3, 8) % 10
    parent = np.full((3, 8), -1, np.int32)
    ref = _retrieve_both(M, [-1, 0, 1], [0, 0, 0], np.array([3, 4, 2], np.int32), tokens, parent,
                         np.array([6, 1, 0], np.int32))
    assert ref["status"].tolist() == [graft.GRAFT_STATUS_BAD_LENGTH] * 3
    for tp, tr in (([-1, 1, 0], [0, 0, 0]), ([-1, 0, 1], [0, 4, 0]), ([-2, 0, 1], [0, 0, 0])):
        ref = _retrieve_both(M, tp, tr, np.array([3, 1, 0], np.int32), tokens, parent, np.array([1, 1, 2], np.int32))
        assert ref["status"][0] == graft.GRAFT_STATUS_BAD_TREE


def _update_both(M0, tokens, n_nodes, logits):
    ref = oracle.matrix_update(M0, tokens, n_nodes, logits)
    M = dev(M0)
    tids = graft.graft_matrix_update(dev(tokens), dev(n_nodes), dev(logits, "f32"), M)
    torch.cuda.synchronize()
    assert (host(tids) == ref["target_ids"]).all()
    assert (host(M) == ref["M"]).all()
    return ref


@pytest.mark.parametrize("B,K,V,k,seed", [(1, 16, 1000, 8, 0), (2, 12, 999, 8, 1), (3, 7, 4099, 16, 2),
                                          (2, 5, 37, 4, 3), (1, 3, 64, 1, 4), (2, 9, 16384, 3, 5)])
def test_update_small(B, K, V, k, seed):
    rng = np.random.default_rng(seed)
    logits = rng.standard_normal((B, K, V)).astype(np.float32)
    logits[0, 0, : V // 2] = np.round(logits[0, 0, : V // 2] * 2) / 2     # exact ties, also +-0
    logits[0, 0, 3] = -0.0
    tokens = rng.integers(0, min(V, 9), (B, K)).astype(np.int32)          # repeated tokens
    tokens[-1, -1] = V + 1
    tokens[0, 1] = -5
    n_nodes = rng.integers(1, K + 1, B).astype(np.int32)
    n_nodes[0] = K
    M0 = rng.integers(0, V, (V, k), dtype=np.int32)
    _update_both(M0, tokens, n_nodes, logits)


def test_update_ties_everywhere():
    """A constant row: the k smallest ids, in order; rows of two values: ids of the larger value first."""
    B, K, V, k = 1, 4, 5000, 8
    logits = np.zeros((B, K, V), np.float32)
    logits[0, 1] = -3.5
    logits[0, 2, ::7] = 1.0
    logits[0, 3, -3:] = 2.0
    tokens = np.array([[10, 11, 12, 13]], np.int32)
    ref = _update_both(np.full((V, k), -1, np.int32), tokens, [4], logits)
    assert ref["M"][10].tolist() == list(range(8)) and ref["M"][11].tolist() == list(range(8))
    assert ref["M"][12].tolist() == [0, 7, 14, 21, 28, 35, 42, 49]
    assert ref["M"][13].tolist() == [4997, 4998, 4999, 0, 1, 2, 3, 4]


@pytest.mark.parametrize("wl", ["c1", "c2", "c3", "c4"])
def test_update_at_workload_size_and_accept_takes_its_ids(wl):
    w = inputs.get_workload(wl)
    s = inputs.make_step_inputs(w, with_logits=True)
    rng = np.random.default_rng(9)
    M0 = rng.integers(0, w.vocab, (w.vocab, 8), dtype=np.int32)
    ref = _update_both(M0, s["tokens"], s["n_nodes"], s["logits"])
    assert (ref["target_ids"] == s["target_ids"]).all()                   # the planted greedy tokens
    # acceptance from these ids = acceptance from the logits
    a1 = oracle.accept(s["parent"], s["tokens"], s["n_nodes"], 16, target_ids=ref["target_ids"])
    a2 = oracle.accept(s["parent"], s["tokens"], s["n_nodes"], 16, logits=s["logits"])
    assert a1["out_tokens"].tolist() == a2["out_tokens"].tolist()


def test_update_then_retrieve_round_trip():
    V, k = 2048, 8
    rng = np.random.default_rng(4)
    logits = rng.standard_normal((1, 1, V)).astype(np.float32)
    M = dev(np.full((V, k), -1, np.int32))
    graft.graft_matrix_update(dev([[77]]), dev([1]), dev(logits, "f32"), M)
    tp, tr = np.full(8, -1, np.int32), np.arange(8, dtype=np.int32)
    tokens = np.zeros((1, 9), np.int32)
    tokens[0, 0] = 77
    t, p, n = dev(tokens), dev(np.full((1, 9), -1, np.int32)), dev([1])
    graft.graft_matrix_retrieve(M, dev(tp), dev(tr), dev([8]), t, p, n)
    torch.cuda.synchronize()
    assert host(t)[0, 1:].tolist() == np.argsort(-logits[0, 0], kind="stable")[:8].tolist()


def test_update_from_a_prefill():
    """App. A Alg. 1 "Update M with prefill logits": a prompt of 4096 positions handed over as 32 rows of 128
    nodes; tokens repeat heavily (Zipf), the last occurrence of a token decides its row."""
    rng = np.random.default_rng(12)
    V, k, L = 4096, 8, 4096
    ranks = np.minimum(rng.zipf(1.3, L), V) - 1
    tokens = rng.permutation(V)[ranks].astype(np.int32).reshape(32, 128)
    logits = rng.standard_normal((32, 128, V)).astype(np.float32)
    n_nodes = np.full(32, 128, np.int32)
    n_nodes[-1] = 77                                                      # a ragged last row
    ref = _update_both(np.full((V, k), -1, np.int32), tokens, n_nodes, logits)
    touched = {int(t) for b in range(32) for t in tokens[b, :n_nodes[b]]}
    assert len(touched) < L // 2                                          # the repetition is real
    assert ((ref["M"][:, 0] >= 0) == np.isin(np.arange(V), list(touched))).all()
