"""GPU parity: graft_retrieve vs the CPU oracle, bit-exact (runs on the MI355X only)."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2605_20104_amd as graft
from gpu_util import assert_same, dev, host_dict

pytestmark = pytest.mark.gpu
KEYS = ("chain_tok", "chain_len", "chain_pos", "chain_match", "n_hits", "status")


def both(ctx, ctx_len, n_min, n_max, C, m, tail=None, tail_len=None):
    ref = oracle.retrieve(ctx, ctx_len, n_min, n_max, C, m, tail, tail_len)
    out = graft.graft_retrieve(dev(ctx), dev(ctx_len), n_min, n_max, C, m, dev(tail), dev(tail_len))
    return host_dict(out), ref


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_workloads(name):
    w = inputs.get_workload(name)
    s = inputs.make_step_inputs(w)
    gpu, ref = both(s["ctx"], s["ctx_len"], w.n_min, w.n_max, w.C, w.m, s["tail"], s["tail_len"])
    assert_same(gpu, ref, KEYS)
    for b in range(w.B):                      # and they are the planted continuations
        assert gpu["chain_pos"][b].tolist() == s["planted_pos"][b][:w.C]


@pytest.mark.parametrize("seed", range(6))
def test_tiny_alphabet_many_overlaps(seed):
    rng = np.random.default_rng(seed)
    B, L_max = 5, int(rng.integers(40, 3000))
    vocab = int(rng.integers(2, 5))
    ctx = rng.integers(0, vocab, size=(B, L_max)).astype(np.int32)
    ctx_len = rng.integers(0, L_max + 1, size=B).astype(np.int32)
    ctx_len[0], ctx_len[1], ctx_len[2] = L_max, 0, 1
    tail = rng.integers(0, vocab, size=(B, 6)).astype(np.int32)
    tail_len = rng.integers(0, 7, size=B).astype(np.int32)
    n_min, n_max = int(rng.integers(1, 4)), int(rng.integers(4, 33))
    C, m = int(rng.integers(1, 9)), int(rng.integers(1, 20))
    use_tail = seed % 2 == 0
    gpu, ref = both(ctx, ctx_len, n_min, n_max, C, m, tail if use_tail else None,
                    tail_len if use_tail else None)
    assert_same(gpu, ref, KEYS)


def test_periodic_long_buffer_and_limits():
    ctx = np.full((2, 70000), 7, np.int32)            # every position is a hit; > one scan sweep
    ctx[1, ::3] = 8
    gpu, ref = both(ctx, [70000, 69999], 1, graft.GRAFT_MAX_NGRAM, graft.GRAFT_MAX_CHAINS, 5)
    assert_same(gpu, ref, KEYS)
    assert gpu["n_hits"][0] == 69999


def test_long_tail_and_query_in_every_place():
    """The query can lie in the tail alone, across the end of the context and the tail, or in the context
    beyond the first chunks; tails longer than a workgroup has threads are read from memory."""
    rng = np.random.default_rng(11)
    B, L_max, tail_max = 4, 40000, 1100
    ctx = rng.integers(0, 6, size=(B, L_max)).astype(np.int32)
    tail = rng.integers(0, 6, size=(B, tail_max)).astype(np.int32)
    ctx_len = np.array([40000, 33000, 16385, 5], np.int32)
    tail_len = np.array([1100, 3, 1060, 0], np.int32)
    gpu, ref = both(ctx, ctx_len, 2, 32, 8, 7, tail, tail_len)
    assert_same(gpu, ref, KEYS)
    assert gpu["status"].tolist() == [0, 0, 0, 0] and gpu["n_hits"][0] > 0


def test_no_hits_and_bad_lengths():
    ctx = np.arange(500, dtype=np.int32).reshape(1, 500).repeat(3, 0)
    gpu, ref = both(ctx, [500, 501, -1], 1, 4, 2, 4)
    assert_same(gpu, ref, KEYS)
    assert gpu["status"].tolist() == [0, graft.GRAFT_STATUS_BAD_LENGTH, graft.GRAFT_STATUS_BAD_LENGTH]
    assert (gpu["chain_tok"] == -1).all()


def test_outputs_fully_overwritten():
    """Stale output buffers must not leak through: run on dirty preallocated outputs."""
    w = inputs.get_workload("c2")
    s = inputs.make_step_inputs(w)
    ref = oracle.retrieve(s["ctx"], s["ctx_len"], w.n_min, w.n_max, 8, 12, s["tail"], s["tail_len"])
    out = {k: torch.full(tuple(ref[k].shape), 12345, dtype=torch.int32, device="cuda") for k in KEYS}
    graft.graft_retrieve(dev(s["ctx"]), dev(s["ctx_len"]), w.n_min, w.n_max, 8, 12, dev(s["tail"]),
                         dev(s["tail_len"]), out=out)
    assert_same(host_dict(out), ref, KEYS)
