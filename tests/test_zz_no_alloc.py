"""graft_accept_noalloc (the entry point for callers that cannot allocate: its argmax partials live in
a device array of the library itself) against graft_accept with a caller workspace, through the C
ABI: bit-exact on two calls in a row, the second with a smaller input, so that whatever the first
call left in the shared array must not leak into the second."""
import numpy as np
import pytest
import torch

import paper_2605_20104_amd as graft
from gpu_util import dev

pytestmark = pytest.mark.gpu

KEYS = ("accept_len", "best_node", "path", "out_tokens", "status")


def _case(rng, B, K, V, depth_cap):
    parent = np.full((B, K), -1, np.int32)
    n_nodes = rng.integers(max(1, K // 2), K + 1, B).astype(np.int32)
    for b in range(B):
        for i in range(1, K):
            parent[b, i] = rng.integers(0, i)
    tokens = rng.integers(0, V, (B, K)).astype(np.int32)
    logits = rng.standard_normal((B, K, V)).astype(np.float32)
    for b in range(B):                          # let the target agree with many nodes so that paths get accepted
        for i in range(1, int(n_nodes[b])):
            if rng.random() < 0.7:
                logits[b, parent[b, i], tokens[b, i]] = 9.0
    logits[0, 0, :] = 1.5                       # a row of ties: the first maximum wins
    return parent, tokens, n_nodes, logits


def _outputs(B, depth_cap):
    i32 = lambda *s: torch.full(s, -7, dtype=torch.int32, device="cuda")
    return {"accept_len": i32(B), "best_node": i32(B), "path": i32(B, depth_cap + 1),
            "out_tokens": i32(B, depth_cap + 1), "status": i32(B)}


def _compare(rng, B, K, V, depth_cap):
    parent, tokens, n_nodes, logits = _case(rng, B, K, V, depth_cap)
    d = [dev(parent), dev(tokens), dev(n_nodes)]
    lg = dev(logits, "f32")
    ref = graft.graft_accept(*d, depth_cap, logits=lg)
    out = _outputs(B, depth_cap)
    ids = torch.full((B, K), -7, dtype=torch.int32, device="cuda")
    before = torch.cuda.memory_allocated()
    graft.graft_accept_noalloc(*d, depth_cap, out, ids, logits=lg)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for k in KEYS:
        assert torch.equal(out[k], ref[k]), k
    assert torch.equal(ids, ref["target_ids"])
    assert int(ref["accept_len"].max()) >= 1
    # target_ids mode (no scratch at all) through the same entry point
    out2 = _outputs(B, depth_cap)
    graft.graft_accept_noalloc(*d, depth_cap, out2, ref["target_ids"])
    torch.cuda.synchronize()
    for k in KEYS:
        assert torch.equal(out2[k], ref[k]), k


def test_noalloc_equals_graft_accept_twice_in_a_row():
    rng = np.random.default_rng(77)
    _compare(rng, 6, 96, 5003, 24)       # 576 logits rows, vocabulary not a multiple of 4
    _compare(rng, 2, 17, 1000, 8)        # smaller: fewer rows, fewer nodes, shorter rows


def test_noalloc_rejects_more_rows_than_its_scratch_holds():
    B, K = 65, 128                        # 8320 rows > GRAFT_NOALLOC_MAX_ROWS
    assert B * K > graft.GRAFT_NOALLOC_MAX_ROWS
    z = torch.zeros((B, K), dtype=torch.int32, device="cuda")
    n = torch.ones(B, dtype=torch.int32, device="cuda")
    lg = torch.zeros((B, K, 4), dtype=torch.float32, device="cuda")
    with pytest.raises(graft.GraftError) as e:
        graft.graft_accept_noalloc(z, z, n, 4, _outputs(B, 4), z.clone(), logits=lg)
    assert e.value.code == graft.GRAFT_ERR_WORKSPACE
