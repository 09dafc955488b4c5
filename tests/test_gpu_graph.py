"""The whole step can be captured in a HIP graph: replays (with eager work and synchronisations in
between) must reproduce the eager results exactly.  The library launches plain kernels only (no
memset nodes), which is what makes this safe."""
import numpy as np
import pytest
import torch

import inputs
import paper_2605_20104_amd as graft
from gpu_util import dev

pytestmark = pytest.mark.gpu


def _buffers(w, seed):
    s = inputs.make_step_inputs(w, seed=seed, with_logits=True)
    att = inputs.make_attention_inputs(w, seed=seed)
    kind = "f32" if w.dtype == "f32" else "bf16"
    d = {k: dev(s[k]) for k in ("ctx", "ctx_len", "tail", "tail_len", "parent", "tokens", "n_nodes", "prefix_len")}
    d.update(q=dev(att["q"][0], kind), k=dev(att["k_cache"][0], kind), v=dev(att["v_cache"][0], kind),
             table=dev(att["block_table"]), logits=dev(s["logits"], "f32"))
    return s, att, d


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_graph_replays_equal_eager(name):
    w = inputs.get_workload(name)
    s, att, d = _buffers(w, seed=None)
    B, K = w.B, w.K
    cu = "cuda"
    i32 = lambda *shape: torch.empty(shape, dtype=torch.int32, device=cu)
    ret = {"chain_tok": i32(B, w.C, w.m), "chain_len": i32(B, w.C), "chain_pos": i32(B, w.C),
           "chain_match": i32(B, w.C), "n_hits": i32(B), "status": i32(B)}
    mk = {"mask": torch.empty((B, K, 2), dtype=torch.int64, device=cu), "pos": i32(B, K), "depth": i32(B, K),
          "paths": i32(B, K, 17), "status": i32(B)}
    o = torch.empty_like(d["q"])
    ws = torch.empty(max(graft.graft_tree_attn_workspace_bytes(B, K, w.Hq, w.Hkv, w.D, d["table"].shape[1],
                                                               graft.GRAFT_F32 if w.dtype == "f32" else graft.GRAFT_BF16), 256),
                     dtype=torch.uint8, device=cu)
    Mx = torch.full((w.vocab, 8), -1, dtype=torch.int32, device=cu)
    ids = i32(B, K)
    mu_ws = torch.empty(graft.graft_matrix_update_workspace_bytes(B, K, w.vocab, 8), dtype=torch.uint8, device=cu)
    acc = {"accept_len": i32(B), "best_node": i32(B), "path": i32(B, 17), "out_tokens": i32(B, 17), "status": i32(B)}

    def step():
        graft.graft_retrieve(d["ctx"], d["ctx_len"], w.n_min, w.n_max, w.C, w.m, d["tail"], d["tail_len"], out=ret)
        graft.graft_build_tree_mask(d["parent"], d["n_nodes"], d["prefix_len"], K, 16, out=mk)
        graft.graft_tree_attn(d["q"], d["k"], d["v"], att["strides"], d["table"], d["prefix_len"], d["n_nodes"],
                              mk["mask"], w.Hkv, att["scale"], out=o, workspace=ws)
        graft.graft_matrix_update(d["tokens"], d["n_nodes"], d["logits"], Mx, target_ids=ids, workspace=mu_ws)
        graft.graft_accept(d["parent"], d["tokens"], d["n_nodes"], 16, target_ids=ids, out=acc)

    outputs = lambda: [t.clone() for t in (*ret.values(), *mk.values(), o, ids, Mx, *acc.values())]
    step()
    torch.cuda.synchronize()
    eager = outputs()

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step()
    for rep in range(4):
        for t in (*ret.values(), o, ids, *acc.values()):          # wipe, so that a replay has to write everything
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(outputs(), eager):
            assert torch.equal(a, b), "replay %d differs from the eager run" % rep
        step()                                                     # eager work between the replays
        torch.cuda.synchronize()
