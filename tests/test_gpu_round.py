"""One whole decoding round (App. A Alg. 1 loop body with Alg. 2) on the GPU, every call feeding
the next, against the same chain of oracle calls: gates + selection -> matrix retrieval -> rebuild
-> tree attention -> matrix refresh -> acceptance -> cache update."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2605_20104_amd as graft
from gpu_util import dev, host
from inputs import templates

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed,dtype,log_tau", [(0, "bf16", [-0.5, -2.0, -60.0]), (1, "bf16", [-60.0, -60.0, -1.0]),
                                                (2, "f32", [-60.0, -60.0, -60.0]), (3, "bf16", [-0.1, -1.0, -2.0])])
def test_round_matches_the_oracle_chain(seed, dtype, log_tau):
    rng = np.random.default_rng(100 + seed)
    B, K, V, kk = 2, 64, 3000, 8
    Hq, Hkv, D = (8, 2, 128) if dtype == "bf16" else (4, 2, 64)
    P = np.array([300, 77], np.int32)
    base = inputs.get_workload("c2")
    import dataclasses
    w = dataclasses.replace(base, name="round", index=20 + seed, B=B, K=K, Hq=Hq, Hkv=Hkv, D=D, P=int(P.max()),
                            dtype=dtype, layers=1, distinct_kv_layers=1, vocab=V)
    # a full 60-node draft tree per sequence with log-probabilities, the matrix, the templates
    n_draft = np.array([60, 60], np.int32)
    parent = np.full((B, K), -1, np.int32)
    for b in range(B):
        depth = [0]
        for i in range(1, 60):
            while True:
                p = int(rng.integers(0, i))
                if depth[p] < 8:
                    break
            parent[b, i] = p
            depth.append(depth[p] + 1)
    tokens = rng.integers(0, V, (B, K)).astype(np.int32)
    logq = np.log(rng.random((B, K)).astype(np.float32) * 0.9 + 0.05).astype(np.float32)
    M0 = rng.integers(0, V, (V, kk), dtype=np.int32)
    tp, tr, td, sizes = templates.retrieval_envelope()
    chk = (np.array([1, 2, 6], np.int32), np.array([8, 24, 40], np.int32),
           np.array([sizes["d0"], sizes["d1"], sizes["d5"]], np.int32))
    att = inputs.make_attention_inputs(w, seed=seed)
    logits = rng.standard_normal((B, K, V)).astype(np.float32)
    kind = "f32" if dtype == "f32" else "bf16"

    # ---- oracle chain
    o1 = oracle.prune_select(parent, tokens, logq, n_draft, chk[0], log_tau, chk[1], chk[2])
    o2 = oracle.matrix_retrieve(M0, tp, tr, o1["n_ret"], o1["tokens"], o1["parent"], o1["n_nodes"])
    assert (o2["n_nodes"] == o1["n_nodes"] + o1["n_ret"]).all() and (o2["n_nodes"] <= 60).all()
    o3 = oracle.build_tree_mask(o2["parent"], o2["n_nodes"], P, K, 16)
    o4 = oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], dtype, att["strides"], att["block_table"],
                          P, o2["n_nodes"], o2["parent"], Hq, Hkv, D, 16, att["scale"])
    # let the target agree with some retrieved tokens so that paths get accepted
    for b in range(B):
        for i in range(1, int(o2["n_nodes"][b])):
            if rng.random() < 0.6 and o2["tokens"][b, i] >= 0:
                logits[b, o2["parent"][b, i], o2["tokens"][b, i]] += 9.0
    o5 = oracle.matrix_update(M0, o2["tokens"], o2["n_nodes"], logits)
    o6 = oracle.accept(o2["parent"], o2["tokens"], o2["n_nodes"], 16, target_ids=o5["target_ids"])
    o7 = oracle.kv_compact(att["k_cache"][0].reshape(-1), att["v_cache"][0].reshape(-1), dtype, 0, 1, att["strides"],
                           att["block_table"], P, o6["path"], o6["accept_len"], K, Hkv, D)

    # ---- the same on the GPU, outputs feeding inputs without leaving the device
    g1 = graft.graft_prune_select(dev(parent), dev(tokens), dev(logq, "f32"), dev(n_draft), dev(chk[0]),
                                  dev(np.array(log_tau, np.float32), "f32"), dev(chk[1]), dev(chk[2]))
    Md = dev(M0)
    graft.graft_matrix_retrieve(Md, dev(tp), dev(tr), g1["n_ret"], g1["tokens"], g1["parent"], g1["n_nodes"])
    Pd = dev(P)
    g3 = graft.graft_build_tree_mask(g1["parent"], g1["n_nodes"], Pd, K, 16)
    kd, vd = dev(att["k_cache"][0], kind), dev(att["v_cache"][0], kind)
    g4 = graft.graft_tree_attn(dev(att["q"][0], kind), kd, vd, att["strides"], dev(att["block_table"]), Pd,
                               g1["n_nodes"], g3["mask"], Hkv, att["scale"])
    ids = graft.graft_matrix_update(g1["tokens"], g1["n_nodes"], dev(logits, "f32"), Md)
    g6 = graft.graft_accept(g1["parent"], g1["tokens"], g1["n_nodes"], 16, target_ids=ids)
    g7 = graft.graft_kv_compact(kd.view(-1), vd.view(-1), 0, 1, att["strides"], dev(att["block_table"]), Pd,
                                g6["path"], g6["accept_len"], K, Hkv, D)
    torch.cuda.synchronize()

    assert (host(g1["stage"]) == o1["stage"]).all() and (host(g1["n_nodes"]) == o2["n_nodes"]).all()
    assert (host(g1["tokens"]) == o2["tokens"]).all() and (host(g1["parent"]) == o2["parent"]).all()
    for key in ("mask", "pos", "depth", "paths"):
        assert (host(g3[key]) == o3[key]).all(), key
    tol = 2e-2 if dtype == "bf16" else 2e-5
    for b in range(B):
        n = int(o2["n_nodes"][b])
        assert np.abs(host(g4)[b, :n] - o4[b, :n]).max() <= tol
    assert (host(ids) == o5["target_ids"]).all() and (host(Md) == o5["M"]).all()
    for key in ("accept_len", "best_node", "path", "out_tokens", "status"):
        assert (host(g6[key]) == o6[key]).all(), key
    assert (host(g7["new_prefix_len"]) == o7["new_prefix_len"]).all() and (host(g7["status"]) == 0).all()
    bits = (lambda t: t.cpu().numpy().reshape(-1)) if dtype == "f32" else \
        (lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1))
    assert (bits(kd) == o7["k_cache"]).all() and (bits(vd) == o7["v_cache"]).all()
    assert int(o6["accept_len"].max()) >= 1                               # the round accepted something
