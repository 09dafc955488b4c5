"""Pins of the oracle's cache update after acceptance (App. A Alg. 1; App. D runtime table)."""
import numpy as np

import inputs
import oracle
from _golden import ints, read_fixture


def _one_head_cache(keys):
    """Logical positions -> a paged cache with one KV head and D = 1, pages scattered on purpose."""
    n = len(keys)
    n_pages = (n + 15) // 16 + 2
    table = np.array([[2, 0, 1][: (n + 15) // 16]], np.int32) if n <= 48 else None
    k = np.zeros(n_pages * 16, np.float32)
    for t, val in enumerate(keys):
        k[table[0, t // 16] * 16 + t % 16] = val
    return k, table, {"page": 16, "token": 1, "head": 1}


def test_hand_worked_update():
    g = read_fixture("kv_compact_small.txt")
    keys = [float(x) for x in g["keys"].split()]
    for pk, ak, nk in (("path", "keys_after", "new_prefix_len"),
                       ("path_chain", "keys_after_chain", "new_prefix_len_chain")):
        k, table, strides = _one_head_cache(keys)
        v = k + 100
        path = ints(g[pk])
        row = np.full((1, 6), -1, np.int32)
        row[0, :len(path)] = path
        r = oracle.kv_compact(k, v, "f32", 0, 1, strides, table, [3], row, [len(path) - 1], 7, 1, 1)
        assert r["status"].tolist() == [0] and r["new_prefix_len"].tolist() == [int(g[nk])]
        got = [r["k_cache"][table[0, t // 16] * 16 + t % 16] for t in range(len(keys))]
        assert got == [float(x) for x in g[ak].split()]
        gotv = [r["v_cache"][table[0, t // 16] * 16 + t % 16] for t in range(len(keys))]
        assert gotv == [float(x) + 100 for x in g[ak].split()]


def _random_case(seed, B=3, Hkv=2, D=8, n_layers=2, P=(5, 30, 17), K=24, token_major=False):
    rng = np.random.default_rng(seed)
    max_pages = (max(P) + K + 15) // 16
    n_pages = B * max_pages + 3
    table = rng.permutation(n_pages)[: B * max_pages].reshape(B, max_pages).astype(np.int32)
    if token_major:
        strides = {"page": 16 * Hkv * D, "token": Hkv * D, "head": D}
    else:
        strides = {"page": Hkv * 16 * D, "token": D, "head": 16 * D}
    layer_stride = n_pages * Hkv * 16 * D
    k = rng.standard_normal(n_layers * layer_stride).astype(np.float32)
    v = rng.standard_normal(n_layers * layer_stride).astype(np.float32)
    depth_cap = 8
    path = np.full((B, depth_cap + 1), -1, np.int32)
    acc = np.zeros(B, np.int32)
    for b in range(B):
        a = int(rng.integers(0, depth_cap + 1))
        nodes = np.sort(rng.choice(np.arange(1, K), size=a, replace=False))
        path[b, 0] = 0
        path[b, 1:a + 1] = nodes
        acc[b] = a
    return dict(k=k, v=v, table=table, strides=strides, layer_stride=layer_stride, n_layers=n_layers,
                P=np.array(P, np.int32), path=path, acc=acc, K=K, Hkv=Hkv, D=D, B=B, n_pages=n_pages)


def _logical(cache, c, layer, b, t, g):
    s = c["strides"]
    off = layer * c["layer_stride"] + int(c["table"][b, t // 16]) * s["page"] + (t % 16) * s["token"] + g * s["head"]
    return cache[off:off + c["D"]]


def test_gather_definition_on_random_paths():
    """new[P + k] = old[P + path[k]], taken from a snapshot; everything else bit-identical."""
    for seed, tm in ((1, False), (2, True), (3, False)):
        c = _random_case(seed, token_major=tm)
        r = oracle.kv_compact(c["k"], c["v"], "f32", c["layer_stride"], c["n_layers"], c["strides"], c["table"],
                              c["P"], c["path"], c["acc"], c["K"], c["Hkv"], c["D"])
        assert r["status"].tolist() == [0] * c["B"]
        assert r["new_prefix_len"].tolist() == (c["P"] + c["acc"] + 1).tolist()
        for name in ("k", "v"):
            want = c[name].copy()
            for l in range(c["n_layers"]):
                for b in range(c["B"]):
                    for kk in range(1, c["acc"][b] + 1):
                        for g in range(c["Hkv"]):
                            src = _logical(c[name], c, l, b, int(c["P"][b] + c["path"][b, kk]), g)
                            _logical(want, c, l, b, int(c["P"][b]) + kk, g)[:] = src
            assert (r[name + "_cache"] == want).all()


def test_accepted_leaf_sees_the_same_attention_before_and_after():
    """Tree attention of the accepted leaf over prefix + its ancestors (before the update) equals
    plain causal attention of the last position over the compacted prefix (after it)."""
    w = inputs.get_workload("c1")
    s = inputs.make_step_inputs(w, with_logits=True)
    att = inputs.make_attention_inputs(w)
    a = oracle.accept(s["parent"], s["tokens"], s["n_nodes"], 8, logits=s["logits"])
    B, K = s["parent"].shape
    assert a["accept_len"][0] >= 1
    kc, vc = att["k_cache"][0], att["v_cache"][0]
    before = oracle.tree_attn(att["q"][0], kc, vc, "f32", att["strides"], att["block_table"], s["prefix_len"],
                              s["n_nodes"], s["parent"], w.Hq, w.Hkv, w.D, 16, att["scale"])
    r = oracle.kv_compact(kc.reshape(-1), vc.reshape(-1), "f32", 0, 1, att["strides"], att["block_table"],
                          s["prefix_len"], a["path"], a["accept_len"], K, w.Hkv, w.D)
    best, al = int(a["best_node"][0]), int(a["accept_len"][0])
    # a one-node "tree" whose root sits at the last accepted position: prefix = everything before it
    q1 = att["q"][0][:, best:best + 1]
    after = oracle.tree_attn(q1, r["k_cache"], r["v_cache"], "f32", att["strides"], att["block_table"],
                             [int(s["prefix_len"][0]) + al], [1], np.array([[-1]], np.int32),
                             w.Hq, w.Hkv, w.D, 16, att["scale"])
    assert np.abs(after[0, 0] - before[0, best]).max() < 1e-12


def test_rejects_bad_paths_and_lengths():
    c = _random_case(7)
    path = c["path"].copy()
    acc = np.array([2, 2, 2], np.int32)
    path[0, :3] = [0, 5, 5]          # not increasing
    path[1, :3] = [1, 2, 3]          # does not start at the root
    path[2, :3] = [0, 3, c["K"]]     # beyond the tree
    r = oracle.kv_compact(c["k"], c["v"], "f32", c["layer_stride"], c["n_layers"], c["strides"], c["table"],
                          c["P"], path, acc, c["K"], c["Hkv"], c["D"])
    assert r["status"].tolist() == [oracle.ST_BAD_TREE] * 3
    assert (r["k_cache"] == c["k"]).all() and r["new_prefix_len"].tolist() == c["P"].tolist()
    r = oracle.kv_compact(c["k"], c["v"], "f32", c["layer_stride"], c["n_layers"], c["strides"], c["table"],
                          [-1, 5, 5], c["path"], [0, 9, -1], c["K"], c["Hkv"], c["D"])
    assert r["status"].tolist() == [oracle.ST_BAD_LENGTH] * 3
