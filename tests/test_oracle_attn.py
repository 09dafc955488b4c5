"""Pins for the oracle's tree attention (no GPU).

The oracle computes, per (node, head), ordinary attention of that node's query
over the prefix followed by its root-to-node path.  It is pinned against a
library causal-attention routine on chain trees, against the masked-softmax
reformulation over all tree slots, and against closed forms.
"""
import math

import numpy as np
import pytest
import torch

import inputs
import oracle


def small_case(seed, B=2, K=9, Hq=4, Hkv=2, D=16, P=21, page=4, dtype="f32", layout="head_major",
               chain=False):
    rng = np.random.default_rng(seed)
    if chain:
        parent = np.tile(np.arange(-1, K - 1, dtype=np.int32), (B, 1))
    else:
        parent = np.stack([inputs.random_recursive_tree(rng, K, 6) for _ in range(B)])
    pages_per_seq = (P + K + page - 1) // page
    n_pages = B * pages_per_seq + 3
    table = rng.permutation(n_pages)[:B * pages_per_seq].astype(np.int32).reshape(B, pages_per_seq)
    shape = (n_pages, Hkv, page, D) if layout == "head_major" else (n_pages, page, Hkv, D)
    k = rng.standard_normal(shape).astype(np.float32)
    v = rng.standard_normal(shape).astype(np.float32)
    q = rng.standard_normal((B, K, Hq, D)).astype(np.float32)
    if dtype == "bf16":
        q, k, v = (inputs.f32_to_bf16_bits(a) for a in (q, k, v))
    if layout == "head_major":
        strides = {"page": Hkv * page * D, "token": D, "head": page * D}
    else:
        strides = {"page": Hkv * page * D, "token": Hkv * D, "head": D}
    return dict(q=q, k=k, v=v, parent=parent, table=table, strides=strides, B=B, K=K, Hq=Hq, Hkv=Hkv,
                D=D, P=P, page=page, dtype=dtype, layout=layout, scale=1.0 / math.sqrt(D))


def run_oracle(c, rows=None, n_nodes=None, prefix=None, scale=None):
    n_nodes = [c["K"]] * c["B"] if n_nodes is None else n_nodes
    prefix = [c["P"]] * c["B"] if prefix is None else prefix
    return oracle.tree_attn(c["q"], c["k"], c["v"], c["dtype"], c["strides"], c["table"], prefix, n_nodes,
                            c["parent"], c["Hq"], c["Hkv"], c["D"], c["page"],
                            c["scale"] if scale is None else scale, rows=rows)


def logical_kv(c, b, cache, n_tok):
    """[n_tok, Hkv, D] float64 view of sequence b's tokens, gathered through the block table."""
    x = cache if c["dtype"] == "f32" else inputs.bf16_bits_to_f32(cache)
    out = np.zeros((n_tok, c["Hkv"], c["D"]))
    for t in range(n_tok):
        pg, off = c["table"][b, t // c["page"]], t % c["page"]
        out[t] = x[pg, :, off, :] if c["layout"] == "head_major" else x[pg, off, :, :]
    return out


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chain_tree_equals_library_causal_attention(dtype):
    """A chain tree is plain causal decoding: compare with torch SDPA in fp64 (GQA by head repeat)."""
    c = small_case(1, chain=True, dtype=dtype, Hq=6, Hkv=2, K=7, P=19)
    out = run_oracle(c)
    G = c["Hq"] // c["Hkv"]
    for b in range(c["B"]):
        n_tok = c["P"] + c["K"]
        k = torch.from_numpy(logical_kv(c, b, c["k"], n_tok)).permute(1, 0, 2)     # [Hkv, T, D]
        v = torch.from_numpy(logical_kv(c, b, c["v"], n_tok)).permute(1, 0, 2)
        qf = c["q"][b] if dtype == "f32" else inputs.bf16_bits_to_f32(c["q"][b])
        q_all = torch.zeros(c["Hq"], n_tok, c["D"], dtype=torch.float64)
        q_all[:, c["P"]:, :] = torch.from_numpy(qf.astype(np.float64)).permute(1, 0, 2)
        ref = torch.nn.functional.scaled_dot_product_attention(
            q_all[None], k.repeat_interleave(G, 0)[None], v.repeat_interleave(G, 0)[None], is_causal=True)
        ref = ref[0, :, c["P"]:, :].permute(1, 0, 2).numpy()                       # [K, Hq, D]
        assert np.abs(out[b] - ref).max() < 1e-12


@pytest.mark.parametrize("seed,layout,dtype", [(2, "head_major", "f32"), (3, "token_major", "f32"),
                                                (4, "head_major", "bf16"), (5, "token_major", "bf16")])
def test_equals_masked_softmax_over_tree_slots(seed, layout, dtype):
    """Per-path attention == softmax over prefix + tree slots restricted by the ancestor mask."""
    c = small_case(seed, layout=layout, dtype=dtype, P=23 + seed)      # P not a page multiple
    out = run_oracle(c)
    mk = oracle.build_tree_mask(c["parent"], [c["K"]] * c["B"], [c["P"]] * c["B"])["mask"]
    G = c["Hq"] // c["Hkv"]
    qf = c["q"] if dtype == "f32" else inputs.bf16_bits_to_f32(c["q"])
    for b in range(c["B"]):
        n_tok = c["P"] + c["K"]
        k, v = logical_kv(c, b, c["k"], n_tok), logical_kv(c, b, c["v"], n_tok)
        for i in range(c["K"]):
            allowed = np.ones(n_tok, bool)
            for j in range(c["K"]):
                allowed[c["P"] + j] = bool((int(mk[b, i, j // 64]) >> (j % 64)) & 1)
            for h in range(c["Hq"]):
                s = k[:, h // G, :] @ qf[b, i, h].astype(np.float64) * c["scale"]
                s[~allowed] = -np.inf
                p = np.exp(s - s.max())
                p /= p.sum()
                ref = p @ v[:, h // G, :]
                assert np.abs(out[b, i, h] - ref).max() < 1e-12


def test_closed_forms():
    c = small_case(6)
    # zero queries: uniform weights -> plain mean of V over prefix + path
    c0 = dict(c, q=np.zeros_like(c["q"]))
    out = run_oracle(c0)
    for b in range(c["B"]):
        v = logical_kv(c, b, c["v"], c["P"] + c["K"])
        for i in range(c["K"]):
            path, j = [], i
            while j != -1:
                path.append(c["P"] + j)
                j = int(c["parent"][b, j])
            idx = list(range(c["P"])) + path
            for h in range(c["Hq"]):
                assert np.abs(out[b, i, h] - v[idx, h // 2, :].mean(axis=0)).max() < 1e-12
    # constant V: output is that constant
    cv = dict(c, v=np.full_like(c["v"], 0.375))
    assert np.abs(run_oracle(cv) - 0.375).max() < 1e-12
    # siblings with equal queries and equal ancestor sets... and a leaf vs its copy: rows with the
    # same path set give the same output.  Root row: prefix + root only.
    r = run_oracle(c, rows=np.array([[0, 0, 1]], np.int32))
    k, v = logical_kv(c, 0, c["k"], c["P"] + 1), logical_kv(c, 0, c["v"], c["P"] + 1)
    s = k[:, 0, :] @ c["q"][0, 0, 1].astype(np.float64) * c["scale"]
    p = np.exp(s - s.max())
    assert np.abs(r[0] - (p / p.sum()) @ v[:, 0, :]).max() < 1e-12


def test_scale_matters_and_rows_subset_matches_full():
    c = small_case(7)
    full = run_oracle(c)
    rows = np.array([[1, 3, 2], [0, 8, 0], [1, 0, 3]], np.int32)
    sub = run_oracle(c, rows=rows)
    for r, (b, i, h) in enumerate(rows):
        assert (sub[r] == full[b, i, h]).all()
    assert np.abs(run_oracle(c, scale=1.0) - full).max() > 1e-3


def test_page_permutation_and_padding_rows():
    c = small_case(8)
    ref = run_oracle(c)
    # move every page: permute the physical pool and remap the table -> same result, bit for bit
    rng = np.random.default_rng(0)
    n_pages = c["k"].shape[0]
    perm = rng.permutation(n_pages)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(n_pages)
    c2 = dict(c, k=c["k"][perm], v=c["v"][perm], table=inv[c["table"]].astype(np.int32))
    assert (run_oracle(c2) == ref).all()
    # fewer nodes: rows of padding nodes are zero, others unchanged (later nodes never affect earlier)
    out = run_oracle(c, n_nodes=[5, 9])
    assert (out[0, 5:] == 0).all() and (out[0, :5] == ref[0, :5]).all() and (out[1] == ref[1]).all()
    # empty prefix: attention over the path only; the root attends to itself alone -> its own V
    out0 = run_oracle(c, prefix=[0, 0])
    v = logical_kv(c, 0, c["v"], 1)
    assert np.abs(out0[0, 0, 0] - v[0, 0]).max() < 1e-12


def test_bf16_storage_is_widened_exactly():
    c = small_case(9, dtype="bf16")
    wide = dict(c, dtype="f32", q=inputs.bf16_bits_to_f32(c["q"]), k=inputs.bf16_bits_to_f32(c["k"]),
                v=inputs.bf16_bits_to_f32(c["v"]))
    assert (run_oracle(c) == run_oracle(wide)).all()
    x = np.array([1.0, 1.00390625, -2.5, 3.1415927, 1e-30], np.float32)
    rt = inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(x))
    assert rt.tolist() == torch.tensor(x).to(torch.bfloat16).to(torch.float32).tolist()
