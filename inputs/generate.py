"""Seeded generators: contexts with planted repeats, hybrid draft trees, paged KV.

Everything is drawn from numpy's PCG64 keyed by (base seed + config index,
sequence, purpose), so the oracle tests and the GPU tests read the same bytes.
No step of the verification path is computed here: the generator only *plants*
structure (repeated spans, a query n-gram with known continuations, a toy
next-token rule that decides which draft tokens are "right") and lays data out.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Tuple

import numpy as np

from .workloads import Workload

BASE_SEED = 0x20104

# purposes (sub-stream keys)
_S_CTX, _S_TREE, _S_TOK, _S_Q, _S_KV, _S_TABLE, _S_LOGITS, _S_PLANT = range(8)


def _rng(seed: int, *path: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, *path])))


# --------------------------------------------------------------------------
# storage helpers
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest even) and return the 16 storage bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 storage bits to fp32 exactly."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_storage(rng: np.random.Generator, shape, dtype: str) -> np.ndarray:
    """N(0,1) values in the storage type: float32 array or uint16 bf16 bits."""
    n = int(np.prod(shape))
    if dtype == "f32":
        return rng.standard_normal(n, dtype=np.float32).reshape(shape)
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        out[lo:hi] = f32_to_bf16_bits(rng.standard_normal(hi - lo, dtype=np.float32))
    return out.reshape(shape)


# --------------------------------------------------------------------------
# toy target: a deterministic "model" deciding the next token from the last 3
# --------------------------------------------------------------------------
_M64 = (1 << 64) - 1


def toy_target(last3, vocab: int, seed: int) -> int:
    """Next token of a fixed pseudo-random rule applied to the last three tokens.

    Stands in for the target model's greedy choice, so that greedy decoding
    with it is a well-defined sequence any verification step can be checked
    against (the lossless property, App. B.4).
    """
    a, b, c = (int(t) for t in last3)
    x = (seed * 0x9E3779B97F4A7C15 + a * 0xBF58476D1CE4E5B9
         + b * 0x94D049BB133111EB + c * 0xD6E8FEB86659FD93 + 0x2545F4914F6CDD1D) & _M64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & _M64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & _M64
    x ^= x >> 31
    return int(x % vocab)


def _path_tokens(parent: np.ndarray, tokens: np.ndarray, i: int) -> List[int]:
    """Tokens on the root->i path, root first (layout helper for the generator)."""
    out = []
    j = i
    while j != -1:
        out.append(int(tokens[j]))
        j = int(parent[j])
    return out[::-1]


def toy_target_for_nodes(ctx_tail3, parent, tokens, n_nodes: int, vocab: int, seed: int) -> np.ndarray:
    """toy_target at every node: the rule applied to (context, then root..node tokens).

    `ctx_tail3` are the three context tokens *before* the root token (the root
    is the last context token and is tokens[0]).
    """
    out = np.full(len(parent), -1, dtype=np.int32)
    for i in range(n_nodes):
        seq = [int(t) for t in ctx_tail3] + _path_tokens(parent, tokens, i)
        out[i] = toy_target(seq[-3:], vocab, seed)
    return out


# --------------------------------------------------------------------------
# trees
# --------------------------------------------------------------------------
def random_recursive_tree(rng: np.random.Generator, n: int, max_depth: int) -> np.ndarray:
    """parent[i] ~ U[0, i), redrawn while the depth would exceed max_depth."""
    parent = np.full(n, -1, dtype=np.int32)
    depth = np.zeros(n, dtype=np.int32)
    for i in range(1, n):
        while True:
            p = int(rng.integers(0, i))
            if depth[p] + 1 <= max_depth:
                break
        parent[i] = p
        depth[i] = depth[p] + 1
    return parent


def _dense_pruned_tree(rng: np.random.Generator, n_keep: int, topk: int, max_depth: int,
                       n_dense: int):
    """A draft tree shaped like a confidence-pruned top-k expansion.

    Synthetic scores replace the draft model (Sec. 3.1: cumulative path score =
    parent's score + log q(child)): every expanded node gets `topk` children
    whose log-probabilities are the top of a log-softmax over seeded N(0, 2^2)
    logits; per depth the `topk` best nodes are expanded; the `n_dense` best
    nodes overall form the dense tree and the `n_keep` best of those are
    retained (App. A, Alg. 2 "keep the top K_draft nodes by cumulative path
    score").  Scores strictly decrease along a path, so both sets are
    ancestor-closed.  Returns (parent, rank, open_nodes): nodes renumbered by
    (depth, -score); rank = sibling rank of the node under its parent;
    open_nodes = retained nodes none of whose children were retained.
    """
    cand_parent = [-1]
    cand_score = [0.0]
    cand_depth = [0]
    cand_rank = [0]
    frontier = [0]
    for d in range(1, max_depth + 1):
        new = []
        for p in frontier:
            logits = rng.standard_normal(32) * 2.0
            lse = math.log(float(np.exp(logits - logits.max()).sum())) + float(logits.max())
            logp = np.sort(logits - lse)[::-1][:topk]
            for r, lp in enumerate(logp):
                cand_parent.append(p)
                cand_score.append(cand_score[p] + float(lp))
                cand_depth.append(d)
                cand_rank.append(r)
                new.append(len(cand_parent) - 1)
        new.sort(key=lambda c: -cand_score[c])
        frontier = new[:topk]
    order = sorted(range(len(cand_parent)), key=lambda c: -cand_score[c])
    dense = order[:max(n_dense, n_keep)]
    keep = dense[:n_keep]
    keep_sorted = sorted(keep, key=lambda c: (cand_depth[c], -cand_score[c]))
    new_id = {c: i for i, c in enumerate(keep_sorted)}
    parent = np.array([new_id[cand_parent[c]] if cand_parent[c] >= 0 else -1
                       for c in keep_sorted], dtype=np.int32)
    rank = np.array([cand_rank[c] for c in keep_sorted], dtype=np.int32)
    has_child = np.zeros(n_keep, dtype=bool)
    has_child[parent[1:]] = True
    open_nodes = [i for i in range(n_keep) if not has_child[i]]
    return parent, rank, open_nodes


def make_tree(w: Workload, seed: int, b: int, ctx_tail4: np.ndarray) -> Dict[str, object]:
    """One sequence's hybrid tree: retained draft nodes first, grafted pieces appended.

    `ctx_tail4` = the last four context tokens; the last of them is the root
    token x_t (retrieval and drafting are rooted at the current token,
    Sec. 3.2).  Returns parent/tokens/kind arrays of length w.K plus the layout
    of the grafted pieces; the retrieved chains' tokens are left at -1 for
    make_context to fill with what it plants.
    """
    rng = _rng(seed, b, _S_TREE)
    pieces = list(w.chains)
    if w.tree == "mixed":
        n_ret = int(rng.integers(1, 4))
        pieces = pieces[:n_ret]
        max_depth = int(rng.integers(2, 8))
    else:
        max_depth = 6
    n_graft = sum(m for _, m in pieces)
    n_nodes = w.K if w.tree != "mixed" else w.K  # every sequence fills its budget
    n_draft = n_nodes - n_graft
    if w.tree == "recursive":
        parent_d = random_recursive_tree(rng, n_draft, 5)
        rank = np.zeros(n_draft, dtype=np.int32)
        seen: Dict[int, int] = {}
        for i in range(1, n_draft):
            rank[i] = seen.get(int(parent_d[i]), 0)
            seen[int(parent_d[i])] = rank[i] + 1
        has_child = np.zeros(n_draft, dtype=bool)
        has_child[parent_d[1:]] = True
        open_nodes = [i for i in range(n_draft) if not has_child[i]]
    else:
        parent_d, rank, open_nodes = _dense_pruned_tree(
            rng, n_draft, topk=10, max_depth=max_depth, n_dense=max(60, n_draft))
    parent = np.full(w.K, -1, dtype=np.int32)
    parent[:n_draft] = parent_d
    kind = np.zeros(w.K, dtype=np.int8)
    tokens = np.full(w.K, -1, dtype=np.int32)
    tokens[0] = int(ctx_tail4[-1])

    # draft tokens: the best-ranked child is the toy target's token with
    # probability 0.75, everything else is a uniform draw distinct from it.
    trng = _rng(seed, b, _S_TOK)
    tseed = seed + 7919 * b
    for i in range(1, n_draft):
        p = int(parent[i])
        seq = [int(t) for t in ctx_tail4[:3]] + _path_tokens(parent, tokens, p)
        right = toy_target(seq[-3:], w.vocab, tseed)
        if rank[i] == 0 and trng.random() < 0.75:
            tokens[i] = right
        else:
            t = int(trng.integers(0, w.vocab))
            tokens[i] = t if t != right else (t + 1) % w.vocab

    # grafted pieces
    layout = []
    nxt = n_draft
    open_sorted = sorted(open_nodes) if open_nodes else [0]
    depth = np.zeros(w.K, dtype=np.int32)
    for i in range(1, n_draft):
        depth[i] = depth[parent[i]] + 1
    ret_attach: Optional[int] = None
    blocks_done = 0
    for kind_name, m in pieces:
        if kind_name == "block":
            # first block hangs off the root, later ones off open draft nodes
            attach = 0 if blocks_done == 0 else open_sorted[(blocks_done * 3) % len(open_sorted)]
            blocks_done += 1
            for j in range(m):
                parent[nxt + j] = attach if j == 0 else nxt + j - 1
                kind[nxt + j] = 2
                seq = [int(t) for t in ctx_tail4[:3]] + _path_tokens(parent, tokens, int(parent[nxt + j]))
                right = toy_target(seq[-3:], w.vocab, tseed)
                if trng.random() < 0.8:
                    tokens[nxt + j] = right
                else:
                    tokens[nxt + j] = (right + 1 + int(trng.integers(0, w.vocab - 1))) % w.vocab
            layout.append({"kind": "block", "start": nxt, "len": m, "attach": attach})
            if ret_attach is None:
                ret_attach = nxt + m - 1        # retrieval continues the first block's tail
            nxt += m
        else:
            if ret_attach is None:
                # a pruned leaf: the shallowest open node that is not the root if any
                cands = [o for o in open_sorted if o != 0] or [0]
                ret_attach = cands[int(rng.integers(0, len(cands)))]
            for j in range(m):
                parent[nxt + j] = ret_attach if j == 0 else nxt + j - 1
                kind[nxt + j] = 1
            layout.append({"kind": "ret", "start": nxt, "len": m, "attach": ret_attach})
            nxt += m
    assert nxt == n_nodes
    tail = _path_tokens(parent, tokens, ret_attach if ret_attach is not None else 0)[1:]
    return {"parent": parent, "tokens": tokens, "kind": kind, "n_nodes": n_nodes,
            "n_draft": n_draft, "layout": layout, "ret_attach": ret_attach,
            "tail": np.array(tail, dtype=np.int32), "toy_seed": tseed}


# --------------------------------------------------------------------------
# context buffers
# --------------------------------------------------------------------------
def _token_sampler(w: Workload, seed: int):
    """Returns draw(rng, n): n tokens, Zipf(s) over the vocabulary or uniform."""
    if w.zipf_s <= 0:
        return lambda rng, n: rng.integers(0, w.vocab, size=n, dtype=np.int64).astype(np.int32)
    ranks = np.arange(1, w.vocab + 1, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-w.zipf_s))
    cdf /= cdf[-1]
    perm = _rng(seed, 0xA11CE).permutation(w.vocab).astype(np.int32)   # rank -> token id

    def draw(rng, n):
        r = np.searchsorted(cdf, rng.random(n), side="left")
        return perm[np.minimum(r, w.vocab - 1)]
    return draw


def make_context(w: Workload, seed: int, b: int, draw=None):
    """Base context of one sequence before the query n-gram is planted.

    Tokens are Zipf(s) over the vocabulary (uniform for the tiny config) with
    `n_spans` repeated spans (each span copied once to another place), as in
    code or meeting transcripts where local stretches recur.  The last n_max
    tokens are drawn uniformly so that the query n-gram is distinctive.
    """
    rng = _rng(seed, b, _S_CTX)
    draw = draw or _token_sampler(w, seed)
    ctx = draw(rng, w.L).astype(np.int32)
    guard = w.L - w.n_max - 1
    for _ in range(w.n_spans):
        ln = int(rng.integers(w.span_lo, w.span_hi + 1))
        src = int(rng.integers(0, guard - ln))
        dst = int(rng.integers(0, guard - ln))
        ctx[dst:dst + ln] = ctx[src:src + ln].copy()
    ctx[w.L - w.n_max:] = rng.integers(0, w.vocab, size=w.n_max, dtype=np.int64).astype(np.int32)
    return ctx


def _plant_query(w: Workload, seed: int, b: int, ctx: np.ndarray, tail: np.ndarray,
                 toy_seed: int, n_occ: int):
    """Copy the query n-gram to n_occ earlier places, each followed by its own continuation.

    The query is the last n_max tokens of (context ++ tail).  Returns the
    planted continuation starts (descending) and their m-token continuations.
    The continuation of the most recent occurrence follows the toy target for
    a random number of tokens, so grafted chains are sometimes accepted.
    """
    rng = _rng(seed, b, _S_PLANT)
    q = np.concatenate([ctx, tail])[-w.n_max:]
    slot = w.n_max + w.m + 2
    limit = w.L - w.n_max - 1 - slot            # keep clear of the query itself
    n_slots = limit // slot
    assert n_slots >= n_occ, "context too short to plant the query n-gram"
    chosen = np.sort(rng.choice(n_slots, size=n_occ, replace=False))
    starts, conts = [], []
    first_tokens = set()
    for k, s in enumerate(chosen):
        at = int(s) * slot + 1
        e = at + w.n_max
        ctx[at:e] = q
        hist = [int(t) for t in np.concatenate([ctx[-4:-1], ctx[-1:], tail])]
        cont = []
        follow = int(rng.integers(0, w.m + 1)) if k == n_occ - 1 else 0
        for j in range(w.m):
            right = toy_target(hist[-3:], w.vocab, toy_seed)
            if j < follow:
                t = right
            else:
                t = (right + 1 + int(rng.integers(0, w.vocab - 1))) % w.vocab
            if j == 0:
                while t in first_tokens:
                    t = (t + 1) % w.vocab
                first_tokens.add(t)
            cont.append(t)
            hist.append(t)
        ctx[e:e + w.m] = np.array(cont, dtype=np.int32)
        # the token right before the planted n-gram must not extend the match
        starts.append(e)
        conts.append(cont)
    order = np.argsort(starts)[::-1]
    return [starts[i] for i in order], [conts[i] for i in order]


# --------------------------------------------------------------------------
# one step's integer inputs (retrieval, tree, acceptance)
# --------------------------------------------------------------------------
def make_step_inputs(w: Workload, seed: Optional[int] = None, with_logits: bool = False):
    """All integer-side inputs of one verification step for workload `w`.

    Keys: ctx [B,L], ctx_len [B], tail [B,tail_max], tail_len [B], parent
    [B,K], tokens [B,K] (retrieved slots filled with the planted
    continuations, i.e. what exact retrieval returns), kind [B,K], n_nodes [B],
    prefix_len [B], target_ids [B,K] (toy target at every node), planted_pos /
    planted_tok (the known answers of retrieval: continuation starts in
    descending order and their tokens), ret_slots (per sequence the start slot
    of each retrieved chain), and optionally logits [B,K,vocab] fp32 whose
    row-wise first maximum is target_ids.
    """
    seed = BASE_SEED + w.index if seed is None else seed
    draw = _token_sampler(w, seed)
    B, K = w.B, w.K
    ctx = np.zeros((B, w.L), dtype=np.int32)
    parent = np.full((B, K), -1, dtype=np.int32)
    tokens = np.full((B, K), -1, dtype=np.int32)
    kind = np.zeros((B, K), dtype=np.int8)
    n_nodes = np.zeros(B, dtype=np.int32)
    target_ids = np.full((B, K), -1, dtype=np.int32)
    tails, planted_pos, planted_tok, ret_slots, layouts = [], [], [], [], []
    n_occ = 3 if w.name == "c1" else w.C + 2
    for b in range(B):
        c = make_context(w, seed, b, draw)
        t = make_tree(w, seed, b, c[-4:])
        pos, conts = _plant_query(w, seed, b, c, t["tail"], t["toy_seed"], n_occ)
        slots = [p["start"] for p in t["layout"] if p["kind"] == "ret"]
        for r, s in enumerate(slots):
            t["tokens"][s:s + w.m] = np.array(conts[r], dtype=np.int32)
        ctx[b] = c
        parent[b], tokens[b], kind[b], n_nodes[b] = t["parent"], t["tokens"], t["kind"], t["n_nodes"]
        target_ids[b] = toy_target_for_nodes(c[-4:-1], t["parent"], t["tokens"], t["n_nodes"],
                                             w.vocab, t["toy_seed"])
        tails.append(t["tail"])
        planted_pos.append(pos)
        planted_tok.append(conts)
        ret_slots.append(slots)
        layouts.append(t["layout"])
    tail_max = max(1, max(len(t) for t in tails))
    tail = np.full((B, tail_max), -1, dtype=np.int32)
    tail_len = np.zeros(B, dtype=np.int32)
    for b, t in enumerate(tails):
        tail[b, :len(t)] = t
        tail_len[b] = len(t)
    out = {
        "ctx": ctx, "ctx_len": np.full(B, w.L, dtype=np.int32),
        "tail": tail, "tail_len": tail_len,
        "parent": parent, "tokens": tokens, "kind": kind, "n_nodes": n_nodes,
        "prefix_len": np.full(B, w.P, dtype=np.int32), "target_ids": target_ids,
        "planted_pos": planted_pos, "planted_tok": planted_tok, "ret_slots": ret_slots,
        "layouts": layouts, "seed": seed,
    }
    if with_logits:
        lrng = _rng(seed, _S_LOGITS)
        logits = lrng.standard_normal((B, K, w.vocab), dtype=np.float32)
        for b in range(B):
            for i in range(int(n_nodes[b])):
                logits[b, i, target_ids[b, i]] = 12.0 + float(lrng.random())
        out["logits"] = logits
    return out


# --------------------------------------------------------------------------
# attention operands
# --------------------------------------------------------------------------
def make_attention_inputs(w: Workload, seed: Optional[int] = None, kv_buffers: Optional[int] = None,
                          q_layers: int = 1, layout: str = "head_major",
                          P: Optional[int] = None, K: Optional[int] = None):
    """Q, the paged K/V caches and the block table for workload `w`.

    Q: [q_layers, B, K, Hq, D]; caches: `kv_buffers` of them (default
    w.distinct_kv_layers), each [n_pages, Hkv, page, D] ("head_major": one
    page of one KV head is contiguous) or [n_pages, page, Hkv, D]
    ("token_major"); values N(0,1) in the storage type (fp32, or bf16 bits as
    uint16).  The pool holds 1.25x the pages in use and the block table
    [B, pages_per_seq] is a random injection into it, never the identity.
    Token t of sequence b (prefix positions 0..P-1, then tree slot j at P+j)
    lives in page block_table[b, t // page] at offset t % page.
    """
    seed = BASE_SEED + w.index if seed is None else seed
    P = w.P if P is None else P
    K = w.K if K is None else K
    nb = w.distinct_kv_layers if kv_buffers is None else kv_buffers
    pages_per_seq = (P + K + w.page_size - 1) // w.page_size
    n_pages = int(math.ceil(1.25 * w.B * pages_per_seq))
    trng = _rng(seed, _S_TABLE)
    block_table = trng.permutation(n_pages)[: w.B * pages_per_seq].astype(np.int32)
    block_table = block_table.reshape(w.B, pages_per_seq)
    shape = ((n_pages, w.Hkv, w.page_size, w.D) if layout == "head_major"
             else (n_pages, w.page_size, w.Hkv, w.D))
    k_caches, v_caches = [], []
    for l in range(nb):
        krng = _rng(seed, _S_KV, l)
        k_caches.append(_normal_storage(krng, shape, w.dtype))
        v_caches.append(_normal_storage(krng, shape, w.dtype))
    q = _normal_storage(_rng(seed, _S_Q), (q_layers, w.B, K, w.Hq, w.D), w.dtype)
    if layout == "head_major":
        strides = {"page": w.Hkv * w.page_size * w.D, "token": w.D, "head": w.page_size * w.D}
    else:
        strides = {"page": w.Hkv * w.page_size * w.D, "token": w.Hkv * w.D, "head": w.D}
    return {"q": q, "k_cache": k_caches, "v_cache": v_caches, "block_table": block_table,
            "strides": strides, "n_pages": n_pages, "pages_per_seq": pages_per_seq,
            "P": P, "K": K, "scale": 1.0 / math.sqrt(w.D)}
