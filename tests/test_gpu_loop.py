"""Several decoding steps in a row on the GPU (App. A Alg. 1 loop body; losslessness, App. B.4):
graft_retrieve -> append of its chains (the merge of Sec. 3.2, a plain concatenation done by the test)
-> graft_build_tree_mask -> graft_tree_attn -> graft_accept -> graft_kv_compact, with the prefix
growing by accept_len + 1 per step.  Every call's output equals the same chain of oracle calls,
attention runs on the cache that the previous step's compaction left behind, and the emitted text
equals plain greedy decoding of the toy target."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2605_20104_amd as graft
from gpu_util import dev, host

pytestmark = pytest.mark.gpu

VOCAB, SEED = 12, 3
C, M = 2, 4
K_MAX = 16
HQ, HKV, D = 8, 2, 128
DEPTH_CAP = K_MAX - 1


def greedy_decode(ctx_tail, n):
    seq = [int(t) for t in ctx_tail]
    out = []
    for _ in range(n):
        t = inputs.toy_target(seq[-3:], VOCAB, SEED)
        out.append(t)
        seq.append(t)
    return out


@pytest.mark.parametrize("steps,start_len", [(24, [40, 23])])
def test_loop_is_lossless_and_matches_the_oracle_chain(steps, start_len):
    rng = np.random.default_rng(11)
    B = len(start_len)
    L_max = max(start_len) + steps * (M + 1) + 8
    pages_per_seq = (L_max + K_MAX + 15) // 16
    n_pages = B * pages_per_seq + 5
    table = rng.permutation(n_pages)[:B * pages_per_seq].astype(np.int32).reshape(B, pages_per_seq)
    strides = {"page": HKV * 16 * D, "token": D, "head": 16 * D}
    scale = 1.0 / np.sqrt(D)
    bf = lambda shape: inputs.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))

    ctx = [[int(t) for t in rng.integers(0, VOCAB, n)] for n in start_len]
    start = [list(c) for c in ctx]
    # the cache holds keys and values of every context token but the last (the root of the next tree)
    k_ref, v_ref = bf((n_pages, HKV, 16, D)), bf((n_pages, HKV, 16, D))
    k_gpu, v_gpu = dev(k_ref, "bf16"), dev(v_ref, "bf16")
    table_d = dev(table)
    emitted = [0] * B

    def put_rows(b, pos, kr, vr):
        """Keys/values [n,HKV,D] of logical positions pos..pos+n-1 of sequence b, into both caches."""
        for j in range(kr.shape[0]):
            page, off = int(table[b, (pos + j) // 16]), (pos + j) % 16
            k_ref[page, :, off, :] = kr[j]
            v_ref[page, :, off, :] = vr[j]
            k_gpu[page, :, off, :] = dev(kr[j], "bf16")
            v_gpu[page, :, off, :] = dev(vr[j], "bf16")

    for step in range(steps):
        L = np.array([len(c) for c in ctx], np.int32)
        P = L - 1                                                # the root (last context token) is tree slot 0
        buf = np.zeros((B, L_max), np.int32)
        for b in range(B):
            buf[b, :L[b]] = ctx[b]
        # ---- retrieval: GPU vs oracle
        g_ret = graft.graft_retrieve(dev(buf), dev(L), 1, 3, C, M)
        o_ret = oracle.retrieve(buf, L, 1, 3, C, M)
        for key in ("chain_tok", "chain_len", "chain_pos", "chain_match", "n_hits", "status"):
            assert (host(g_ret[key]) == o_ret[key]).all(), (step, key)
        # ---- merge: root + three random "draft" nodes + the chains the GPU returned, under the root
        chain_len, chain_tok = host(g_ret["chain_len"]), host(g_ret["chain_tok"])
        parent = np.full((B, K_MAX), -1, np.int32)
        tokens = np.full((B, K_MAX), -1, np.int32)
        n_nodes = np.zeros(B, np.int32)
        target = np.full((B, K_MAX), -1, np.int32)
        for b in range(B):
            par, tok = [-1], [ctx[b][-1]]
            for _ in range(3):
                par.append(int(rng.integers(0, len(par))))
                tok.append(int(rng.integers(0, VOCAB)))
            for c in range(C):
                prev = 0
                for j in range(int(chain_len[b, c])):
                    par.append(prev)
                    tok.append(int(chain_tok[b, c, j]))
                    prev = len(par) - 1
            n = len(par)
            assert n <= K_MAX
            parent[b, :n], tokens[b, :n], n_nodes[b] = par, tok, n
            target[b] = inputs.toy_target_for_nodes(ctx[b][-4:-1], parent[b], tokens[b], n, VOCAB, SEED)
            put_rows(b, int(P[b]), bf((n, HKV, D)), bf((n, HKV, D)))     # the tree tokens' keys and values
        # ---- rebuild
        g_mk = graft.graft_build_tree_mask(dev(parent), dev(n_nodes), dev(P), K_MAX, DEPTH_CAP)
        o_mk = oracle.build_tree_mask(parent, n_nodes, P, K_MAX, DEPTH_CAP)
        for key in ("mask", "pos", "depth", "paths", "status"):
            assert (host(g_mk[key]) == o_mk[key]).all(), (step, key)
        # ---- attention on the cache as the previous steps left it
        q = bf((B, K_MAX, HQ, D))
        g_o = graft.graft_tree_attn(dev(q, "bf16"), k_gpu, v_gpu, strides, table_d, dev(P), dev(n_nodes),
                                    g_mk["mask"], HKV, scale)
        o_o = oracle.tree_attn(q, k_ref, v_ref, "bf16", strides, table, P, n_nodes, parent, HQ, HKV, D, 16, scale)
        err = np.abs(host(g_o).astype(np.float64) - o_o).max()
        assert err <= 2e-2, (step, err)
        # ---- acceptance
        g_acc = graft.graft_accept(dev(parent), dev(tokens), dev(n_nodes), DEPTH_CAP, target_ids=dev(target))
        o_acc = oracle.accept(parent, tokens, n_nodes, DEPTH_CAP, target_ids=target)
        for key in ("accept_len", "best_node", "path", "out_tokens", "status"):
            assert (host(g_acc[key]) == o_acc[key]).all(), (step, key)
        # ---- cache update, in place on the GPU
        g_kc = graft.graft_kv_compact(k_gpu.view(-1), v_gpu.view(-1), 0, 1, strides, table_d, dev(P), g_acc["path"],
                                      g_acc["accept_len"], K_MAX, HKV, D)
        o_kc = oracle.kv_compact(k_ref.reshape(-1), v_ref.reshape(-1), "bf16", 0, 1, strides, table, P,
                                 o_acc["path"], o_acc["accept_len"], K_MAX, HKV, D)
        torch.cuda.synchronize()
        assert (host(g_kc["status"]) == 0).all() and (o_kc["status"] == 0).all()
        assert (host(g_kc["new_prefix_len"]) == o_kc["new_prefix_len"]).all()
        k_ref, v_ref = o_kc["k_cache"].reshape(k_ref.shape), o_kc["v_cache"].reshape(v_ref.shape)
        bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
        assert (bits(k_gpu) == k_ref).all() and (bits(v_gpu) == v_ref).all(), step
        # ---- append the accepted tokens and the bonus token
        for b in range(B):
            a = int(o_acc["accept_len"][b])
            ctx[b] += [int(t) for t in o_acc["out_tokens"][b, :a + 1]]
            emitted[b] += a + 1
            assert o_kc["new_prefix_len"][b] == len(ctx[b]) - 1
    for b in range(B):
        assert ctx[b][len(start[b]):] == greedy_decode(start[b], emitted[b]), b
    assert sum(emitted) > B * steps                    # retrieval got something accepted along the way
