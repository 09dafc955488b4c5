"""Helpers for the GPU parity tests: host<->device transfers and workload runners."""
import numpy as np
import torch

import paper_2605_20104_amd as graft


def dev(a, dtype="i32"):
    """numpy -> cuda tensor.  dtype 'bf16' takes uint16 storage bits."""
    if a is None:
        return None
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).cuda()
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def host(t):
    """cuda tensor -> numpy; bfloat16 comes back widened to float32; mask words as uint64."""
    if t is None:
        return None
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    if t.dtype == torch.int64:
        return t.cpu().numpy().view(np.uint64)
    return t.cpu().numpy()


def host_dict(d):
    torch.cuda.synchronize()
    return {k: host(v) for k, v in d.items()}


def assert_same(gpu: dict, ref: dict, keys):
    for k in keys:
        a, b = gpu[k], ref[k]
        assert a.shape == b.shape, (k, a.shape, b.shape)
        assert (a == b).all(), "%s differs:\n gpu %s\n ref %s" % (k, a.ravel()[:32], b.ravel()[:32])


def run_attn(att, dtype, prefix_len, n_nodes, mask, Hkv, layer=0, kv=0):
    """att: dict from inputs.make_attention_inputs (or same keys).  Returns float32 numpy [B,K,Hq,D]."""
    q = dev(att["q"][layer], dtype)
    k = dev(att["k_cache"][kv], dtype)
    v = dev(att["v_cache"][kv], dtype)
    out = graft.graft_tree_attn(q, k, v, att["strides"], dev(att["block_table"]), dev(prefix_len),
                                dev(n_nodes), mask, Hkv, att["scale"])
    torch.cuda.synchronize()
    return host(out).astype(np.float32)
