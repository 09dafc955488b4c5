"""Thin Python binding of libgraft.so, the C-ABI library declared in include/graft.h.

Argument marshalling only: every step of the verification path runs in the HIP
kernels behind the four entry points.  PyTorch is used for device memory and
streams; tensors are passed as raw device pointers.  There is no CPU fallback:
if the library is not built the import of its symbols raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libgraft.so")

GRAFT_MAX_NODES = 128
GRAFT_MASK_WORDS = 2
GRAFT_MAX_CHAINS = 8
GRAFT_MAX_NGRAM = 32
GRAFT_PAGE_SIZE = 16
GRAFT_MAX_SUCCESSORS = 16
GRAFT_MAX_CHECKPOINTS = 16
GRAFT_NOALLOC_MAX_ROWS = 8192
GRAFT_OK, GRAFT_ERR_NULL, GRAFT_ERR_SHAPE, GRAFT_ERR_DTYPE, GRAFT_ERR_WORKSPACE, GRAFT_ERR_HIP = range(6)
GRAFT_STATUS_BAD_LENGTH, GRAFT_STATUS_BAD_TREE, GRAFT_STATUS_PATH_OVERFLOW = 1, 2, 4
GRAFT_F32, GRAFT_BF16 = 0, 1

_ERR_NAMES = {1: "GRAFT_ERR_NULL", 2: "GRAFT_ERR_SHAPE", 3: "GRAFT_ERR_DTYPE",
              4: "GRAFT_ERR_WORKSPACE", 5: "GRAFT_ERR_HIP"}

_i32, _i64, _f32, _vp, _sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
_SIGNATURES = {
    "graft_last_hip_error": (_i32, []),
    "graft_version": (_i32, []),
    "graft_retrieve": (_i32, [_vp, _vp, _i32, _i32, _vp, _vp, _i32, _i32, _i32, _i32, _i32,
                              _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "graft_build_tree_mask": (_i32, [_vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp]),
    "graft_tree_attn_workspace_bytes": (_sz, [_i32] * 7),
    "graft_tree_attn": (_i32, [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _i32, _vp, _vp, _vp,
                               _i32, _i32, _i32, _i32, _i32, _i32, _f32, _i32, _vp, _vp, _sz, _vp]),
    "graft_attn_profile_events": (_i32, [_vp, _vp, _i32]),
    "graft_accept_workspace_bytes": (_sz, [_i32] * 3),
    "graft_accept": (_i32, [_vp, _vp, _vp, _vp, _i32, _vp, _i32, _i32, _i32,
                            _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "graft_accept_noalloc": (_i32, [_vp, _vp, _vp, _vp, _i32, _vp, _i32, _i32, _i32,
                                    _vp, _vp, _vp, _vp, _vp, _vp]),
    "graft_prune_select": (_i32, [_vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _i32] + [_vp] * 8),
    "graft_matrix_retrieve": (_i32, [_vp, _i32, _i32, _vp, _vp, _i32, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp]),
    "graft_matrix_update_workspace_bytes": (_sz, [_i32] * 4),
    "graft_matrix_update": (_i32, [_vp, _vp, _vp, _i32, _i32, _i32, _vp, _i32, _vp, _vp, _sz, _vp]),
    "graft_kv_compact": (_i32, [_vp, _vp, _i64, _i32, _i64, _i64, _i64, _vp, _i32, _vp, _vp, _vp,
                                _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp]),
}
EXPORTED_SYMBOLS = tuple(_SIGNATURES)

_lib = None


class GraftError(RuntimeError):
    def __init__(self, fn: str, code: int, hip: int = 0):
        self.code = code
        msg = "%s returned %s" % (fn, _ERR_NAMES.get(code, str(code)))
        if code == GRAFT_ERR_HIP:
            msg += " (hipError_t %d)" % hip
        super().__init__(msg)


def load_library():
    """dlopen libgraft.so and declare its signatures.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_2605_20104_amd.build` "
                "(there is no fallback path)" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            f = getattr(lib, name)
            f.restype, f.argtypes = res, args
        _lib = lib
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors cross the C ABI as dense row-major arrays"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(fn: str, rc: int):
    if rc != GRAFT_OK:
        raise GraftError(fn, rc, load_library().graft_last_hip_error())


def graft_retrieve(ctx, ctx_len, n_min: int, n_max: int, C: int, m: int, tail=None, tail_len=None,
                   out=None, stream=None):
    """Ranked continuation chains of the suffix n-gram.  ctx int32 [B,L_max] on the GPU.

    Returns a dict of device tensors: chain_tok [B,C,m], chain_len, chain_pos,
    chain_match [B,C], n_hits [B], status [B].  `out` may carry preallocated ones.
    """
    B, L_max = ctx.shape
    dev = ctx.device
    if out is None:
        out = {
            "chain_tok": torch.empty((B, C, m), dtype=torch.int32, device=dev),
            "chain_len": torch.empty((B, C), dtype=torch.int32, device=dev),
            "chain_pos": torch.empty((B, C), dtype=torch.int32, device=dev),
            "chain_match": torch.empty((B, C), dtype=torch.int32, device=dev),
            "n_hits": torch.empty(B, dtype=torch.int32, device=dev),
            "status": torch.empty(B, dtype=torch.int32, device=dev),
        }
    tail_max = 0 if tail is None else tail.shape[1]
    rc = load_library().graft_retrieve(
        _ptr(ctx), _ptr(ctx_len), B, L_max, _ptr(tail), _ptr(tail_len), tail_max, n_min, n_max, C, m,
        _ptr(out["chain_tok"]), _ptr(out["chain_len"]), _ptr(out["chain_pos"]), _ptr(out["chain_match"]),
        _ptr(out["n_hits"]), _ptr(out["status"]), _stream(stream))
    _check("graft_retrieve", rc)
    return out


def graft_build_tree_mask(parent, n_nodes, prefix_len, n_leaf_max: int = 0, depth_cap: int = 0,
                          out=None, stream=None):
    """Ancestor masks [B,K,2] (int64 storage of the uint64 words), pos, depth, optional leaf paths."""
    B, K_max = parent.shape
    dev = parent.device
    if out is None:
        out = {
            "mask": torch.empty((B, K_max, GRAFT_MASK_WORDS), dtype=torch.int64, device=dev),
            "pos": torch.empty((B, K_max), dtype=torch.int32, device=dev),
            "depth": torch.empty((B, K_max), dtype=torch.int32, device=dev),
            "paths": (torch.empty((B, n_leaf_max, depth_cap + 1), dtype=torch.int32, device=dev)
                      if n_leaf_max > 0 else None),
            "status": torch.empty(B, dtype=torch.int32, device=dev),
        }
    rc = load_library().graft_build_tree_mask(
        _ptr(parent), _ptr(n_nodes), _ptr(prefix_len), B, K_max, _ptr(out["mask"]), _ptr(out["pos"]),
        _ptr(out["depth"]), _ptr(out["paths"]), n_leaf_max, depth_cap, _ptr(out["status"]), _stream(stream))
    _check("graft_build_tree_mask", rc)
    return out


def graft_tree_attn_workspace_bytes(B: int, K_max: int, Hq: int, Hkv: int, D: int, max_pages: int,
                                    dtype: int) -> int:
    return int(load_library().graft_tree_attn_workspace_bytes(B, K_max, Hq, Hkv, D, max_pages, dtype))


def graft_tree_attn(q, k_cache, v_cache, strides, block_table, prefix_len, n_nodes, mask, Hkv: int,
                    scale: float, out=None, workspace=None, stream=None):
    """Tree-masked GQA attention, one layer.  q [B,K,Hq,D] float32 or bfloat16 on the GPU.

    strides: dict with 'page', 'token', 'head' in elements.  workspace: uint8 device
    tensor of at least graft_tree_attn_workspace_bytes(...) bytes (allocated if None).
    """
    B, K_max, Hq, D = q.shape
    dtype = GRAFT_F32 if q.dtype == torch.float32 else GRAFT_BF16
    assert q.dtype in (torch.float32, torch.bfloat16) and k_cache.dtype == q.dtype and v_cache.dtype == q.dtype
    max_pages = block_table.shape[1]
    if out is None:
        out = torch.empty_like(q)
    need = graft_tree_attn_workspace_bytes(B, K_max, Hq, Hkv, D, max_pages, dtype)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    rc = load_library().graft_tree_attn(
        _ptr(q), _ptr(k_cache), _ptr(v_cache), int(strides["page"]), int(strides["token"]),
        int(strides["head"]), _ptr(block_table), max_pages, _ptr(prefix_len), _ptr(n_nodes), _ptr(mask),
        B, K_max, Hq, Hkv, D, GRAFT_PAGE_SIZE, float(scale), dtype, _ptr(out),
        _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream))
    _check("graft_tree_attn", rc)
    return out


def graft_accept_workspace_bytes(B: int, K_max: int, V: int) -> int:
    return int(load_library().graft_accept_workspace_bytes(B, K_max, V))


def graft_accept(parent, tokens, n_nodes, depth_cap: int, target_ids=None, logits=None, out=None,
                 workspace=None, stream=None):
    """Greedy acceptance walk.  Give target_ids int32 [B,K] or logits float32 [B,K,V] (then
    the argmax per node is returned in out['target_ids'])."""
    B, K_max = parent.shape
    dev = parent.device
    V = 0
    if logits is not None:
        V = logits.shape[2]
        target_ids = torch.empty((B, K_max), dtype=torch.int32, device=dev)
        need = graft_accept_workspace_bytes(B, K_max, V)
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    if out is None:
        out = {
            "accept_len": torch.empty(B, dtype=torch.int32, device=dev),
            "best_node": torch.empty(B, dtype=torch.int32, device=dev),
            "path": torch.empty((B, depth_cap + 1), dtype=torch.int32, device=dev),
            "out_tokens": torch.empty((B, depth_cap + 1), dtype=torch.int32, device=dev),
            "status": torch.empty(B, dtype=torch.int32, device=dev),
        }
    out["target_ids"] = target_ids
    rc = load_library().graft_accept(
        _ptr(parent), _ptr(tokens), _ptr(n_nodes), _ptr(logits), V, _ptr(target_ids), B, K_max, depth_cap,
        _ptr(out["accept_len"]), _ptr(out["best_node"]), _ptr(out["path"]), _ptr(out["out_tokens"]),
        _ptr(out["status"]), _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream))
    _check("graft_accept", rc)
    return out


def graft_accept_noalloc(parent, tokens, n_nodes, depth_cap: int, out, target_ids, logits=None, stream=None):
    """graft_accept without a workspace and without any allocation, here or in the library: every
    output tensor is the caller's (out: accept_len, best_node, path, out_tokens, status; target_ids
    is an input in target_ids mode and an output in logits mode)."""
    B, K_max = parent.shape
    V = 0 if logits is None else logits.shape[2]
    rc = load_library().graft_accept_noalloc(
        _ptr(parent), _ptr(tokens), _ptr(n_nodes), _ptr(logits), V, _ptr(target_ids), B, K_max, depth_cap,
        _ptr(out["accept_len"]), _ptr(out["best_node"]), _ptr(out["path"]), _ptr(out["out_tokens"]),
        _ptr(out["status"]), _stream(stream))
    _check("graft_accept_noalloc", rc)
    return out


def graft_matrix_retrieve(M, tpl_parent, tpl_rank, n_ret, tokens, parent, n_nodes, status=None, stream=None):
    """Fills the first n_ret[b] template nodes by lookups in M [V,k] and appends them to the tree
    (tokens, parent [B,K_max] and n_nodes [B] are updated in place).  Returns status [B]."""
    V, k = M.shape
    B, K_max = tokens.shape
    if status is None:
        status = torch.empty(B, dtype=torch.int32, device=tokens.device)
    rc = load_library().graft_matrix_retrieve(
        _ptr(M), V, k, _ptr(tpl_parent), _ptr(tpl_rank), tpl_parent.shape[0], _ptr(n_ret), B, K_max,
        _ptr(tokens), _ptr(parent), _ptr(n_nodes), _ptr(status), _stream(stream))
    _check("graft_matrix_retrieve", rc)
    return status


def graft_matrix_update_workspace_bytes(B: int, K_max: int, V: int, k: int) -> int:
    return int(load_library().graft_matrix_update_workspace_bytes(B, K_max, V, k))


def graft_matrix_update(tokens, n_nodes, logits, M, target_ids=None, workspace=None, stream=None):
    """M[tokens[b,i]] <- ids of the k largest logits of node i (M [V,k] updated in place).
    Returns target_ids [B,K_max] (the greedy token per node)."""
    B, K_max, V = logits.shape
    k = M.shape[1]
    if target_ids is None:
        target_ids = torch.empty((B, K_max), dtype=torch.int32, device=logits.device)
    if workspace is None:
        workspace = torch.empty(max(graft_matrix_update_workspace_bytes(B, K_max, V, k), 8), dtype=torch.uint8,
                                device=logits.device)
    rc = load_library().graft_matrix_update(
        _ptr(tokens), _ptr(n_nodes), _ptr(logits), V, B, K_max, _ptr(M), k, _ptr(target_ids),
        _ptr(workspace), workspace.numel(), _stream(stream))
    _check("graft_matrix_update", rc)
    return target_ids


def graft_kv_compact(k_cache, v_cache, layer_stride: int, n_layers: int, strides, block_table, prefix_len,
                     path, accept_len, K_max: int, Hkv: int, D: int, out=None, stream=None):
    """Moves the accepted path's keys/values behind the prefix in place (all n_layers layers).
    Returns dict(new_prefix_len [B], status [B])."""
    B, width = path.shape
    dtype = GRAFT_F32 if k_cache.dtype == torch.float32 else GRAFT_BF16
    assert k_cache.dtype in (torch.float32, torch.bfloat16) and v_cache.dtype == k_cache.dtype
    if out is None:
        out = {"new_prefix_len": torch.empty(B, dtype=torch.int32, device=path.device),
               "status": torch.empty(B, dtype=torch.int32, device=path.device)}
    rc = load_library().graft_kv_compact(
        _ptr(k_cache), _ptr(v_cache), int(layer_stride), n_layers, int(strides["page"]), int(strides["token"]),
        int(strides["head"]), _ptr(block_table), block_table.shape[1], _ptr(prefix_len), _ptr(path),
        _ptr(accept_len), B, width - 1, K_max, Hkv, D, dtype, _ptr(out["new_prefix_len"]), _ptr(out["status"]),
        _stream(stream))
    _check("graft_kv_compact", rc)
    return out


def graft_prune_select(parent, tokens, logq, n_nodes, chk_depth, chk_log_tau, chk_keep, chk_ret, out=None,
                       stream=None):
    """Confidence gates + selection of the retained draft nodes.  Returns a dict of device tensors:
    parent, tokens, index [B,K_max], n_nodes, stage, n_ret, status [B]."""
    B, K_max = parent.shape
    dev = parent.device
    if out is None:
        out = {k: torch.empty((B, K_max), dtype=torch.int32, device=dev) for k in ("parent", "tokens", "index")}
        out.update({k: torch.empty(B, dtype=torch.int32, device=dev) for k in ("n_nodes", "stage", "n_ret", "status")})
    rc = load_library().graft_prune_select(
        _ptr(parent), _ptr(tokens), _ptr(logq), _ptr(n_nodes), B, K_max, _ptr(chk_depth), _ptr(chk_log_tau),
        _ptr(chk_keep), _ptr(chk_ret), chk_depth.shape[0], _ptr(out["parent"]), _ptr(out["tokens"]),
        _ptr(out["index"]), _ptr(out["n_nodes"]), _ptr(out["stage"]), _ptr(out["n_ret"]), _ptr(out["status"]),
        _stream(stream))
    _check("graft_prune_select", rc)
    return out
