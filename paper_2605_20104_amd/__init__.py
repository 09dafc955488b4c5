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
