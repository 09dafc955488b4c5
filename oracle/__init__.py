"""ctypes front end of the CPU oracle (oracle/graft_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  It imports nothing from the GPU package and the
GPU package imports nothing from here.  Arguments and results are numpy arrays
on the host; bf16 tensors travel as uint16 storage bits.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "graft_oracle.c")
_SO = os.path.join(_HERE, "libgraft_oracle.so")

ST_BAD_LENGTH, ST_BAD_TREE, ST_PATH_OVERFLOW = 1, 2, 4
MASK_WORDS = 2
_lib = None


_SO_SAN = os.path.join(_HERE, "libgraft_oracle_san.so")
SANITIZE_ENV = "GRAFT_ORACLE_SANITIZE"       # set to 1: the tests run against the sanitized build


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math).

    sanitize=True builds a second library with AddressSanitizer and UndefinedBehaviorSanitizer
    (every report is fatal).  A process can only load it when the AddressSanitizer runtime was
    loaded first (see sanitizer_env()).
    """
    so = _SO_SAN if sanitize else _SO
    if force or not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(_SRC):
        tmp = so + ".tmp%d" % os.getpid()
        flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                 "-fno-omit-frame-pointer"] if sanitize else ["-O2"]
        subprocess.check_call(["gcc", *flags, "-std=c11", "-fopenmp", "-shared", "-fPIC",
                               "-Wall", "-Wextra", _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, so)
    return so


def sanitizer_env(env=None) -> dict:
    """Environment for a child process that is to load the sanitized build: the switch that makes
    this module pick it, and the AddressSanitizer runtime in front of whatever is preloaded already."""
    env = dict(os.environ if env is None else env)
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    env[SANITIZE_ENV] = "1"
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"      # the interpreter's own leaks are not the subject
    return env


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build(sanitize=os.environ.get(SANITIZE_ENV) == "1"))
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def retrieve(ctx, ctx_len, n_min: int, n_max: int, C: int, m: int, tail=None, tail_len=None):
    """Ranked continuation chains of the suffix n-gram (see oracle_retrieve)."""
    ctx = _i32(ctx)
    B, L_max = ctx.shape
    ctx_len = _i32(ctx_len)
    if tail is not None:
        tail, tail_len = _i32(tail), _i32(tail_len)
        tail_max = tail.shape[1]
    else:
        tail_max = 0
    out = {
        "chain_tok": np.zeros((B, C, m), np.int32), "chain_len": np.zeros((B, C), np.int32),
        "chain_pos": np.zeros((B, C), np.int32), "chain_match": np.zeros((B, C), np.int32),
        "n_hits": np.zeros(B, np.int32), "status": np.zeros(B, np.int32),
    }
    _load().oracle_retrieve(_p(ctx), _p(ctx_len), B, L_max, _p(tail), _p(tail_len), tail_max,
                            n_min, n_max, C, m, _p(out["chain_tok"]), _p(out["chain_len"]),
                            _p(out["chain_pos"]), _p(out["chain_match"]), _p(out["n_hits"]),
                            _p(out["status"]))
    return out


def build_tree_mask(parent, n_nodes, prefix_len, n_leaf_max: int = 0, depth_cap: int = 0):
    """Ancestor bitmasks, depths, positions and optional root-to-leaf path table."""
    parent = _i32(parent)
    B, K_max = parent.shape
    n_nodes, prefix_len = _i32(n_nodes), _i32(prefix_len)
    out = {
        "mask": np.zeros((B, K_max, MASK_WORDS), np.uint64), "pos": np.zeros((B, K_max), np.int32),
        "depth": np.zeros((B, K_max), np.int32), "status": np.zeros(B, np.int32),
        "paths": (np.zeros((B, n_leaf_max, depth_cap + 1), np.int32) if n_leaf_max > 0 else None),
    }
    _load().oracle_build_tree_mask(_p(parent), _p(n_nodes), _p(prefix_len), B, K_max,
                                   _p(out["mask"]), _p(out["pos"]), _p(out["depth"]),
                                   _p(out["paths"]), n_leaf_max, depth_cap, _p(out["status"]))
    return out


def tree_attn(q, k_cache, v_cache, dtype: str, strides, block_table, prefix_len, n_nodes, parent,
              Hq: int, Hkv: int, D: int, page_size: int, scale: float, rows=None) -> np.ndarray:
    """Per-path causal attention for every (sequence, node, head) or for the listed rows.

    q: [B,K,Hq,D]; caches: any array whose flat element order matches `strides`
    (dict with 'page', 'token', 'head' in elements); dtype 'f32' (float32
    arrays) or 'bf16' (uint16 storage bits).  Returns float64 [B,K,Hq,D], or
    [n_rows,D] when rows (int32 [n_rows,3] of (b,i,h)) is given.
    """
    want = np.float32 if dtype == "f32" else np.uint16
    q, k_cache, v_cache = (np.ascontiguousarray(a, dtype=want) for a in (q, k_cache, v_cache))
    parent = _i32(parent)
    B, K_max = parent.shape
    block_table = _i32(block_table)
    prefix_len, n_nodes = _i32(prefix_len), _i32(n_nodes)
    if rows is None:
        out = np.zeros((B, K_max, Hq, D), np.float64)
        n_rows = 0
    else:
        rows = _i32(rows).reshape(-1, 3)
        n_rows = rows.shape[0]
        out = np.zeros((n_rows, D), np.float64)
    f = _load().oracle_tree_attn
    f.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int32] + [ctypes.c_int64] * 3 + \
                 [ctypes.c_void_p, ctypes.c_int32] + [ctypes.c_void_p] * 3 + [ctypes.c_int32] * 6 + \
                 [ctypes.c_double, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    f(_p(q), _p(k_cache), _p(v_cache), 0 if dtype == "f32" else 1,
      int(strides["page"]), int(strides["token"]), int(strides["head"]),
      _p(block_table), block_table.shape[1], _p(prefix_len), _p(n_nodes), _p(parent),
      B, K_max, Hq, Hkv, D, page_size, float(scale), _p(rows), n_rows, _p(out))
    return out


def accept(parent, tokens, n_nodes, depth_cap: int, target_ids=None, logits=None):
    """Greedy acceptance walk (see oracle_accept).  Give target_ids or fp32 logits [B,K,V]."""
    parent, tokens, n_nodes = _i32(parent), _i32(tokens), _i32(n_nodes)
    B, K_max = parent.shape
    if logits is not None:
        logits = np.ascontiguousarray(logits, dtype=np.float32)
        V = logits.shape[2]
        tids = np.full((B, K_max), -1, np.int32)
    else:
        V = 0
        tids = _i32(target_ids).copy()
    out = {
        "accept_len": np.zeros(B, np.int32), "best_node": np.zeros(B, np.int32),
        "path": np.zeros((B, depth_cap + 1), np.int32), "out_tokens": np.zeros((B, depth_cap + 1), np.int32),
        "status": np.zeros(B, np.int32), "target_ids": tids,
    }
    _load().oracle_accept(_p(parent), _p(tokens), _p(n_nodes), _p(logits), V, _p(tids), B, K_max,
                          depth_cap, _p(out["accept_len"]), _p(out["best_node"]), _p(out["path"]),
                          _p(out["out_tokens"]), _p(out["status"]))
    return out


def matrix_retrieve(M, tpl_parent, tpl_rank, n_ret, tokens, parent, n_nodes):
    """Template fill by matrix lookups, appended to the draft nodes (see oracle_matrix_retrieve).

    Returns copies: tokens, parent [B,K_max], n_nodes [B], status [B].
    """
    M = _i32(M)
    V, k = M.shape
    tpl_parent, tpl_rank = _i32(tpl_parent), _i32(tpl_rank)
    tokens, parent, n_nodes, n_ret = _i32(tokens).copy(), _i32(parent).copy(), _i32(n_nodes).copy(), _i32(n_ret)
    B, K_max = tokens.shape
    status = np.zeros(B, np.int32)
    _load().oracle_matrix_retrieve(_p(M), V, k, _p(tpl_parent), _p(tpl_rank), tpl_parent.shape[0], _p(n_ret),
                                   B, K_max, _p(tokens), _p(parent), _p(n_nodes), _p(status))
    return {"tokens": tokens, "parent": parent, "n_nodes": n_nodes, "status": status}


def matrix_update(M, tokens, n_nodes, logits):
    """M[x_i] <- ids of the k largest logits of node i (see oracle_matrix_update).  Returns M', target_ids."""
    M = _i32(M).copy()
    V, k = M.shape
    tokens, n_nodes = _i32(tokens), _i32(n_nodes)
    B, K_max = tokens.shape
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    assert logits.shape == (B, K_max, V)
    tids = np.zeros((B, K_max), np.int32)
    _load().oracle_matrix_update(_p(tokens), _p(n_nodes), _p(logits), V, B, K_max, _p(M), k, _p(tids))
    return {"M": M, "target_ids": tids}


def kv_compact(k_cache, v_cache, dtype: str, layer_stride: int, n_layers: int, strides, block_table,
               prefix_len, path, accept_len, K_max: int, Hkv: int, D: int, page_size: int = 16):
    """Moves the accepted path's keys/values behind the prefix (see oracle_kv_compact).

    Caches: flat arrays (float32, or uint16 storage bits for 'bf16'); copies are returned.
    """
    want = np.float32 if dtype == "f32" else np.uint16
    k_cache, v_cache = (np.ascontiguousarray(a, dtype=want).copy() for a in (k_cache, v_cache))
    block_table, prefix_len, path, accept_len = _i32(block_table), _i32(prefix_len), _i32(path), _i32(accept_len)
    B, width = path.shape
    new_len, status = np.zeros(B, np.int32), np.zeros(B, np.int32)
    f = _load().oracle_kv_compact
    f.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                  ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int32] * 5 + [ctypes.c_void_p] * 2
    f(_p(k_cache), _p(v_cache), 0 if dtype == "f32" else 1, int(layer_stride), n_layers,
      int(strides["page"]), int(strides["token"]), int(strides["head"]), _p(block_table), block_table.shape[1],
      page_size, _p(prefix_len), _p(path), _p(accept_len), B, width - 1, K_max, Hkv, D, _p(new_len), _p(status))
    return {"k_cache": k_cache, "v_cache": v_cache, "new_prefix_len": new_len, "status": status}


def prune_select(parent, tokens, logq, n_nodes, chk_depth, chk_log_tau, chk_keep, chk_ret):
    """Confidence gates + top-K_draft selection on a finished draft tree (see oracle_prune_select)."""
    parent, tokens, n_nodes = _i32(parent), _i32(tokens), _i32(n_nodes)
    logq = np.ascontiguousarray(logq, dtype=np.float32)
    chk_depth, chk_keep, chk_ret = _i32(chk_depth), _i32(chk_keep), _i32(chk_ret)
    chk_log_tau = np.ascontiguousarray(chk_log_tau, dtype=np.float32)
    B, K_max = parent.shape
    out = {"parent": np.zeros((B, K_max), np.int32), "tokens": np.zeros((B, K_max), np.int32),
           "index": np.zeros((B, K_max), np.int32), "n_nodes": np.zeros(B, np.int32),
           "stage": np.zeros(B, np.int32), "n_ret": np.zeros(B, np.int32), "status": np.zeros(B, np.int32)}
    _load().oracle_prune_select(_p(parent), _p(tokens), _p(logq), _p(n_nodes), B, K_max, _p(chk_depth),
                                _p(chk_log_tau), _p(chk_keep), _p(chk_ret), chk_depth.shape[0],
                                _p(out["parent"]), _p(out["tokens"]), _p(out["index"]), _p(out["n_nodes"]),
                                _p(out["stage"]), _p(out["n_ret"]), _p(out["status"]))
    return out
