"""The five benchmark workloads, as plain data.

Shapes follow the models the paper evaluates (Table "Model configurations":
layers and vocabulary sizes; head counts are the public architectures') and
its tree budget (Sec. 3.2: a 60-node budget keeping 8 / 24 / 40 draft nodes
and giving the rest to retrieval).  `chains` lists the grafted pieces in
append order (App. A, Alg. 2: retrieved nodes are appended after the retained
draft nodes): ("ret", m) is a retrieved m-token continuation chain, ("block",
m) an m-token linear block in the style of the block-drafter demo (App. G).
"""
from dataclasses import dataclass
from typing import Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # 1-based config number, also the seed offset
    dtype: str            # "f32" or "bf16": storage type of Q, K, V and O
    B: int                # sequences
    layers: int           # attention launches per step
    Hq: int
    Hkv: int
    D: int
    P: int                # prefix tokens already in the KV cache (per sequence)
    K: int                # tree nodes per sequence, root included
    tree: str             # "recursive" | "dense" | "mixed"
    chains: Tuple[Tuple[str, int], ...]
    vocab: int
    L: int                # context token buffer length (per sequence)
    zipf_s: float         # 0 => uniform token draw
    n_spans: int          # planted repeated spans (besides the query n-gram)
    span_lo: int
    span_hi: int
    n_min: int
    n_max: int
    C: int                # chains returned by retrieval
    m: int                # tokens per retrieved chain
    page_size: int = 16
    distinct_kv_layers: int = 1   # KV buffers rotated over the layers

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def n_ret(self) -> int:
        return sum(1 for kind, _ in self.chains if kind == "ret")


WORKLOADS = {
    # Tiny fp32 check.
    "c1": Workload(name="c1", index=1, dtype="f32", B=1, layers=1, Hq=8, Hkv=2, D=64,
                   P=256, K=16, tree="recursive", chains=(("ret", 4),),
                   vocab=1000, L=256, zipf_s=0.0, n_spans=0, span_lo=0, span_hi=0,
                   n_min=4, n_max=4, C=1, m=4),
    # LLaMA3.1-8B-shaped short context: stage "prune after depth 1" keeps 24 draft nodes.
    "c2": Workload(name="c2", index=2, dtype="bf16", B=1, layers=32, Hq=32, Hkv=8, D=128,
                   P=2048, K=40, tree="dense", chains=(("ret", 8), ("ret", 8)),
                   vocab=128256, L=2048, zipf_s=1.1, n_spans=40, span_lo=8, span_hi=16,
                   n_min=2, n_max=8, C=2, m=8, distinct_kv_layers=32),
    # Qwen3-14B-shaped long context: stage "prune after depth 5" keeps 40 draft nodes.
    "c3": Workload(name="c3", index=3, dtype="bf16", B=1, layers=1, Hq=40, Hkv=8, D=128,
                   P=32768, K=64, tree="dense", chains=(("ret", 8),) * 3,
                   vocab=151936, L=32768, zipf_s=1.1, n_spans=200, span_lo=6, span_hi=24,
                   n_min=2, n_max=8, C=3, m=8),
    # Qwen3-235B-A22B-shaped, one GPU's share of heads, batch 8.
    "c4": Workload(name="c4", index=4, dtype="bf16", B=8, layers=94, Hq=64, Hkv=4, D=128,
                   P=4096, K=48, tree="mixed", chains=(("ret", 8),) * 3,
                   vocab=151936, L=4096, zipf_s=1.1, n_spans=30, span_lo=6, span_hi=24,
                   n_min=2, n_max=8, C=3, m=8, distinct_kv_layers=4),
    # LLaMA3.1-8B-shaped long context, batch 4, block-drafting style pieces.
    "c5": Workload(name="c5", index=5, dtype="bf16", B=4, layers=1, Hq=32, Hkv=8, D=128,
                   P=65536, K=96, tree="dense",
                   chains=(("block", 16),) * 3 + (("ret", 8),) * 2,
                   vocab=128256, L=65536, zipf_s=1.1, n_spans=500, span_lo=6, span_hi=24,
                   n_min=2, n_max=8, C=2, m=8),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name.lower()]
