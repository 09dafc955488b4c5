"""Seeded synthetic inputs for the hybrid-tree verification hot path.

This package is shared by the CPU oracle's tests and by the GPU tests and
benchmark.  It holds data recipes only: random draws, planting of repeated
spans, tree topologies and storage layouts.  None of the method's arithmetic
(retrieval matching, ancestor masks, attention, acceptance) lives here, and it
imports neither the oracle nor the GPU package.

Stand-in statement: the paper evaluates on public benchmarks (Sec. 4
"Experimental setup": five short-context suites and five long-context
LongBench tasks).  Those are not reproduced; the workloads below only mimic
their sizes and structure (2K-class prompts, 4K-64K long prompts, locally
repeated spans, a 60-node verification budget split into retained draft nodes
and grafted retrieval nodes, Sec. 3.2 and App. A "Stage-adaptive budget").
"""
from .workloads import WORKLOADS, Workload, get_workload
from .generate import (
    BASE_SEED,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_attention_inputs,
    make_context,
    make_step_inputs,
    make_tree,
    random_recursive_tree,
    toy_target,
    toy_target_for_nodes,
)

__all__ = [
    "WORKLOADS", "Workload", "get_workload", "BASE_SEED",
    "bf16_bits_to_f32", "f32_to_bf16_bits", "make_attention_inputs",
    "make_context", "make_step_inputs", "make_tree", "random_recursive_tree",
    "toy_target", "toy_target_for_nodes",
]
