"""GPU parity: graft_tree_attn vs the CPU oracle (MI355X only).

Tolerances: bf16 storage with fp32 accumulation must be within 2e-2 max-abs of the
fp64 oracle (outputs compared in fp32); the fp32 path within 1e-4.  The 2e-2 holds for inputs
like the workloads' (N(0,1) operands: scaled scores of unit size).  The bf16 path rounds the
pre-scaled query q * scale * log2(e) to bf16 once, a relative 2^-9 per element on top of the
bf16 storage of q; the noise this puts on a score, and with it on a softmax weight, grows in
proportion to the size of the scores.  A test that multiplies the scores by s on purpose
therefore allows s times the tolerance for the largest error (and checks the rms error
against the plain tolerance): score_scale_tolerance().
"""
import dataclasses
import math

import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2605_20104_amd as graft
from gpu_util import dev, host, run_attn

pytestmark = pytest.mark.gpu
TOL_BF16 = 2e-2
TOL_F32 = 1e-4


def score_scale_tolerance(got, ref, s_rms, what):
    """Largest error within TOL_BF16 * max(1, s_rms), s_rms = the rms size of the scaled scores (1 for
    the workloads' inputs); rms error within TOL_BF16 / 4.  Prints what was measured."""
    err = np.abs(got.astype(np.float64) - np.asarray(ref, np.float64))
    rms = float(np.sqrt((err ** 2).mean()))
    print("%s: max abs err %.3e, rms err %.3e, largest |ref| %.2f, score rms %.2f"
          % (what, err.max(), rms, np.abs(ref).max(), s_rms))
    assert err.max() <= TOL_BF16 * max(1.0, s_rms) and rms <= TOL_BF16 / 4


def gpu_mask(parent, n_nodes, prefix):
    out = graft.graft_build_tree_mask(dev(parent), dev(n_nodes), dev(prefix))
    return out["mask"]


def shape_workload(B, K, Hq, Hkv, D, P, dtype="bf16"):
    base = inputs.get_workload("c2")
    return dataclasses.replace(base, name="t", index=9, B=B, K=K, Hq=Hq, Hkv=Hkv, D=D, P=P, dtype=dtype,
                               distinct_kv_layers=1)


def check_case(w, seed, layout="head_major", n_nodes=None, prefix=None, tol=TOL_BF16, max_depth=8,
               rows=None):
    rng = np.random.default_rng(seed)
    att = inputs.make_attention_inputs(w, seed=seed, layout=layout)
    parent = np.stack([inputs.random_recursive_tree(rng, w.K, max_depth) for _ in range(w.B)])
    n_nodes = np.full(w.B, w.K, np.int32) if n_nodes is None else np.asarray(n_nodes, np.int32)
    prefix = np.full(w.B, w.P, np.int32) if prefix is None else np.asarray(prefix, np.int32)
    mask = gpu_mask(parent, n_nodes, prefix)
    got = run_attn(att, w.dtype, prefix, n_nodes, mask, w.Hkv)
    ref = oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], w.dtype, att["strides"],
                           att["block_table"], prefix, n_nodes, parent, w.Hq, w.Hkv, w.D, w.page_size,
                           att["scale"], rows=rows)
    if rows is None:
        err = np.abs(got - ref.astype(np.float32)).max()
    else:
        sel = np.stack([got[b, i, h] for b, i, h in rows])
        err = np.abs(sel - ref.astype(np.float32)).max()
    assert np.isfinite(got).all()
    assert err <= tol, "max abs err %.3e > %.1e" % (err, tol)
    return got, ref, err


def test_c1_fp32_full():
    w = inputs.get_workload("c1")
    s = inputs.make_step_inputs(w)
    att = inputs.make_attention_inputs(w)
    mask = gpu_mask(s["parent"], s["n_nodes"], s["prefix_len"])
    got = run_attn(att, "f32", s["prefix_len"], s["n_nodes"], mask, w.Hkv)
    ref = oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], "f32", att["strides"],
                           att["block_table"], s["prefix_len"], s["n_nodes"], s["parent"], w.Hq, w.Hkv, w.D,
                           w.page_size, att["scale"])
    assert np.abs(got - ref.astype(np.float32)).max() <= TOL_F32


# (B, K, Hq, Hkv, P): chosen to hit every (row blocks per wavefront) variant of the MFMA kernel,
# both mask words, ragged prefixes (not a multiple of 16, 32 or 64), and several KV splits.
MFMA_CASES = [
    (1, 1, 1, 1, 0),          # a lone root, empty prefix
    (1, 1, 8, 8, 5),
    (2, 16, 8, 2, 333),       # R = 64
    (1, 40, 32, 8, 1000),     # R = 160 (config 2 shape, shorter prefix)
    (1, 64, 40, 8, 777),      # R = 320 (config 3 shape): 3 + 2 row blocks
    (2, 48, 32, 2, 300),      # R = 768 (config 4 group size 16): two row tiles
    (1, 96, 8, 2, 1201),      # R = 384 (config 5 shape)
    (1, 128, 4, 2, 130),      # K = 128: both mask words
    (3, 33, 6, 2, 64),        # odd sizes, prefix exactly one stage
    (1, 20, 16, 16, 31),      # group size 1
    (1, 128, 32, 2, 100),     # R = 2048: the largest row count, seven row tiles
    (16, 8, 16, 8, 95),       # many sequences, few rows: one workgroup per (sequence, head)
    (1, 64, 40, 8, 20000),    # R = 320 with five row blocks per wavefront and more than 16 splits, every row
]


@pytest.mark.parametrize("case", MFMA_CASES, ids=lambda c: "B%d_K%d_Hq%d_Hkv%d_P%d" % c)
def test_bf16_mfma_shapes(case):
    B, K, Hq, Hkv, P = case
    w = shape_workload(B, K, Hq, Hkv, 128, P)
    check_case(w, seed=1000 + K + P)


def test_bf16_ragged_batch_and_padding_nodes():
    w = shape_workload(4, 48, 16, 4, 128, 500)
    n_nodes = [48, 1, 17, 33]
    prefix = [500, 0, 123, 17]
    got, _, _ = check_case(w, seed=5, n_nodes=n_nodes, prefix=prefix)
    for b, n in enumerate(n_nodes):
        assert (got[b, n:] == 0).all()                  # padding rows are zeros


def test_bf16_capacity_far_beyond_the_length():
    """The launch is planned from the block table's capacity: with a table for 64K tokens and a few hundred
    actual ones most splits have nothing to do and must contribute nothing."""
    w = shape_workload(2, 40, 16, 4, 128, 300)
    rng = np.random.default_rng(21)
    att = inputs.make_attention_inputs(w, seed=21)
    table = att["block_table"]
    wide = np.zeros((w.B, 4096), np.int32)                      # unused entries point at page 0 (readable)
    wide[:, :table.shape[1]] = table
    att = dict(att, block_table=wide)
    parent = np.stack([inputs.random_recursive_tree(rng, w.K, 8) for _ in range(w.B)])
    n_nodes, prefix = np.array([40, 23], np.int32), np.array([300, 31], np.int32)
    got = run_attn(att, "bf16", prefix, n_nodes, gpu_mask(parent, n_nodes, prefix), w.Hkv)
    ref = oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], "bf16", att["strides"], wide, prefix,
                           n_nodes, parent, w.Hq, w.Hkv, w.D, 16, att["scale"])
    assert np.abs(got - ref.astype(np.float32)).max() <= TOL_BF16


@pytest.mark.parametrize("P,Hkv", [(40000, 2), (9000, 1), (2500, 4)])
def test_bf16_many_splits(P, Hkv):
    """A long prefix for a single sequence with few KV heads takes the most splits the plan allows
    (up to 64): the combine step then merges through several wavefronts per tile (more than 16
    splits), or through its 16-, 8- and 4-split variants.  Sampled rows against the oracle."""
    w = shape_workload(1, 16, 4 * Hkv, Hkv, 128, P)
    rng = np.random.default_rng(P)
    rows = [(0, int(rng.integers(w.K)), int(rng.integers(w.Hq))) for _ in range(24)]
    rows += [(0, 0, 0), (0, w.K - 1, w.Hq - 1)]
    check_case(w, seed=P, rows=rows)


def test_bf16_token_major_layout_and_deep_chain():
    w = shape_workload(2, 64, 8, 2, 128, 200)
    check_case(w, seed=6, layout="token_major", max_depth=63)


def test_bf16_invalid_tree_size_gives_zeros():
    w = shape_workload(2, 16, 8, 2, 128, 100)
    got, _, _ = check_case(w, seed=7, n_nodes=[0, 16])
    assert (got[0] == 0).all()


def test_bf16_head_dim_64_and_fp32_head_dim_128():
    check_case(shape_workload(2, 12, 8, 4, 64, 90), seed=8)
    check_case(shape_workload(1, 9, 4, 2, 128, 70, dtype="f32"), seed=9, tol=TOL_F32)
    check_case(shape_workload(2, 12, 8, 4, 64, 600, dtype="f32"), seed=10, tol=TOL_F32)


def test_mfma_matches_plain_kernel_on_gpu():
    """Cross-check of the two GPU paths: same bf16 inputs through the MFMA kernel and, widened to
    fp32, through the plain kernel."""
    w = shape_workload(1, 24, 8, 2, 128, 450)
    got, ref, _ = check_case(w, seed=11)
    att = inputs.make_attention_inputs(w, seed=11)
    wide = dict(att, q=[inputs.bf16_bits_to_f32(att["q"][0])],
                k_cache=[inputs.bf16_bits_to_f32(att["k_cache"][0])],
                v_cache=[inputs.bf16_bits_to_f32(att["v_cache"][0])])
    rng = np.random.default_rng(11)
    parent = np.stack([inputs.random_recursive_tree(rng, w.K, 8)])
    mask = gpu_mask(parent, [w.K], [w.P])
    plain = run_attn(wide, "f32", np.array([w.P], np.int32), np.array([w.K], np.int32), mask, w.Hkv)
    assert np.abs(plain - ref.astype(np.float32)).max() <= TOL_F32
    assert np.abs(plain - got).max() <= TOL_BF16


def test_large_scores_stay_finite():
    """Peaked softmax (large |q.k|): the lazy running max must not overflow."""
    w = shape_workload(1, 16, 8, 2, 128, 400)
    att = inputs.make_attention_inputs(w, seed=12)
    qf = inputs.bf16_bits_to_f32(att["q"][0]) * 6.0
    att["q"] = [inputs.f32_to_bf16_bits(qf)]
    rng = np.random.default_rng(12)
    parent = np.stack([inputs.random_recursive_tree(rng, w.K, 8)])
    mask = gpu_mask(parent, [w.K], [w.P])
    got = run_attn(att, "bf16", np.array([w.P], np.int32), np.array([w.K], np.int32), mask, w.Hkv)
    ref = oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], "bf16", att["strides"],
                           att["block_table"], [w.P], [w.K], parent, w.Hq, w.Hkv, w.D, 16, att["scale"])
    assert np.isfinite(got).all()
    s_rms = float(np.sqrt(w.D) * att["scale"] * 6.0)                # q and k are N(0,1), q times 6
    score_scale_tolerance(got, ref, s_rms, "peaked softmax")


def test_scores_that_outgrow_the_reference():
    """Scores rising steadily along the sequence (by far more than the lazy bound of the fast
    path) force the exact running-max fallback; falling scores must stay on the fast path.
    Both must match the oracle."""
    w = shape_workload(2, 24, 8, 2, 128, 700)
    att = inputs.make_attention_inputs(w, seed=13)
    pages = att["pages_per_seq"]
    k = inputs.bf16_bits_to_f32(att["k_cache"][0]).copy()
    q = inputs.bf16_bits_to_f32(att["q"][0]).copy()
    for b in range(w.B):
        for lp in range(pages):
            t = lp * 16 + np.arange(16)
            k[att["block_table"][b, lp]] = (t * 0.0153)[None, :, None]       # k_t = t * beta in every dim
    q[:] = 1.0
    q[:, :, 1::2, :] = -1.0                                                  # odd heads: falling scores
    q[:, :, 2, :] = 0.01                                                     # one nearly flat head
    att["k_cache"] = [inputs.f32_to_bf16_bits(k)]
    att["q"] = [inputs.f32_to_bf16_bits(q)]
    rng = np.random.default_rng(13)
    parent = np.stack([inputs.random_recursive_tree(rng, w.K, 8) for _ in range(w.B)])
    n_nodes = np.array([w.K, w.K], np.int32)
    prefix = np.array([w.P, 333], np.int32)
    mask = gpu_mask(parent, n_nodes, prefix)
    got = run_attn(att, "bf16", prefix, n_nodes, mask, w.Hkv)
    ref = oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], "bf16", att["strides"],
                           att["block_table"], prefix, n_nodes, parent, w.Hq, w.Hkv, w.D, 16, att["scale"])
    assert np.isfinite(got).all()
    err = np.abs(got - ref.astype(np.float32)).max()
    print("scores outgrow the reference: max abs err %.3e" % err)
    assert err <= TOL_BF16


@pytest.mark.parametrize("log2_scale", [-100, -20, 40, 100])
def test_value_magnitudes_across_the_bf16_range(log2_scale):
    """The splits' partial rows pass through memory as fp16 scaled per row by a power of two:
    values far outside the fp16 range (V multiplied by 2^-100 .. 2^100, exact in bf16) must come
    out as accurately as O(1) values, and so must dims whose magnitudes differ by 2^12 within a
    row (they stay inside fp16's normal range below the row maximum).  Many splits: a long
    prefix for a batch of one."""
    w = shape_workload(1, 24, 8, 2, 128, 6000)
    att = inputs.make_attention_inputs(w, seed=21)
    v = inputs.bf16_bits_to_f32(att["v_cache"][0]).astype(np.float64)
    spread = np.exp2(np.linspace(-6, 6, w.D).round())                       # per dim, exact powers of two
    v = v * spread * np.exp2(float(log2_scale))
    att["v_cache"] = [inputs.f32_to_bf16_bits(v.astype(np.float32))]
    rng = np.random.default_rng(21)
    parent = np.stack([inputs.random_recursive_tree(rng, w.K, 8)])
    mask = gpu_mask(parent, [w.K], [w.P])
    got = run_attn(att, "bf16", np.array([w.P], np.int32), np.array([w.K], np.int32), mask, w.Hkv)
    ref = oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], "bf16", att["strides"],
                           att["block_table"], [w.P], [w.K], parent, w.Hq, w.Hkv, w.D, 16, att["scale"])
    assert np.isfinite(got).all()
    # every dim's values share a magnitude: the error of a dim is taken relative to that dim's
    # largest output (what TOL_BF16 means for O(1) values)
    unit = np.abs(ref).max(axis=(0, 1, 2), keepdims=True)
    assert (unit > 0).all()
    err = (np.abs(got.astype(np.float64) - ref) / unit).max()
    assert err <= TOL_BF16, "max err relative to the dim's largest output %.3e" % err


def test_scores_that_outgrow_the_reference_in_long_splits():
    """The same rising and falling scores with many (sequence, head) units, so that every workgroup
    runs several stages: wavefronts leave the fast path in the middle of their split, at an even or
    an odd sub-tile, while transfers of later stages are still to be issued."""
    w = shape_workload(8, 16, 8, 8, 128, 1500)
    att = inputs.make_attention_inputs(w, seed=14)
    pages = att["pages_per_seq"]
    k = inputs.bf16_bits_to_f32(att["k_cache"][0]).copy()
    q = inputs.bf16_bits_to_f32(att["q"][0]).copy()
    prefix = np.array([1500, 1484, 1001, 777, 1500, 1203, 690, 1499], np.int32)
    for b in range(w.B):
        for lp in range(pages):
            t = lp * 16 + np.arange(16)
            # flat for a while, then rising: the reference is outgrown at a different place per sequence
            ramp = np.maximum(t - (100 + 97 * b), 0) * 0.0153
            k[att["block_table"][b, lp]] = ramp[None, :, None]
    q[:] = 1.0
    q[:, :, 1::2, :] = -1.0                                                  # odd heads: falling scores
    att["k_cache"] = [inputs.f32_to_bf16_bits(k)]
    att["q"] = [inputs.f32_to_bf16_bits(q)]
    rng = np.random.default_rng(14)
    parent = np.stack([inputs.random_recursive_tree(rng, w.K, 8) for _ in range(w.B)])
    n_nodes = np.full(w.B, w.K, np.int32)
    mask = gpu_mask(parent, n_nodes, prefix)
    got = run_attn(att, "bf16", prefix, n_nodes, mask, w.Hkv)
    ref = oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], "bf16", att["strides"],
                           att["block_table"], prefix, n_nodes, parent, w.Hq, w.Hkv, w.D, 16, att["scale"])
    assert np.isfinite(got).all()
    err = np.abs(got - ref.astype(np.float32)).max()
    print("scores outgrow the reference: max abs err %.3e" % err)
    assert err <= TOL_BF16


def test_c2_full_size_all_rows():
    w = inputs.get_workload("c2")
    s = inputs.make_step_inputs(w)
    att = inputs.make_attention_inputs(w, kv_buffers=1)
    mask = gpu_mask(s["parent"], s["n_nodes"], s["prefix_len"])
    got = run_attn(att, "bf16", s["prefix_len"], s["n_nodes"], mask, w.Hkv)
    ref = oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], "bf16", att["strides"],
                           att["block_table"], s["prefix_len"], s["n_nodes"], s["parent"], w.Hq, w.Hkv, w.D,
                           16, att["scale"])
    assert np.abs(got - ref.astype(np.float32)).max() <= TOL_BF16


@pytest.mark.parametrize("name", ["c3", "c4", "c5"])
def test_full_size_all_rows(name):
    """Full benchmark sizes in the benchmark's launch configuration, every (sequence, node, head) row
    against the oracle."""
    w = inputs.get_workload(name)
    s = inputs.make_step_inputs(w)
    att = inputs.make_attention_inputs(w, kv_buffers=1)
    mask = gpu_mask(s["parent"], s["n_nodes"], s["prefix_len"])
    got = run_attn(att, "bf16", s["prefix_len"], s["n_nodes"], mask, w.Hkv)
    ref = oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], "bf16", att["strides"],
                           att["block_table"], s["prefix_len"], s["n_nodes"], s["parent"], w.Hq, w.Hkv, w.D,
                           16, att["scale"])
    assert np.isfinite(got).all()
    err = np.abs(got - ref.astype(np.float32)).max()
    print("%s all %d rows: max abs err %.3e" % (name, w.B * w.K * w.Hq, err))
    assert err <= TOL_BF16


def _plan_splits(B, K, Hq, Hkv, max_pages):
    """Number of KV splits the library plans: read off the workspace size (272 bytes per partial row;
    one split needs no workspace)."""
    R = K * (Hq // Hkv)
    assert R <= 320
    r_pad = -(-R // 64) * 64
    ws = graft.graft_tree_attn_workspace_bytes(B, K, Hq, Hkv, 128, max_pages, graft.GRAFT_BF16)
    if ws == 0:
        return 1
    assert ws % (B * Hkv * r_pad * 272) == 0
    return ws // (B * Hkv * r_pad * 272)


def test_many_splits_agree_with_a_single_split():
    """The split-KV merge against a run that needs none: the same sequence alone (a batch of one is cut
    into many splits) and replicated 64 times (enough (sequence, head) units to fill the chip, so the
    plan takes one split).  Outputs may differ by the rounding of the partial results only (fp16 rows
    scaled to each split's own largest entry, which is larger than the merged row's) and by a final
    bf16 rounding that flips: within one bf16 unit in the last place of the row's largest entry."""
    w1 = shape_workload(1, 24, 16, 4, 128, 6000)
    att = inputs.make_attention_inputs(w1, seed=31)
    rng = np.random.default_rng(31)
    parent = np.stack([inputs.random_recursive_tree(rng, w1.K, 8)])
    n1, p1 = np.array([w1.K], np.int32), np.array([w1.P], np.int32)
    pages = att["block_table"].shape[1]
    assert _plan_splits(1, w1.K, w1.Hq, w1.Hkv, pages) >= 16
    one = run_attn(att, "bf16", p1, n1, gpu_mask(parent, n1, p1), w1.Hkv)
    B = 64
    assert _plan_splits(B, w1.K, w1.Hq, w1.Hkv, pages) == 1
    rep = dict(att, q=[np.repeat(att["q"][0], B, axis=0)], block_table=np.repeat(att["block_table"], B, axis=0))
    nB, pB = np.full(B, w1.K, np.int32), np.full(B, w1.P, np.int32)
    many = run_attn(rep, "bf16", pB, nB, gpu_mask(np.repeat(parent, B, axis=0), nB, pB), w1.Hkv)
    assert (many == many[0:1]).all()                           # every replica computes the same thing
    diff = np.abs(one[0].astype(np.float64) - many[0])
    ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(many[0]), 1e-30))) - 7)
    row_max = np.abs(many[0]).max(axis=-1, keepdims=True)
    print("split vs single: %d of %d entries differ, max %.3e" % (int((diff > 0).sum()), diff.size, diff.max()))
    row_ulp = np.exp2(np.floor(np.log2(row_max)) - 7)
    print("largest difference in units of the row's bf16 ulp: %.3f" % (diff / row_ulp).max())
    assert (diff <= np.maximum(ulp, row_ulp)).all()
    ref = oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], "bf16", att["strides"],
                           att["block_table"], p1, n1, parent, w1.Hq, w1.Hkv, w1.D, 16, att["scale"])
    assert np.abs(one - ref.astype(np.float32)).max() <= TOL_BF16 and np.abs(many[:1] - ref.astype(np.float32)).max() <= TOL_BF16


def test_timing_build_gives_the_same_rows_and_ordered_stamps():
    """The timing build (the kernel with time stamps, libgraft_timing.so) computes what the product
    library computes, bit for bit, with a plan of its own choice and with a held plan against the
    oracle; the stamps of every workgroup that ran are in order."""
    import ctypes
    from paper_2605_20104_amd import build
    import os
    if not os.path.exists(build.LIB_TIMING):
        pytest.skip("libgraft_timing.so is not built (python -m paper_2605_20104_amd.build --timing)")
    timing = ctypes.CDLL(build.LIB_TIMING)
    for name in ("graft_tree_attn", "graft_tree_attn_workspace_bytes"):
        f = getattr(timing, name)
        f.restype, f.argtypes = graft._SIGNATURES[name]
    timing.graft_attn_stamp_buffer.restype, timing.graft_attn_stamp_buffer.argtypes = ctypes.c_int32, [ctypes.c_void_p, ctypes.c_size_t]
    timing.graft_attn_force_plan.restype, timing.graft_attn_force_plan.argtypes = ctypes.c_int32, [ctypes.c_int32, ctypes.c_int32]
    n_stamps = timing.graft_attn_stamp_count()

    w = shape_workload(2, 40, 16, 4, 128, 3000)
    rng = np.random.default_rng(5)
    att = inputs.make_attention_inputs(w, seed=5)
    parent = np.stack([inputs.random_recursive_tree(rng, w.K, 8) for _ in range(w.B)])
    n_nodes, prefix = np.array([40, 33], np.int32), np.array([3000, 1777], np.int32)
    mask = gpu_mask(parent, n_nodes, prefix)
    q, k, v = (dev(att[x][0], "bf16") for x in ("q", "k_cache", "v_cache"))
    table, d_prefix, d_nodes = dev(att["block_table"]), dev(prefix), dev(n_nodes)
    product = graft.graft_tree_attn(q, k, v, att["strides"], table, d_prefix, d_nodes, mask, w.Hkv, att["scale"])

    def run_timing():
        shape = (w.B, w.K, w.Hq, w.Hkv, w.D, table.shape[1], graft.GRAFT_BF16)
        need = timing.graft_tree_attn_workspace_bytes(*shape)
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        stamps = torch.zeros(4096 * n_stamps, dtype=torch.int64, device="cuda")
        out = torch.empty_like(q)
        timing.graft_attn_stamp_buffer(stamps.data_ptr(), stamps.numel() * 8)
        rc = timing.graft_tree_attn(
            q.data_ptr(), k.data_ptr(), v.data_ptr(), int(att["strides"]["page"]), int(att["strides"]["token"]),
            int(att["strides"]["head"]), table.data_ptr(), table.shape[1], d_prefix.data_ptr(), d_nodes.data_ptr(),
            mask.data_ptr(), w.B, w.K, w.Hq, w.Hkv, w.D, graft.GRAFT_PAGE_SIZE, float(att["scale"]), graft.GRAFT_BF16,
            out.data_ptr(), ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        timing.graft_attn_stamp_buffer(None, 0)
        assert rc == 0
        st = stamps.cpu().numpy().reshape(4096, n_stamps)
        return out, st[st[:, 14] == 1]

    out, st = run_timing()
    assert torch.equal(out.view(torch.int16), product.view(torch.int16))
    assert len(st) > 0
    assert (np.diff(st[:, 1:11], axis=1) >= 0).all()          # the points of a workgroup's life, in order
    assert (st[:, 12] > st[:, 11]).all() and (st[:, 10] < 100000).all()   # cycles advance; under a millisecond

    timing.graft_attn_force_plan(3, 1)                         # three splits, all rows in one tile
    try:
        held, st_held = run_timing()
    finally:
        timing.graft_attn_force_plan(0, 0)
    assert len(st_held) == w.B * w.Hkv * 3
    ref = oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], w.dtype, att["strides"],
                           att["block_table"], prefix, n_nodes, parent, w.Hq, w.Hkv, w.D, w.page_size, att["scale"])
    err = np.abs(host(held).astype(np.float64) - np.asarray(ref, np.float64))
    assert err[0].max() <= TOL_BF16 and err[1, :33].max() <= TOL_BF16
