#!/usr/bin/env python3
"""Benchmark of the hybrid-tree verification step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
    graft_retrieve -> graft_build_tree_mask -> layers x graft_tree_attn -> graft_accept
on one stream, inputs resident in HBM.  Prints ONE JSON line:
  metric / value : tree-verify attention algorithmic bytes per step divided by the whole
                   step's time (GB/s), plus us per step in extra keys;
  roofline       : the dominant kernel (the MFMA tree-attention kernel) timed with HIP
                   events that the library attaches to that kernel's dispatch;
  cpu_baseline   : the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 peak
MALL_BYTES = 256 << 20         # Infinity Cache: KV buffers are rotated to exceed it


class Hip:
    """The few HIP runtime calls the benchmark needs for its own event timing."""

    def __init__(self):
        self.lib = ctypes.CDLL("libamdhip64.so")
        self.lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.lib.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.lib.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.lib.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def event(self):
        e = ctypes.c_void_p()
        assert self.lib.hipEventCreate(ctypes.byref(e)) == 0
        return e

    def record(self, e, stream):
        assert self.lib.hipEventRecord(e, ctypes.c_void_p(stream)) == 0

    def elapsed_ms(self, a, b):
        assert self.lib.hipEventSynchronize(b) == 0
        ms = ctypes.c_float()
        assert self.lib.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        return float(ms.value)


def attention_bytes_and_flops(w):
    """Algorithmic traffic of one attention layer: K and V read once, Q read, O written, block table."""
    e = 2 if w.dtype == "bf16" else 4
    T = w.P + w.K
    kv = 2 * T * w.Hkv * w.D * e
    qo = 2 * w.K * w.Hq * w.D * e
    table = 4 * ((T + w.page_size - 1) // w.page_size)
    return w.B * (kv + qo + table), 4.0 * w.K * w.Hq * w.D * T * w.B


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--graph", action="store_true",
                    help="also replay the step from a captured HIP graph and report its time per step")
    ap.add_argument("--no-rotate", action="store_true",
                    help="reuse one KV buffer for every layer (Infinity-Cache-resident figure for small workloads)")
    ap.add_argument("--logits", action="store_true",
                    help="graft_accept takes fp32 logits [B,K,V] (argmax scan on the GPU) instead of target ids")
    ap.add_argument("--extended", action="store_true",
                    help="also time the steps around verification (matrix retrieval, matrix refresh from the "
                         "logits, cache update after acceptance) and report them in extra keys; the timed step "
                         "and the headline metric stay the same")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="default run only: do not time c5 and c2 after the c3 steps")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run five plain 1 GiB -> 1 GiB elementwise copies and exit: the reference that the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import inputs
    import paper_2605_20104_amd as graft

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    graft.load_library()                       # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = (1 << 30) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)       # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read_per_launch": n * 4,
                          "bytes_written_per_launch": n * 4, "launches": 5}))
        return
    steps = args.steps if args.steps is not None else {"c1": 200, "c2": 100, "c3": 100, "c4": 20, "c5": 30}[args.workload]
    warmup = args.warmup if args.warmup is not None else 10
    result = run_workload(args, args.workload, steps, warmup, light=False)
    if args.workload == "c3" and not args.no_other_workloads:
        # the largest and the short-context workload ride along with few steps (kernel time, roofline
        # fractions, step time), and a plain copy kernel gives the bandwidth this box really reaches
        result["practical_hbm_GBps"] = round(copy_bandwidth_GBps(), 1)
        result["other_workloads"] = {}
        for name, st in (("c5", 12), ("c2", 30)):
            r = run_workload(args, name, st, 3, light=True)
            result["other_workloads"][name] = {
                "workload": r["config"]["workload"], "steps": st, "us_per_step": r["us_per_step"],
                "kernel_avg_us": r["roofline"]["kernel_avg_us"], "frac": r["roofline"]["frac"],
                "achieved_GBps": r["roofline"]["achieved"], "mfma_frac": r["roofline"]["mfma_frac"],
                "attn_call_us": r["per_call_us"]["tree_attn_layer"],
            }
    print(json.dumps(result))


def copy_bandwidth_GBps():
    """Read + write rate of a plain elementwise copy of 1 GiB (torch's kernel), best of 5."""
    import torch
    n = (1 << 30) // 4
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    best = 0.0
    for _ in range(6):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        torch.mul(src, 1.0, out=dst)
        b.record()
        torch.cuda.synchronize()
        best = max(best, 2.0 * n * 4 / (a.elapsed_time(b) * 1e-3) / 1e9)
    del src, dst
    torch.cuda.empty_cache()
    return best


def run_workload(args, name, steps, warmup, light):
    """Times `steps` steps of workload `name`; light = no per-call extras, no CPU baseline."""
    import torch
    import inputs
    import paper_2605_20104_amd as graft
    hip = Hip()
    w = inputs.get_workload(name)
    att_bytes, att_flops = attention_bytes_and_flops(w)

    # ---- inputs -> HBM
    s = inputs.make_step_inputs(w, with_logits=args.logits)
    kv_bytes_one = att_bytes  # per layer
    n_kv = max(w.distinct_kv_layers, 1)
    while n_kv * kv_bytes_one < 2 * MALL_BYTES and n_kv < 64 and w.name != "c1" and not args.no_rotate:
        n_kv += 1                              # rotate buffers so that every launch streams from HBM
    att = inputs.make_attention_inputs(w, kv_buffers=n_kv, q_layers=min(w.layers, 4))
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32

    def up(a, kind="i32"):
        if kind == "store":
            if w.dtype == "bf16":
                return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
            return torch.from_numpy(a).cuda()
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()

    d = {k: up(s[k]) for k in ("ctx", "ctx_len", "tail", "tail_len", "parent", "tokens", "n_nodes",
                               "prefix_len", "target_ids")}
    q = [up(att["q"][l], "store") for l in range(att["q"].shape[0])]
    kc = [up(a, "store") for a in att["k_cache"]]
    vc = [up(a, "store") for a in att["v_cache"]]
    table = up(att["block_table"])
    B, K = w.B, w.K
    dev = "cuda"
    ret_out = {
        "chain_tok": torch.empty((B, w.C, w.m), dtype=torch.int32, device=dev),
        "chain_len": torch.empty((B, w.C), dtype=torch.int32, device=dev),
        "chain_pos": torch.empty((B, w.C), dtype=torch.int32, device=dev),
        "chain_match": torch.empty((B, w.C), dtype=torch.int32, device=dev),
        "n_hits": torch.empty(B, dtype=torch.int32, device=dev),
        "status": torch.empty(B, dtype=torch.int32, device=dev),
    }
    depth_cap = 48
    mask_out = {
        "mask": torch.empty((B, K, 2), dtype=torch.int64, device=dev),
        "pos": torch.empty((B, K), dtype=torch.int32, device=dev),
        "depth": torch.empty((B, K), dtype=torch.int32, device=dev),
        "paths": torch.empty((B, K, depth_cap + 1), dtype=torch.int32, device=dev),
        "status": torch.empty(B, dtype=torch.int32, device=dev),
    }
    acc_out = {
        "accept_len": torch.empty(B, dtype=torch.int32, device=dev),
        "best_node": torch.empty(B, dtype=torch.int32, device=dev),
        "path": torch.empty((B, depth_cap + 1), dtype=torch.int32, device=dev),
        "out_tokens": torch.empty((B, depth_cap + 1), dtype=torch.int32, device=dev),
        "status": torch.empty(B, dtype=torch.int32, device=dev),
    }
    o = torch.empty((B, K, w.Hq, w.D), dtype=tdt, device=dev)
    ws_bytes = graft.graft_tree_attn_workspace_bytes(B, K, w.Hq, w.Hkv, w.D, table.shape[1],
                                                     graft.GRAFT_BF16 if w.dtype == "bf16" else graft.GRAFT_F32)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    layer_counter = [0]
    logits = torch.from_numpy(s["logits"]).cuda() if args.logits else None
    acc_ws = (torch.empty(graft.graft_accept_workspace_bytes(B, K, w.vocab), dtype=torch.uint8, device=dev)
              if args.logits else None)
    ids_out = torch.empty((B, K), dtype=torch.int32, device=dev)

    def step():
        graft.graft_retrieve(d["ctx"], d["ctx_len"], w.n_min, w.n_max, w.C, w.m, d["tail"], d["tail_len"],
                             out=ret_out)
        graft.graft_build_tree_mask(d["parent"], d["n_nodes"], d["prefix_len"], K, depth_cap, out=mask_out)
        for l in range(w.layers):
            i = layer_counter[0]
            layer_counter[0] += 1
            graft.graft_tree_attn(q[l % len(q)], kc[i % n_kv], vc[i % n_kv], att["strides"], table,
                                  d["prefix_len"], d["n_nodes"], mask_out["mask"], w.Hkv, att["scale"],
                                  out=o, workspace=ws)
        accept()

    def accept():
        if args.logits:
            lib_.graft_accept(d["parent"].data_ptr(), d["tokens"].data_ptr(), d["n_nodes"].data_ptr(),
                              logits.data_ptr(), w.vocab, ids_out.data_ptr(), B, K, depth_cap,
                              acc_out["accept_len"].data_ptr(), acc_out["best_node"].data_ptr(),
                              acc_out["path"].data_ptr(), acc_out["out_tokens"].data_ptr(),
                              acc_out["status"].data_ptr(), acc_ws.data_ptr(), acc_ws.numel(),
                              torch.cuda.current_stream().cuda_stream)
        else:
            graft.graft_accept(d["parent"], d["tokens"], d["n_nodes"], depth_cap, target_ids=d["target_ids"],
                               out=acc_out)

    lib_ = graft.load_library()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps; the library attaches an event pair to the main
    #      attention kernel of its first n_ev attention calls
    n_ev = min(steps * w.layers, 64 if light else 256)      # attaching events costs host time per launch: bound it
    ev_a = (ctypes.c_void_p * n_ev)(*[hip.event() for _ in range(n_ev)])
    ev_b = (ctypes.c_void_p * n_ev)(*[hip.event() for _ in range(n_ev)])
    lib = graft.load_library()
    assert lib.graft_attn_profile_events(ev_a, ev_b, n_ev) == 0
    marks = [hip.event() for _ in range(steps + 1)]          # step boundaries (for the percentiles)
    torch.cuda.synchronize()
    hip.record(marks[0], stream)
    t0 = time.perf_counter()
    for i in range(steps):
        step()
        hip.record(marks[i + 1], stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    total_ms = hip.elapsed_ms(marks[0], marks[steps])
    step_us = np.array([hip.elapsed_ms(marks[i], marks[i + 1]) for i in range(steps)]) * 1e3
    lib.graft_attn_profile_events(None, None, 0)
    kern_ms = np.array([hip.elapsed_ms(ev_a[i], ev_b[i]) for i in range(n_ev)])
    ms_per_step = total_ms / steps
    kernel_avg_ms = float(kern_ms.mean())

    # ---- per-call timings (separate, untimed-region loop): median over a few repetitions
    def time_call(fn, reps=20):
        ts = []
        for _ in range(reps):
            a, b = hip.event(), hip.event()
            hip.record(a, stream)
            fn()
            hip.record(b, stream)
            ts.append(hip.elapsed_ms(a, b) * 1e3)
        return float(np.median(ts))

    per_call_us = {
        "retrieve": time_call(lambda: graft.graft_retrieve(d["ctx"], d["ctx_len"], w.n_min, w.n_max, w.C, w.m,
                                                            d["tail"], d["tail_len"], out=ret_out)),
        "build_tree_mask": time_call(lambda: graft.graft_build_tree_mask(
            d["parent"], d["n_nodes"], d["prefix_len"], K, depth_cap, out=mask_out)),
        "tree_attn_layer": time_call(lambda: graft.graft_tree_attn(
            q[0], kc[layer_counter[0] % n_kv], vc[layer_counter[0] % n_kv], att["strides"], table,
            d["prefix_len"], d["n_nodes"], mask_out["mask"], w.Hkv, att["scale"], out=o, workspace=ws)),
        "accept": time_call(accept),
    }

    # ---- optional: the steps around verification, each timed on its own (medians)
    extended = None
    if args.extended and not light:
        from inputs import templates
        tp, tr, _, sizes = templates.retrieval_envelope()
        kk = 8
        rng = np.random.default_rng(inputs.generate.BASE_SEED + 77)
        M = torch.from_numpy(rng.integers(0, w.vocab, (w.vocab, kk), dtype=np.int32)).cuda()
        tpl_p, tpl_r = up(tp), up(tr)
        n_ret = up(np.full(B, sizes["d5"], np.int32))
        n_draft = max(1, min(K - sizes["d5"], K // 2))
        tok2, par2 = d["tokens"].clone(), d["parent"].clone()
        nn2 = torch.full((B,), n_draft, dtype=torch.int32, device=dev)
        st2 = torch.empty(B, dtype=torch.int32, device=dev)

        def matrix_retrieve():
            nn2.fill_(n_draft)
            graft.graft_matrix_retrieve(M, tpl_p, tpl_r, n_ret, tok2, par2, nn2, status=st2)

        lg = logits if logits is not None else torch.from_numpy(
            inputs.make_step_inputs(w, with_logits=True)["logits"]).cuda()
        mu_ws = torch.empty(graft.graft_matrix_update_workspace_bytes(B, K, w.vocab, kk), dtype=torch.uint8, device=dev)
        ids2 = torch.empty((B, K), dtype=torch.int32, device=dev)

        def matrix_update():
            graft.graft_matrix_update(d["tokens"], d["n_nodes"], lg, M, target_ids=ids2, workspace=mu_ws)

        n_l = min(w.layers, n_kv)
        kv_all_k = torch.cat([x.reshape(-1) for x in kc[:n_l]])
        kv_all_v = torch.cat([x.reshape(-1) for x in vc[:n_l]])
        kc_out = {"new_prefix_len": torch.empty(B, dtype=torch.int32, device=dev),
                  "status": torch.empty(B, dtype=torch.int32, device=dev)}

        def kv_compact():
            graft.graft_kv_compact(kv_all_k, kv_all_v, kc[0].numel(), n_l, att["strides"], table, d["prefix_len"],
                                   acc_out["path"], acc_out["accept_len"], K, w.Hkv, w.D, out=kc_out)

        lq = torch.from_numpy(np.log(rng.random((B, K)).astype(np.float32) * 0.9 + 0.05)).cuda()
        chk = [up(np.array(a, np.int32)) for a in ([1, 2, 6], [8, 24, 40], [52, 36, 20])]
        chk_tau = torch.tensor([-0.5, -2.0, -6.0], dtype=torch.float32, device=dev)
        ps_out = {k_: torch.empty((B, K), dtype=torch.int32, device=dev) for k_ in ("parent", "tokens", "index")}
        ps_out.update({k_: torch.empty(B, dtype=torch.int32, device=dev) for k_ in ("n_nodes", "stage", "n_ret", "status")})

        def prune_select():
            graft.graft_prune_select(d["parent"], d["tokens"], lq, d["n_nodes"], chk[0], chk_tau, chk[1], chk[2],
                                     out=ps_out)

        t_ps = time_call(prune_select)
        t_mr, t_mu, t_kc = time_call(matrix_retrieve), time_call(matrix_update), time_call(kv_compact)
        torch.cuda.synchronize()
        assert torch.equal(ids2, d["target_ids"]) and int(st2.max()) == 0 and int(kc_out["status"].max()) == 0
        scan_bytes = 4.0 * B * K * w.vocab
        extended = {
            "prune_select_us": round(t_ps, 2),
            "matrix_retrieve_us": round(t_mr, 2), "template_nodes": int(sizes["d5"]),
            "matrix_update_us": round(t_mu, 2), "matrix_update_logits_bytes": int(scan_bytes), "successors_k": kk,
            "matrix_update_GBps_incl_launch": round(scan_bytes / (t_mu * 1e-6) / 1e9, 1),
            "kv_compact_us": round(t_kc, 2), "kv_compact_layers": n_l,
            "kv_compact_accept_len": [int(x) for x in acc_out["accept_len"].cpu().numpy()],
        }

    # ---- optional: the same step replayed from a captured HIP graph (launch overhead removed)
    graph_us = None
    if args.graph and not light:
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            step()                                   # warm-up on the capture stream
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step()
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        a, b_ = hip.event(), hip.event()
        cur = torch.cuda.current_stream().cuda_stream
        hip.record(a, cur)
        for _ in range(steps):
            g.replay()
        hip.record(b_, cur)
        torch.cuda.synchronize()
        graph_us = hip.elapsed_ms(a, b_) * 1e3 / steps

    # ---- sanity of the timed outputs against the generator's planted answers
    torch.cuda.synchronize()
    pos = ret_out["chain_pos"].cpu().numpy()
    for b in range(B):
        assert pos[b].tolist() == s["planted_pos"][b][:w.C], "retrieval lost the planted chains"
    assert torch.isfinite(o.float()).all()
    if args.logits:
        assert torch.equal(ids_out, d["target_ids"]), "argmax over the logits lost the planted target ids"

    step_att_bytes = att_bytes * w.layers
    value = step_att_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = att_bytes / (kernel_avg_ms * 1e-3) / 1e9
    mfma_tflops = att_flops / (kernel_avg_ms * 1e-3) / 1e12
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % w.name)
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get("traffic_bytes_per_launch")

    result = {
        "metric": "tree-verify attention HBM GB/s (% of peak) + retrieve+verify us/step",
        "value": round(value, 2), "unit": "GB/s",
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "us_per_step": round(ms_per_step * 1e3, 2),
        "us_per_step_p10_p50_p90": [round(float(np.percentile(step_us, q)), 2) for q in (10, 50, 90)],
        "us_per_step_hip_graph": None if graph_us is None else round(graph_us, 2),
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 5),
        "host_wall_ms_per_step": round(wall * 1e3 / steps, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {
            "workload": "%s: B=%d, prefix=%d, tree nodes=%d, Hq/Hkv/D=%d/%d/%d, layers=%d, paged KV block 16"
                        % (w.name, w.B, w.P, w.K, w.Hq, w.Hkv, w.D, w.layers),
            "step": "graft_retrieve + graft_build_tree_mask + %d x graft_tree_attn + graft_accept(%s)"
                    % (w.layers, "logits" if args.logits else "target_ids"),
            "kv_buffers_rotated": n_kv, "context_len": w.L, "vocab": w.vocab,
            "accept_mode": "logits" if args.logits else "target_ids",
            "attention_bytes_per_layer": att_bytes, "attention_flops_per_layer": att_flops,
        },
        "per_call_us": {k: round(v, 2) for k, v in per_call_us.items()},
        "extended": extended,
        "roofline": {
            "kernel": "tree_attn_mfma_kernel" if (w.dtype == "bf16" and w.D == 128) else "tree_attn_simple_kernel",
            "bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
            "kernel_avg_us": round(kernel_avg_ms * 1e3, 3), "launches_timed": n_ev,
            "mfma_tflops": round(mfma_tflops, 2), "mfma_frac": round(mfma_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
            "arithmetic_intensity_flop_per_byte": round(att_flops / att_bytes, 1),
        },
    }

    if not args.no_cpu_baseline and not light:
        result["cpu_baseline"] = cpu_baseline(w, s, att, att_bytes, args.cpu_seconds)
    del kc, vc, q
    torch.cuda.empty_cache()
    return result


def cpu_baseline(w, s, att, att_bytes, budget_s):
    """The oracle, as it stands, timed on the host: integer steps in full, attention on a
    seeded sample of (sequence, node, head) rows sized to the time budget, scaled to one step."""
    import oracle
    t0 = time.perf_counter()
    oracle.retrieve(s["ctx"], s["ctx_len"], w.n_min, w.n_max, w.C, w.m, s["tail"], s["tail_len"])
    oracle.build_tree_mask(s["parent"], s["n_nodes"], s["prefix_len"], w.K, 48)
    oracle.accept(s["parent"], s["tokens"], s["n_nodes"], 48, target_ids=s["target_ids"])
    t_int = time.perf_counter() - t0
    cores = len(os.sched_getaffinity(0))
    omp = os.environ.get("OMP_NUM_THREADS")
    threads = min(cores, int(omp)) if omp else cores
    total_rows = w.B * w.K * w.Hq
    rng = np.random.default_rng(1)

    def run(n):
        rows = np.stack([rng.integers(0, w.B, n), rng.integers(0, w.K, n), rng.integers(0, w.Hq, n)],
                        axis=1).astype(np.int32)
        t = time.perf_counter()
        oracle.tree_attn(att["q"][0], att["k_cache"][0], att["v_cache"][0], w.dtype, att["strides"],
                         att["block_table"], s["prefix_len"], s["n_nodes"], s["parent"], w.Hq, w.Hkv, w.D,
                         w.page_size, att["scale"], rows=rows)
        return time.perf_counter() - t
    n = min(total_rows, 4 * threads)
    t = run(n)
    per_row = t / n
    n2 = int(min(total_rows, max(n, budget_s / max(per_row, 1e-9))))
    t2 = run(n2)
    per_row = t2 / n2
    est_step = t_int + per_row * total_rows * w.layers
    return {
        "value": round(att_bytes * w.layers / est_step / 1e9, 4), "unit": "GB/s",
        "cores": threads, "kind": "oracle",
        "sample": "integer steps in full (%.4f s) + attention on %d of %d (sequence,node,head) rows of one layer "
                  "(%.2f s), scaled to %d layers: %.1f s per step" % (t_int, n2, total_rows, t2, w.layers, est_step),
        "est_seconds_per_step": round(est_step, 3),
    }


if __name__ == "__main__":
    main()
