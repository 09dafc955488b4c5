"""Where the time of the MFMA attention kernel goes, workgroup by workgroup.

    python -m paper_2605_20104_amd.build --timing
    python -m paper_2605_20104_amd.timing --workload c3
    python -m paper_2605_20104_amd.timing --workload c3 --kv-heads 1 --splits 31 --row-tiles 1
    python -m paper_2605_20104_amd.timing --mfma-calibration

Runs graft_tree_attn of the timing build (libgraft_timing.so: the same kernel compiled with
-DGRAFT_ATTN_STAMPS, which makes every workgroup record the 100 MHz real-time counter at the
points of its life and the core-clock counter at both ends of its stage loop) on the seeded
inputs of a workload and prints, over all workgroups that ran the full number of stages, when
each point was passed, the clock the stage loop ran at, and when the last workgroup ended.
--kv-heads runs the same shape with fewer KV heads (fewer workgroups) and --splits /
--row-tiles hold the launch plan, so that runs differ in the load on the chip only.
--mfma-calibration instead runs a plain stream of independent v_mfma_f32_16x16x32_bf16 on every
compute unit, with operands that are all zero, all one, or N(0,1) like the workloads' data, and
prints the rate and the clock the chip holds under each: the ceiling the attention kernel's matrix
work has on this machine, for its kind of data.
Needs a GPU; the numbers of the product library are not affected (the stamps cost about
0.3 us per workgroup).
"""
from __future__ import annotations

import argparse
import ctypes
import dataclasses
import os
import sys

import numpy as np
import torch

import paper_2605_20104_amd as graft
from paper_2605_20104_amd import build as graft_build

POINTS = ["lengths known", "table entries requested", "Q converted", "table and masks in LDS", "stage 0 requested",
          "accumulators zeroed, stage 1 requested", "stage loop entered", "first keys arrived", "stage loop left",
          "results written"]


def mfma_calibration(lib):
    lib.graft_mfma_calibration.restype = ctypes.c_int32
    lib.graft_mfma_calibration.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                           ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    gen = torch.Generator(device="cpu").manual_seed(20104)
    kinds = {
        "all zero": torch.zeros(8 * 64 * 8, dtype=torch.bfloat16),
        "all one": torch.ones(8 * 64 * 8, dtype=torch.bfloat16),
        "N(0,1)": torch.randn(8 * 64 * 8, generator=gen).to(torch.bfloat16),
    }
    stream = torch.cuda.current_stream().cuda_stream
    print("plain stream of v_mfma_f32_16x16x32_bf16, eight independent accumulators per wavefront, %d compute units" % cus)
    print("  operands   wavefronts/SIMD  workgroups   time (us)  by events   TFLOP/s   clock (GHz)  cycles per MFMA of a wavefront, its loop (us)")
    for threads in (256, 512, 768, 1024):
        for n_wg in (cus // 8, cus):
            for name, host in kinds.items():
                ops = host.cuda()
                iters = 8000 * 256 // threads
                sink = torch.empty(n_wg * threads, dtype=torch.float32, device="cuda")
                n_waves = n_wg * (threads // 64)
                stamps = torch.zeros(n_waves * 4, dtype=torch.int64, device="cuda")
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                for _ in range(3):                                   # the last launch is reported
                    e0.record()
                    rc = lib.graft_mfma_calibration(ops.data_ptr(), sink.data_ptr(), stamps.data_ptr(), n_wg, threads,
                                                    iters, stream)
                    e1.record()
                    assert rc == 0, rc
                torch.cuda.synchronize()
                event_us = e0.elapsed_time(e1) * 1e3
                if name == "all one":                                # every MFMA adds 32 to its 16 x 16 sums
                    assert float(sink.min()) == float(sink.max()) == 1024.0 * iters, (float(sink.min()), iters)
                st = stamps.cpu().numpy().view(np.uint64).reshape(n_waves, 4).astype(np.float64)
                assert (st[:, 3] == 1).all()
                span_us = (st[:, 1].max() - st[:, 0].min()) / 100.0      # first loop entered to last loop left
                loop_us = (st[:, 1] - st[:, 0]) / 100.0
                clk = (st[:, 2] / (loop_us * 1e3)).mean()                 # each wavefront's own loop
                flops = float(n_waves) * iters * 8 * 16384.0
                print("  %-10s %9d %13d %11.1f %10.1f %9.0f %11.3f %12.2f %10.1f"
                      % (name, threads // 256, n_wg, span_us, event_us, flops / (span_us * 1e-6) / 1e12, clk,
                         st[:, 2].mean() / (iters * 8), loop_us.mean()))


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--workload", default="c3", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--kv-heads", type=int, default=0, help="run with this many KV heads (same group size)")
    ap.add_argument("--splits", type=int, default=0, help="hold the plan at this many splits (with --row-tiles)")
    ap.add_argument("--row-tiles", type=int, default=0)
    ap.add_argument("--kv-buffers", type=int, default=0, help="K/V buffers the calls rotate over (default 4 for c3, else 1)")
    ap.add_argument("--calls", type=int, default=9, help="launches; the last one is reported")
    ap.add_argument("--mfma-calibration", action="store_true", help="rate and clock of a plain MFMA stream instead")
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        sys.exit("timing needs a GPU")
    if not os.path.exists(graft_build.LIB_TIMING):
        sys.exit("%s is missing: build it with `python -m paper_2605_20104_amd.build --timing`" % graft_build.LIB_TIMING)
    sys.path.insert(0, graft_build.ROOT)
    import inputs

    graft.LIB_PATH = graft_build.LIB_TIMING
    lib = graft.load_library()
    if args.mfma_calibration:
        return mfma_calibration(lib)
    lib.graft_attn_stamp_buffer.restype, lib.graft_attn_stamp_buffer.argtypes = ctypes.c_int32, [ctypes.c_void_p, ctypes.c_size_t]
    lib.graft_attn_force_plan.restype, lib.graft_attn_force_plan.argtypes = ctypes.c_int32, [ctypes.c_int32, ctypes.c_int32]
    n_stamps = lib.graft_attn_stamp_count()

    w = inputs.get_workload(args.workload)
    if args.kv_heads:
        w = dataclasses.replace(w, Hkv=args.kv_heads, Hq=args.kv_heads * (w.Hq // w.Hkv))
    n_kv = args.kv_buffers or (4 if args.workload == "c3" else 1)
    att = inputs.make_attention_inputs(w, kv_buffers=n_kv, q_layers=1)

    def up(a):
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()

    q = up(att["q"][0])
    kc, vc = [up(a) for a in att["k_cache"]], [up(a) for a in att["v_cache"]]
    table = torch.from_numpy(att["block_table"].astype(np.int32)).cuda()
    s = inputs.make_step_inputs(w)
    parent, n_nodes, prefix = (torch.from_numpy(s[k]).cuda() for k in ("parent", "n_nodes", "prefix_len"))
    mask = graft.graft_build_tree_mask(parent, n_nodes, prefix)["mask"]
    out = torch.empty((w.B, w.K, w.Hq, w.D), dtype=torch.bfloat16, device="cuda")

    lib.graft_attn_force_plan(args.splits, args.row_tiles)
    need = graft.graft_tree_attn_workspace_bytes(w.B, w.K, w.Hq, w.Hkv, w.D, table.shape[1], 1)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    max_wgs = 1 << 16
    stamps = torch.zeros(max_wgs * n_stamps, dtype=torch.int64, device="cuda")
    lib.graft_attn_stamp_buffer(stamps.data_ptr(), stamps.numel() * 8)
    for i in range(args.calls):
        graft.graft_tree_attn(q, kc[i % n_kv], vc[i % n_kv], att["strides"], table, prefix, n_nodes, mask, w.Hkv,
                              att["scale"], out=out, workspace=ws)
    torch.cuda.synchronize()
    lib.graft_attn_stamp_buffer(None, 0)
    lib.graft_attn_force_plan(0, 0)

    st = stamps.cpu().numpy().view(np.uint64).reshape(max_wgs, n_stamps).astype(np.float64)
    wg = np.nonzero(st[:, 14] == 1)[0]           # (workgroups of the grid's padding record nothing)
    st = st[wg]
    if not len(st):
        sys.exit("no stamps: this shape does not take the MFMA path")
    full = st[:, 13] == st[:, 13].max()
    print("%s, %d KV heads: %d workgroups, %d of them with %d stages; K/V rotating over %d buffer(s)"
          % (w.name, w.Hkv, len(st), int(full.sum()), int(st[:, 13].max()), n_kv))
    print("  microseconds after the workgroup's start, workgroups with all stages:   mean    p10    p50    p90    max")
    for k, name in enumerate(POINTS, 1):
        v = st[full, k] / 100.0
        print("  %-72s %6.2f %6.2f %6.2f %6.2f %6.2f" % (name, v.mean(), *np.percentile(v, [10, 50, 90, 100])))
    loop_us = (st[full, 9] - st[full, 7]) / 100.0
    cyc = st[full, 12] - st[full, 11]
    clk = cyc / (loop_us * 1e3)
    print("  stage loop: %.1f us, %.1f k cycles, clock %.3f GHz (p10 %.3f, p90 %.3f)"
          % (loop_us.mean(), cyc.mean() / 1e3, clk.mean(), *np.percentile(clk, [10, 90])))
    if n_stamps > 16:
        n_full = st[full, 13]
        print("  wavefront 0, per stage: %.0f cycles waiting for its transfers, %.0f at the stage barrier"
              % ((st[full, 15] / n_full).mean(), (st[full, 16] / n_full).mean()))
    start = (st[:, 0] - st[:, 0].min()) / 100.0
    end = start + st[:, 10] / 100.0
    print("  workgroups start within %.2f us; the last one ends %.2f us after the first one started" % (start.max(), end.max()))
    xcd = wg % 8                                   # workgroups go to the XCDs round-robin
    if full.sum() >= 64:
        print("  mean end by XCD (us): " + " ".join(
            "%.1f" % end[full & (xcd == x)].mean() if (full & (xcd == x)).any() else "-" for x in range(8)))


if __name__ == "__main__":
    main()
