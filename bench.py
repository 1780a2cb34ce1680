#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: paged decode attention through a layout view
(KV bytes/s against the HBM roofline, microseconds per layer) and kv_repack GB/s.

A step is one paged_decode_attn call (main kernel + split-KV merge) over one batch of the
workload, inputs resident in HBM.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak


def ensure_built():
    from paper_2602_22593_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2602_22593_amd.build import build
        build()


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(case, target_seconds=10.0):
    """The oracle as it stands, timed on the host cores on the same inputs (pool copy 0): full passes
    on all its threads, then one pass of a quarter of the sequences on a single thread for scale."""
    import numpy as np
    import oracle
    w = case.workload
    view = oracle.View(oracle.Geometry(w.n_q_heads, w.n_kv_heads, w.head_dim, w.base_block_size),
                       *case.triple)
    pool = case.pools[0].view(dtype=__import__("torch").int16).cpu().numpy().view(np.uint16)
    q = case.q.view(dtype=__import__("torch").int16).cpu().numpy().view(np.uint16)
    table, ctx = case.tables[0], case.ctx
    threads = oracle.num_threads()
    reps, spent = 0, 0.0
    while reps < 8 and spent < target_seconds:
        t0 = time.perf_counter()
        ref = oracle.paged_decode(view, q, pool, table, ctx)
        spent += time.perf_counter() - t0
        reps += 1
    # one thread, every fourth sequence (the rest given length 0), scaled by the token share
    sub = np.where(np.arange(len(ctx)) % 4 == 0, ctx, 0).astype(np.int32)
    oracle.set_num_threads(1)
    try:
        t0 = time.perf_counter()
        oracle.paged_decode(view, q, pool, table, sub)
        one = time.perf_counter() - t0
    finally:
        oracle.set_num_threads(threads)
    one_full = one * float(ctx.sum()) / max(float(sub.sum()), 1.0)
    return {
        "value": round(case.kv_bytes * reps / spent / 1e9, 4), "unit": "GB/s", "cores": threads,
        "kind": "oracle", "cpu_model": cpu_model(),
        "seconds_per_pass": round(spent / reps, 4),
        "one_thread_s": round(one_full, 3),
        "sample": f"all {len(ctx)} sequences of the workload, {reps} full passes on {threads} threads, "
                  f"{spent / reps:.2f} s per pass, {spent * threads:.0f} core-seconds in all "
                  f"(fp64, OpenMP over (sequence, query head)); one_thread_s: every fourth sequence on one "
                  f"thread ({one:.2f} s), scaled to the whole batch by tokens",
    }, ref


def library_context(kv, wqkv, wo):
    """What torch's own kernels (the vendor libraries behind them) do on this GPU for the same shapes:
    causal SDPA on contiguous, un-paged K/V, and matmul on contiguous weights.  Each GEMM is timed
    as a replayed HIP graph of one call per weight copy, and so is kv_linear_view beside it, so that
    neither side pays per-call host time.  Context for the reader, not a target and not a parity check."""
    import torch
    import torch.nn.functional as F

    def graph_us(calls):
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(3):
                for c in calls:
                    c()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for c in calls:
                c()
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (20 * len(calls)) * 1e3

    out = {"sdpa_causal_contiguous": [], "matmul_graph": []}
    for what, B, hq, hkv, S in (("8 prompts of 4096 tokens, 32 q / 8 kv heads", 8, 32, 8, 4096),
                                ("8 prompts of 4096 tokens, 16 q / 4 kv heads", 8, 16, 4, 4096)):
        q = torch.randn(B, hq, S, 128, device="cuda", dtype=torch.bfloat16)
        k = torch.randn(B, hkv, S, 128, device="cuda", dtype=torch.bfloat16)
        v = torch.randn(B, hkv, S, 128, device="cuda", dtype=torch.bfloat16)
        fn = lambda: F.scaled_dot_product_attention(q, k, v, is_causal=True, enable_gqa=True)
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        flops = 4.0 * 128 * hq * B * (S * (S + 1) / 2)
        out["sdpa_causal_contiguous"].append({"what": what, "ms": round(ms, 4), "TFLOPs": round(flops / ms / 1e9, 1)})
        del q, k, v
        torch.cuda.empty_cache()
    hq, hkv, d, hidden, M = 32, 8, 128, 4096, 64
    x = torch.randn((M, hidden), device="cuda").to(torch.bfloat16)
    for name, ws, view in (("qkv", wqkv, kv.kv_weight_view_fused_qkv(hq, hkv, d, hidden, 0, 1)),
                           ("wo", wo, kv.kv_weight_view_make(1, 0, 1, hidden, hq * d))):
        ys = [torch.empty((M, w.shape[0]), dtype=torch.bfloat16, device="cuda") for w in ws]
        lib_us = graph_us([(lambda w=w, y=y: torch.matmul(x, w.t(), out=y)) for w, y in zip(ws, ys)])
        own_us = graph_us([(lambda w=w, y=y: kv.kv_linear_view(x, w, view, out=y)) for w, y in zip(ws, ys)])
        out["matmul_graph"].append({"layer": name, "M": M, "tp_degree": 1, "torch_matmul_us": round(lib_us, 2),
                                    "kv_linear_view_us": round(own_us, 2)})
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama8b_dp_b64")
    ap.add_argument("--view", default=None, help="layout,p,r (default: the workload's first view)")
    ap.add_argument("--copies", type=int, default=4, help="independent pools cycled through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip repack and the other workloads")
    ap.add_argument("--library-context", action="store_true",
                    help="also time the vendor libraries through torch on the same shapes (context only): "
                         "SDPA on contiguous K/V for the prefill cases, matmul on the weight slices")
    ap.add_argument("--probe", action="store_true",
                    help="only run the known-traffic streaming kernels (read 1 GiB, copy 1 GiB) and exit")
    ap.add_argument("--placement", action="store_true",
                    help="only run the placement probe (which XCD each workgroup index runs on, and how "
                         "fast each XCD streams its share of 256 MiB) and exit")
    ap.add_argument("--extras-only", default=None, metavar="SECTION[:INDEX]",
                    help="of the rows beyond the headline workload, run only this section of the output's "
                         "'extras' (kv_repack, kv_repack_long, other_workloads, mixed_layout_decode, "
                         "paged_prefill_attn, kv_linear_view), or only its INDEX-th case: for profiler runs")
    ap.add_argument("--option", action="append", default=[], metavar="KEY=VALUE",
                    help="set a library option (kv_set_option) before measuring; may be repeated")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    ensure_built()
    import numpy as np
    import torch
    from paper_2602_22593_amd import binding as kv
    from paper_2602_22593_amd import harness, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    def stream_ceiling(n_bytes=1 << 30, iters=10):
        """Measured read and copy rates of the trivial streaming kernels (GB/s)."""
        src = torch.empty(n_bytes, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty(n_bytes, dtype=torch.uint8, device="cuda")
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        rd = harness.time_calls(lambda i: kv.kv_probe_read(src, n_cu), iters, 3)
        cp = harness.time_calls(lambda i: kv.kv_probe_copy(dst, src, n_cu), iters, 3)
        # the paged pattern: a random 5/6 of the 64 KiB blocks of the buffer, each read whole
        n_blk = n_bytes // 65536
        ids = torch.randperm(n_blk, device="cuda", dtype=torch.int32)[: n_blk * 5 // 6].contiguous()
        pg = harness.time_calls(lambda i: kv.kv_probe_read_blocks(src, ids, 65536, n_cu), iters, 3)
        return {"read_GBps": round(n_bytes / rd / 1e6, 1), "copy_read_plus_write_GBps": round(2 * n_bytes / cp / 1e6, 1),
                "paged_64KiB_blocks_read_GBps": round(int(ids.numel()) * 65536 / pg / 1e6, 1),
                "bytes": n_bytes, "workgroups": n_cu}

    if args.probe:
        print(json.dumps({"probe": stream_ceiling()}))
        return
    if args.placement:
        # 256 workgroups (one per compute unit, 1 MiB each) as the decode kernels launch them
        n_wg = torch.cuda.get_device_properties(0).multi_processor_count
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        runs = []
        for _ in range(6):
            rec = kv.kv_probe_read_placed(src, n_wg)
            torch.cuda.synchronize()
            runs.append(rec.cpu().numpy())
        runs = runs[1:]                                  # the first launch is the cold one
        xcc = runs[0][:, 0]
        same_every_run = all((r[:, 0] == xcc).all() for r in runs)
        by_rule = bool((xcc == np.arange(n_wg) % 8).all())
        dur = np.mean([(r[:, 2] - r[:, 1]) * 0.01 for r in runs], axis=0)        # us per workgroup
        end = np.mean([(r[:, 2] - r[:, 1].min()) * 0.01 for r in runs], axis=0)  # end after the first start
        per_xcd = {int(x): {"workgroups": int((xcc == x).sum()), "mean_stream_us": round(float(dur[xcc == x].mean()), 2),
                            "mean_end_us": round(float(end[xcc == x].mean()), 2)} for x in np.unique(xcc)}
        print(json.dumps({"placement": {"workgroups": n_wg, "bytes": int(src.numel()),
                                        "xcd_of_workgroup_is_index_mod_8": by_rule,
                                        "same_in_every_launch": bool(same_every_run),
                                        "first_16_workgroups_xcd": [int(v) for v in xcc[:16]], "per_xcd": per_xcd}}))
        return
    for item in args.option:
        key, _, val = item.partition("=")
        kv.kv_set_option(key, int(val))
    w = wl.WORKLOADS[args.workload]
    triple = tuple(int(x) for x in args.view.split(",")) if args.view else w.views[0]

    case = harness.build_decode_case(w, triple, n_copies=args.copies)
    run = case.prepared()

    # --- timed region: exactly K steps between two synchronisations ---------------------------
    for i in range(args.warmup):
        run(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run(args.warmup + i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    gbps = case.kv_bytes / (ms_per_step * 1e-3) / 1e9

    # --- single calls between pairs of events on the launch stream: median and minimum beside the mean
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for i, (e0, e1) in enumerate(ev):
        e0.record()
        run(i)
        e1.record()
    torch.cuda.synchronize()
    call_us = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in ev)

    # --- per-kernel durations from HIP events on the launch stream (separate pass, switched on after
    #     the warm-up above): the kernels' own start and end times, taken by the launch itself ------
    kv.kv_profile_enable(True)
    for i in range(args.steps):
        run(i)
    torch.cuda.synchronize()
    main_ms, n_main = kv.kv_profile_read(kv.KV_PROF_DECODE_MAIN)
    merge_ms, n_merge = kv.kv_profile_read(kv.KV_PROF_DECODE_MERGE)
    kv.kv_profile_enable(False)
    main_avg_ms = main_ms / max(n_main, 1)
    achieved = case.kv_bytes / (main_avg_ms * 1e-3) / 1e9

    # HBM traffic per launch is not measured in this run: it comes from the committed counter
    # summaries (profiles/), keyed by workload and view; null where no summary covers the case
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(f"{w.name}:{','.join(map(str, triple))}")
            traffic_source = "profiles/traffic.json (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by the copy probe)" \
                if traffic is not None else None
        except Exception:
            traffic = None

    result = {
        "metric": "decode-attn KV bytes/s", "value": round(gbps, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "us_per_layer": round(ms_per_step * 1e3, 2),
        "us_per_call_median": round(call_us[len(call_us) // 2], 2), "us_per_call_min": round(call_us[0], 2),
        "pct_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "view": {"layout": "DP" if triple[0] == 0 else "TP",
                                                "tp_degree": triple[1], "rank": triple[2]},
                   "n_q_local": case.view.n_q_local, "n_kv_local": case.view.n_kv_local,
                   "head_dim": w.head_dim, "block_tokens": case.view.block_tokens,
                   "batch": w.batch, "tokens": int(case.ctx.sum()), "kv_bytes": case.kv_bytes,
                   "pool_copies": args.copies, "storage": "bf16 K/V/q/out", "accumulate": "fp32",
                   "library_options": {k: int(v) for k, _, v in (o.partition("=") for o in args.option)}},
        "roofline": {"bound": "hbm", "kernel": "paged decode main kernel",
                     "achieved": round(achieved, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_source": traffic_source,
                     "avg_kernel_us": round(main_avg_ms * 1e3, 2),
                     "merge_kernel_us": round(merge_ms / max(n_merge, 1) * 1e3, 2) if n_merge else None,
                     "algorithmic_bytes_per_launch": case.kv_bytes},
    }
    result["roofline"]["measured_stream_ceiling"] = stream_ceiling()

    if not args.no_cpu_baseline:
        base, ref = cpu_baseline(case)
        result["cpu_baseline"] = base
        # the timed configuration must also be right: compare against the oracle's output
        out = case.run(0)
        torch.cuda.synchronize()
        got = (out.view(dtype=torch.int16).cpu().numpy().view(np.uint16).astype(np.uint32) << 16) \
            .view(np.float32).astype(np.float64)
        err = np.abs(got - ref)
        result["parity_vs_oracle"] = {"max_abs": float(err.max()), "mean_abs": float(err.mean()),
                                      "ok": bool(err.max() <= 2e-2 and err.mean() <= 2e-3)}

    if not args.no_extras:
        extras = {}
        del case, run
        torch.cuda.empty_cache()
        # kv_repack: the 8B batch-128 lengths, DP layout -> rank-0 TP4 layout and back; and the two
        # 131072-token sequences of the long-context mix, DP -> rank-0 TP4
        def timed_repack(fn, steps):
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            kv.kv_profile_enable(True)           # after the warm-up: only the timed launches are recorded
            ms = harness.time_calls(lambda i: fn(), steps, 0)
            k_ms, k_n = kv.kv_profile_read(kv.KV_PROF_REPACK)
            kv.kv_profile_enable(False)
            return ms, k_ms / max(k_n, 1)

        def repack_row(moved, ms, k_ms):
            return {"us": round(ms * 1e3, 2), "kernel_us": round(k_ms * 1e3, 2),
                    "read_plus_write_GBps": round(2 * moved / (ms * 1e-3) / 1e9, 1),
                    "roofline": {"bound": "hbm", "achieved": round(2 * moved / (k_ms * 1e-3) / 1e9, 1),
                                 "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                 "frac": round(2 * moved / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}}

        only_section, _, only_index = (args.extras_only or "").partition(":")

        def want(section, index=None):
            if not only_section:
                return True
            return section == only_section and (only_index == "" or index is None or int(only_index) == index)

        steps = max(50, args.steps // 2)
        if want("kv_repack"):
            rw = wl.WORKLOADS["llama8b_tp_b128"]
            rc = harness.build_repack_case(rw, (0, 1, 0), (1, 4, 0))
            fwd = timed_repack(rc.forward, steps)
            bwd = timed_repack(rc.backward, steps)
            extras["kv_repack"] = {"workload": rw.name, "moved_bytes": rc.moved_bytes, "calls_timed": steps,
                                   "dp_to_tp4_r0": repack_row(rc.moved_bytes, *fwd),
                                   "tp4_r0_to_dp": repack_row(rc.moved_bytes, *bwd)}
            del rc
            torch.cuda.empty_cache()
        if want("kv_repack_long"):
            lw = wl.WORKLOADS["llama8b_tp4_longmix"]
            rc = harness.build_repack_case(lw, (0, 1, 0), (1, 4, 0), np.array([131072, 131072], dtype=np.int32))
            fwd = timed_repack(rc.forward, steps)
            extras["kv_repack_long"] = {"workload": lw.name, "what": "the two 131072-token sequences, DP -> TP4 rank 0",
                                        "moved_bytes": rc.moved_bytes, "calls_timed": steps,
                                        "dp_to_tp4_r0": repack_row(rc.moved_bytes, *fwd)}
            del rc
            torch.cuda.empty_cache()
        others = []
        for name in ("llama8b_tp_b128", "llama70b_tp8_b256", "llama8b_tp4_longmix") if want("other_workloads") else ():
            ow = wl.WORKLOADS[name]
            for tr in ow.views:
                oc = harness.build_decode_case(ow, tr, n_copies=args.copies)
                orun = oc.prepared()
                ms = harness.time_calls(orun, max(50, args.steps // 2), 10)
                kv.kv_profile_enable(True)
                for i in range(20):
                    orun(i)
                torch.cuda.synchronize()
                k_ms, k_n = kv.kv_profile_read(kv.KV_PROF_DECODE_MAIN)
                m_ms, m_n = kv.kv_profile_read(kv.KV_PROF_DECODE_MERGE)
                kv.kv_profile_enable(False)
                k_ms /= max(k_n, 1)
                others.append({"workload": name, "view": list(tr), "kv_bytes": oc.kv_bytes,
                               "us_per_layer": round(ms * 1e3, 2),
                               "GBps": round(oc.kv_bytes / (ms * 1e-3) / 1e9, 1),
                               "pct_hbm_peak": round(100 * oc.kv_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
                               "main_kernel_us": round(k_ms * 1e3, 2),
                               "merge_kernel_us": round(m_ms / m_n * 1e3, 2) if m_n else None,
                               "roofline": {"bound": "hbm", "achieved": round(oc.kv_bytes / k_ms / 1e6, 1),
                                            "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                            "frac": round(oc.kv_bytes / k_ms / 1e6 / HBM_PEAK_GBPS, 4)}})
                del oc, orun
                torch.cuda.empty_cache()
        if want("other_workloads"):
            extras["other_workloads"] = others

        # --- rows beyond the headline path, each against its own roofline -------------------------
        MFMA_BF16_PEAK_TFLOPS = 2500.0
        if want("mixed_layout_decode"):
            mw = wl.WORKLOADS["llama8b_tp_b128"]
            mc = harness.build_mixed_case(mw, 2, 0)
            ms = harness.time_calls(mc.run, max(10, args.steps // 2), 5)
            extras["mixed_layout_decode"] = {
                "workload": mw.name, "what": "TP2 rank 0; every other sequence read in place from DP-layout blocks; one launch",
                "us_per_layer": round(ms * 1e3, 2), "GBps": round(mc.kv_bytes / (ms * 1e-3) / 1e9, 1),
                "pct_hbm_peak": round(100 * mc.kv_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2)}
            del mc
            torch.cuda.empty_cache()

        pre = []
        w8 = wl.Workload("llama8b_recompute", 90, 32, 8, 128, 16, 8, "fixed", ())
        for case_no, (label, tr, ctx, ql) in enumerate((
                ("8 prompts of 4096 tokens, whole", (0, 1, 0), [4096] * 8, [4096] * 8),
                ("8 prompts of 4096 tokens, whole", (1, 2, 0), [4096] * 8, [4096] * 8),
                ("16 chunks of 512 tokens on 8192 cached", (0, 1, 0), [8192] * 16, [512] * 16),
                ("1 chunk of 512 tokens on 131072 cached (key range split over workgroups)", (0, 1, 0), [131072], [512]))):
            if not want("paged_prefill_attn", case_no):
                continue
            pc = harness.build_prefill_case(w8, tr, ctx, ql)
            for i in range(3):
                pc.run(i)
            torch.cuda.synchronize()
            kv.kv_profile_enable(True)
            ms = harness.time_calls(pc.run, 10, 0)
            k_ms, k_n = kv.kv_profile_read(kv.KV_PROF_PREFILL)
            kv.kv_profile_enable(False)
            k_ms /= max(k_n, 1)
            pre.append({"what": label, "view": list(tr), "ms": round(ms, 4), "kernel_ms": round(k_ms, 4),
                        "algorithmic_TFLOP": round(pc.flops / 1e12, 3),
                        "roofline": {"bound": "mfma", "achieved": round(pc.flops / k_ms / 1e9, 1),
                                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                     "frac": round(pc.flops / k_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)}})
            del pc
            torch.cuda.empty_cache()
        if pre:
            extras["paged_prefill_attn"] = pre

        lin = []
        hq, hkv, d, hidden = 32, 8, 128, 4096
        g = torch.Generator(device="cuda")
        g.manual_seed(wl.SEED_BASE + 777)
        n_w = 6   # distinct weights cycled through, so that no call finds its weight in the last-level cache
        wqkv = [torch.randn(((hq + 2 * hkv) * d, hidden), generator=g, device="cuda").to(torch.bfloat16) for _ in range(n_w)]
        wo = [torch.randn((hidden, hq * d), generator=g, device="cuda").to(torch.bfloat16) for _ in range(n_w)]
        case_no = -1
        for M, m in ((64, 1), (64, 2), (128, 2), (256, 8)):
            x = torch.randn((M, hidden), generator=g, device="cuda").to(torch.bfloat16)
            a_full = torch.randn((M, hq * d), generator=g, device="cuda").to(torch.bfloat16)
            for name, view, xin, ws in (("qkv", kv.kv_weight_view_fused_qkv(hq, hkv, d, hidden, 0, m), x, wqkv),
                                        ("wo", kv.kv_weight_view_make(1, 0, m, hidden, hq * d), None, wo)):
                case_no += 1
                if not want("kv_linear_view", case_no):
                    continue
                if xin is None:
                    xin = a_full[:, :view.col_count]
                out = torch.empty((M, view.n_rows), dtype=torch.bfloat16, device="cuda")
                for i in range(4):
                    kv.kv_linear_view(xin, ws[i % n_w], view, out=out)
                torch.cuda.synchronize()
                kv.kv_profile_enable(True)
                for i in range(24):
                    kv.kv_linear_view(xin, ws[i % n_w], view, out=out)
                torch.cuda.synchronize()
                k_ms, k_n = kv.kv_profile_read(kv.KV_PROF_LINEAR)
                kv.kv_profile_enable(False)
                k_ms /= max(k_n, 1)
                wbytes = view.n_rows * view.col_count * 2
                lin.append({"layer": name, "M": M, "tp_degree": m, "weight_slice_bytes": wbytes,
                            "kernel_us": round(k_ms * 1e3, 2),
                            "roofline": {"bound": "hbm", "achieved": round(wbytes / k_ms / 1e6, 1), "peak": HBM_PEAK_GBPS,
                                         "unit": "GB/s", "frac": round(wbytes / k_ms / 1e6 / HBM_PEAK_GBPS, 4)},
                            "TFLOPs": round(2.0 * M * view.n_rows * view.col_count / k_ms / 1e9, 1)})
        if lin:
            extras["kv_linear_view"] = lin
        if args.library_context:
            extras["library_context"] = library_context(kv, wqkv, wo)
        result["extras"] = extras

    print(json.dumps(result))


if __name__ == "__main__":
    main()
