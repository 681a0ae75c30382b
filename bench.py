#!/usr/bin/env python3
"""Decode-step benchmark of libshadowkv on one MI355X.

One "step" = one shadowkv_decode_step (landmark scoring, selection, key rebuild + RoPE,
value gather, attention) for the whole batch of a synthetic workload shaped like the
paper's; the metric is decode tokens/s = batch / step time, inputs resident before the
timed region.  Prints ONE JSON line (see the fields below) with a `roofline` object for
the dominant kernel (landmark scoring, HBM-bound), a `rooflines` list with one such object
per memory-bound stage (scoring, attention + combine, the pre-filling call), and a
`cpu_baseline` object (the CPU oracle timed on this host on a bounded sample, on all
cores and on one thread).  `--workload all` runs the benchmark's configurations one after
the other, each in a process of its own, and prints one such line per configuration.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth


def algorithmic_bytes(wl, kv_bytes: int = 2) -> dict:
    """Bytes the method itself has to move per decode step, by consumer: ``kv_bytes`` per element of the KV-cache
    tensors (2 = bf16, 1 = FP8 E5M2), 2 per element of the query and the output."""
    d, c, r, k, o, w, G = wl.head_dim, wl.chunk_size, wl.rank, wl.topk_chunks, wl.n_outlier_chunks, wl.local_len, wl.group
    u, e = wl.units, kv_bytes
    per = {
        "landmarks": e * d * wl.n_landmarks,            # read once for all G heads of the group
        "A_rows": e * r * k * c,                        # gathered rows of the left factor
        "B": e * r * d,
        "values": e * d * k * c,                        # selected chunks' values, read once
        "resident_kv": 2 * e * d * (o * c + w),         # outlier + recent keys and values
        "q_out": 2 * 2 * d * G,
    }
    tot = {n: v * u for n, v in per.items()}
    tot["total"] = sum(tot.values())
    return tot


def equivalent_bandwidth(S: int, C: int, K: int, O: int, alpha: float, b_gpu: float, b_pcie: float) -> float:
    """The paper's equivalent-bandwidth model (section "Theoretical Equivalent Bandwidth"): the bandwidth a dense
    attention over S tokens would need to take the time ShadowKV takes -- landmarks S/C and attended K, V rows
    2(K+O)C at GPU bandwidth, the missed share (1 - alpha) of the K*C selected value rows at PCIe bandwidth.
    Same unit as ``b_gpu`` / ``b_pcie``.  Reported for context next to the measured numbers."""
    return 2.0 * S * b_gpu / (S / C + 2.0 * (K + O) * C + (1.0 - alpha) * K * C * b_gpu / b_pcie)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c3-hbm", help="c1 | c2 | c3-hbm | c3-host | c4 | c5 (the benchmark's configurations), c3-g7, c3-g8")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time budget of the oracle leg")
    ap.add_argument("--side-stream", action="store_true",
                    help="run the value gather as a launch of its own on a second stream (default: it shares the "
                         "launch of the attention's key phase)")
    ap.add_argument("--copies", type=int, default=1,
                    help="copies of the layer's tensors used in turn (defeats reuse of the previous step's data in "
                         "the last-level cache; default 1 = the one layer the configurations name)")
    ap.add_argument("--no-graph", action="store_true", help="enqueue the timed steps eagerly instead of replaying a HIP graph")
    ap.add_argument("--force-graph", action="store_true",
                    help="replay a HIP graph also where the default is eager (--side-stream)")
    ap.add_argument("--chunk-cache", action="store_true",
                    help="run shadowkv_decode_step_cached over a ring of correlated queries (values fetched only for "
                         "chunks missing from last step's selection); meant for the host-store workloads")
    ap.add_argument("--cache-slots", type=int, default=0,
                    help="slots per (sequence, KV head) of the chunk cache (default: topk_chunks = last selection only)")
    ap.add_argument("--rho-q", type=float, default=0.93, help="step-to-step correlation of the queries with --chunk-cache")
    ap.add_argument("--append", type=int, default=0, metavar="N",
                    help="lay the context arrays out with room for N more chunks and time N shadowkv_append_chunk calls "
                         "after the decode measurement (reported as append_chunk_ms)")
    ap.add_argument("--kv-dtype", choices=["bf16", "fp8"], default="bf16",
                    help="storage type of the KV-cache tensors: bf16, or FP8 E5M2 (the paper's second precision)")
    ap.add_argument("--factorize", action="store_true",
                    help="also time shadowkv_factorize_keys (the SVD line of the pre-filling algorithm) on the workload's "
                         "pre-RoPE keys (reported as factorize_ms, with the Gram kernel's fp64 matrix rate)")
    ap.add_argument("--stage-values", action="store_true",
                    help="stage the selected values with the gather kernel even for an HBM store "
                         "(gives profiles a plain copy kernel of known size: k*c*d*2 bytes per unit each way)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2
    if args.workload == "all":
        # one child process per configuration (nothing in this process has touched the GPU), their lines passed on
        import subprocess
        rc = 0
        for name in ("c1", "c2", "c3-host", "c3-hbm", "c4", "c5"):
            argv = [sys.executable, os.path.abspath(__file__)]
            skip = False
            for a in sys.argv[1:]:
                if skip:
                    skip = False
                elif a == "--workload":
                    skip = True
                elif not a.startswith("--workload="):
                    argv.append(a)
            r = subprocess.run(argv + ["--workload", name])
            rc = rc or r.returncode
        return rc

    import torch
    from paper_2410_21465_amd import shadowkv as S
    from workloads import (CONFIGS, EXTRA_CONFIGS, generate, generated_chunk, query_sequence, to_fp8_storage,
                                                with_capacity)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    wl = {**CONFIGS, **EXTRA_CONFIGS}[args.workload]
    dev = "cuda"
    t0 = time.time()
    print(f"[bench] drawing {wl.name}", file=sys.stderr, flush=True)
    t = generate(wl, device=dev, want_k_pre=args.factorize)
    ctx_cap = wl.ctx_len + args.append * wl.chunk_size
    if args.append:
        t = with_capacity(t, wl, ctx_cap)
    fp8 = args.kv_dtype == "fp8"
    kv_dtype = S.KV_FP8_E5M2 if fp8 else S.KV_BF16
    t_bf16 = t
    if fp8:
        t = to_fp8_storage(t)
        t_bf16 = {"A": t_bf16["A"], "B": t_bf16["B"]} if args.append else None   # generated_chunk draws from these
    print("[bench] inputs drawn", file=sys.stderr, flush=True)
    p = S.Params.from_workload(wl, flags=S.FLAG_STAGE_VALUES if args.stage_values else 0,
                               ctx_capacity=ctx_cap if args.append else 0, kv_dtype=kv_dtype)
    # pre-filling algorithm (after the SVD) through the library itself
    torch.cuda.synchronize()
    tb = time.time()
    bl = S.build_landmarks(p, t["k_rope"], t["v"])
    torch.cuda.synchronize()
    build_ms_first = (time.time() - tb) * 1e3
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(3):
        S.build_landmarks(p, t["k_rope"], t["v"], workspace=bl["workspace"])
    ev1.record()
    torch.cuda.synchronize()
    build_ms = ev0.elapsed_time(ev1) / 3
    setup_s = time.time() - t0
    print(f"[bench] landmarks built ({build_ms:.3f} ms per call)", file=sys.stderr, flush=True)

    ws = S.alloc_workspace(S.decode_workspace_bytes(p))
    out = torch.empty(wl.batch, wl.n_q_heads, wl.head_dim, dtype=torch.bfloat16, device=dev)
    ids = torch.empty(wl.batch, wl.n_kv_heads, wl.topk_chunks, dtype=torch.int32, device=dev)
    side = torch.cuda.Stream() if args.side_stream else None
    pool = t["q_pool"]
    cache = None
    if args.chunk_cache:
        pool = query_sequence(wl, 64, args.rho_q, device=dev)   # a ring: replaying it has no jump at the wrap
        cache = S.ValueCache(p, slots=args.cache_slots or None, device=dev)

    # --copies N: N copies of the layer's device tensors, used in turn, so that no step finds the previous step's
    # data in the 256 MB last-level cache (what a model with many layers would see); the default is the single
    # layer the benchmark configurations name.
    def layer_copy():
        def dup(x):
            return x.clone() if x.device.type == "cuda" else x      # a pinned host store is shared: it is not cached
        return ({k: dup(t[k]) for k in ("A", "B", "k_local", "v_local", "v")},
                {k: dup(bl[k]) for k in ("landmarks", "landmark_chunk_ids", "k_outlier", "v_outlier")})
    layers = [(t, bl)] + [layer_copy() for _ in range(max(args.copies, 1) - 1)]
    if len(layers) > 1 and (args.chunk_cache or args.append):
        print("bench.py: --copies is for the plain decode step only", file=sys.stderr)
        return 2

    def step(i: int):
        if cache is not None:
            S.decode_step_cached(p, pool[i % pool.shape[0]], t["A"], t["B"], bl["landmarks"], bl["landmark_chunk_ids"],
                                 bl["k_outlier"], bl["v_outlier"], t["k_local"], t["v_local"], t["v"], cache,
                                 t["pos_offset"], out=out, out_chunk_ids=ids, workspace=ws, side_stream=side)
            return
        lt, lb = layers[i % len(layers)]
        S.decode_step(p, pool[i % pool.shape[0]], lt["A"], lt["B"], lb["landmarks"], lb["landmark_chunk_ids"],
                      lb["k_outlier"], lb["v_outlier"], lt["k_local"], lt["v_local"], lt["v"], t["pos_offset"],
                      out=out, out_chunk_ids=ids, workspace=ws, side_stream=side)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # Timed region.  Default: the decode steps are captured once into a HIP graph (one graph = one pass over
    # the query pool, i.e. len(pool) consecutive steps with different queries) and replayed, which removes the
    # host launch gaps between the five kernels of a step; --no-graph enqueues every step eagerly instead.
    n_pool = pool.shape[0]
    graph = None
    # With --side-stream a step whose values come through a gather forks to the second stream; a replayed HIP
    # graph does not overlap the two branches on this runtime (measured: replay = serial time), so such runs
    # are timed with eager enqueues unless --force-graph is given.
    two_phase = side is not None and (wl.value_location == "host" or args.chunk_cache or args.stage_values)
    use_graph = not args.no_graph and (args.force_graph or not two_phase)
    if use_graph and args.steps >= n_pool:
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(cap):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=cap):
                for i in range(n_pool):
                    step(i)
        torch.cuda.current_stream().wait_stream(cap)
        graph.replay()                      # one untimed replay
        torch.cuda.synchronize()
    n_rep, n_eager = (args.steps // n_pool, args.steps % n_pool) if graph is not None else (0, args.steps)
    # exactly args.steps steps between two synchronisations; an event after every graph replay (one pass over the
    # query pool) or eager step gives the distribution, and the median of those per-step times is what is reported
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_rep + n_eager + 1)]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    marks[0].record()
    for j in range(n_rep):
        graph.replay()
        marks[j + 1].record()
    for i in range(n_eager):
        step(i)
        marks[n_rep + i + 1].record()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    ms_per_step_mean = (t2 - t1) * 1e3 / args.steps
    import statistics
    per_step = [marks[j].elapsed_time(marks[j + 1]) / (n_pool if j < n_rep else 1) for j in range(n_rep + n_eager)]
    # (median over the replays when there are any: the few eager steps behind them carry host launch gaps)
    ms_per_step = statistics.median(per_step[:n_rep]) if n_rep else statistics.median(per_step)
    value = wl.batch / (ms_per_step * 1e-3)
    print(f"[bench] timed steps done (median {ms_per_step:.4f} ms per step, mean {ms_per_step_mean:.4f})", file=sys.stderr, flush=True)

    # Per-stage times: the same number of steps again, eagerly, with HIP events at the stage boundaries.
    S.profile_begin(args.steps)
    t3 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    eager_ms_per_step = (time.perf_counter() - t3) * 1e3 / args.steps
    prof = S.profile_end()

    hit_rate = None
    if cache is not None:   # one more pass over the ring, reading the miss counts back after every step
        miss = []
        for i in range(pool.shape[0]):
            step(args.steps + i)
            miss.append(float(cache.miss_count.float().mean().item()) / wl.topk_chunks)
        hit_rate = 1.0 - sum(miss) / len(miss)

    factorize = None
    if args.factorize:   # A, B <- SVD(K) through the library (untimed part of set-up in the paper; timed here on request)
        kp = t["k_pre"].to(torch.float8_e5m2) if fp8 else t["k_pre"]
        pf = S.Params.from_workload(wl, kv_dtype=kv_dtype)
        f = S.factorize_keys(pf, kp)
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(2):
            S.factorize_keys(pf, kp, workspace=f["workspace"])
        ev1.record()
        torch.cuda.synchronize()
        fms = ev0.elapsed_time(ev1) / 2
        Dk = wl.key_width
        nb = (Dk + 63) // 64
        gram_flop = 2.0 * wl.batch * wl.ctx_len * (nb * (nb + 1) // 2) * 64 * 64
        factorize = {"ms": fms, "gram_fp64_flop": gram_flop, "projection_fp64_flop": 2.0 * wl.batch * wl.ctx_len * Dk * wl.rank}
        del f, kp

    append_ms = None
    if args.append:   # grow the context chunk by chunk (the step after decode once c tokens left the window)
        chunks = [generated_chunk(wl, t_bf16, i, device=dev) for i in range(min(args.append, 4))]
        if fp8:
            chunks = [tuple(x.to(torch.float8_e5m2) for x in ch) for ch in chunks]
        torch.cuda.synchronize()
        ev0.record()
        for i in range(args.append):
            kp, kr, vv = chunks[i % len(chunks)]
            pa = S.Params.from_workload(wl, ctx_len=wl.ctx_len + i * wl.chunk_size, ctx_capacity=ctx_cap, kv_dtype=kv_dtype)
            S.append_chunk(pa, kp, kr, vv, t["B"], t["A"], bl["landmarks"], bl["landmark_chunk_ids"], t["v"])
        ev1.record()
        torch.cuda.synchronize()
        append_ms = ev0.elapsed_time(ev1) / args.append

    # what a plain device copy reaches on this machine (1 GiB, read + write counted), for scale
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ev0.record()
    for _ in range(10):
        dst.copy_(src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbps = 10 * 2 * src.numel() / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del src, dst
    h2d_gbps = None
    if wl.value_location == "host":   # what a plain pinned-host -> device copy reaches (the link the gather reads over)
        hsrc = torch.empty(1 << 28, dtype=torch.uint8, pin_memory=True)
        ddst = torch.empty(1 << 28, dtype=torch.uint8, device=dev)
        ddst.copy_(hsrc, non_blocking=True)
        ev0.record()
        for _ in range(4):
            ddst.copy_(hsrc, non_blocking=True)
        ev1.record()
        torch.cuda.synchronize()
        h2d_gbps = 4 * hsrc.numel() / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
        del hsrc, ddst

    eb = 1 if fp8 else 2
    ab = algorithmic_bytes(wl, eb)
    score_ms = prof["ms"]["score"]
    score_bytes = ab["landmarks"] + ab["q_out"] // 2
    achieved = score_bytes / (score_ms * 1e-3) / 1e9
    # HBM bytes per launch by the chip's counters: a figure stored with the profiles (this run collects no
    # counters), with the file and the commit it was collected at
    tag = wl.name + ("-fp8" if fp8 else "")

    def stored_traffic(kernel):
        path = os.path.join(ROOT, "profiles", f"{kernel}_{tag}_traffic.txt")   # committed rocprofv3 --pmc summary
        val, commit = None, None
        if os.path.exists(path):
            for line in open(path):
                if line.startswith("hbm_bytes_per_launch:"):
                    val = int(line.split(":")[1])
                if line.startswith("collected_at_commit:"):
                    commit = line.split(":")[1].strip()
        src = (f"profiles/{os.path.basename(path)}: rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE scaled by a copy kernel of known "
               f"size, collected at commit {commit}; not measured by this run") if val is not None else None
        return val, src
    traffic, traffic_src = stored_traffic("score_kernel")
    # the other memory-bound stages: attention + combine (gathered A rows and values, resident keys and values, B,
    # queries, outputs) and the pre-filling call (every context key read once, every landmark written once)
    plan = S.decode_plan(p)
    # (where the resident rows are attended over by extra workgroups of the selection launch, their bytes are not
    # the attention stage's)
    res_in_select = plan["resident_rows_in_selection_launch"] and cache is None
    attn_bytes = (ab["A_rows"] + ab["B"] + ab["q_out"] + (0 if res_in_select else ab["resident_kv"])
                  + (ab["values"] if wl.value_location == "hbm" else 0))
    attn_ms = prof["ms"]["attention"]
    attn_traffic, attn_src = stored_traffic("attention")
    build_bytes = wl.units * eb * wl.head_dim * (wl.ctx_len + wl.n_landmarks + 2 * 2 * wl.n_outlier_chunks * wl.chunk_size)
    rooflines = [
        {"kernel": "score_kernel (landmark scoring, P = Q L^T)", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS,
         "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_src,
         "algorithmic_bytes_per_launch": score_bytes, "avg_launch_ms": score_ms},
        {"kernel": "sparse attention + combine (key rebuild, RoPE, softmax x V over selected and resident rows)"
                   + ("; selected values arrive over PCIe and are not counted" if wl.value_location == "host" else ""),
         "bound": "hbm", "achieved": attn_bytes / (attn_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
         "frac": attn_bytes / (attn_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, "traffic": attn_traffic, "traffic_source": attn_src,
         "algorithmic_bytes_per_launch": attn_bytes, "avg_launch_ms": attn_ms},
        {"kernel": "shadowkv_build_landmarks (chunk_stats_kernel + outlier selection + gathers; once per context)",
         "bound": "hbm", "achieved": build_bytes / (build_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
         "frac": build_bytes / (build_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, "traffic": None, "traffic_source": None,
         "algorithmic_bytes_per_launch": build_bytes, "avg_launch_ms": build_ms},
    ]
    res = {
        "metric": "decode_tokens_per_s", "value": value, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "ms_per_step_mean": ms_per_step_mean,
        "ms_per_step_statistic": f"median over {n_rep} graph replays of {n_pool} steps" if n_rep else f"median over {n_eager} eager steps",
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: batch {wl.batch} x context {wl.ctx_len}, {wl.n_q_heads}q/{wl.n_kv_heads}kv "
                               f"heads, d={wl.head_dim}, c={wl.chunk_size}, r={wl.rank}, k={wl.topk_chunks}, "
                               f"o={wl.n_outlier_chunks}, w={wl.local_len}, values in {wl.value_location}"
                               + (", KV cache stored as FP8 E5M2" if fp8 else ""),
                   "layers": 1, "tensor_copies": len(layers), "side_stream": side is not None, "kv_storage": "fp8_e5m2" if fp8 else "bf16"},
        "roofline": {"kernel": "score_kernel (landmark scoring, P = Q L^T)", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "traffic_source": traffic_src,
                     "algorithmic_bytes_per_launch": score_bytes, "avg_launch_ms": score_ms,
                     # the same launch priced on the fp64 matrix pipe it computes on (4 heads x d FMAs per landmark row
                     # and head group): what bounds it once the landmarks are one byte per element
                     "fp64_mfma_tflops": 2.0 * wl.units * ((wl.group + 3) // 4) * 4 * wl.n_landmarks * wl.head_dim
                                         / (score_ms * 1e-3) / 1e12,
                     "fp64_mfma_peak_tflops": 78.6},
        "rooflines": rooflines,
        "launch_plan": plan,
        "stage_ms": prof["ms"],
        "timed_region": "hip-graph replay" if graph is not None else "eager",
        "eager_ms_per_step_with_events": eager_ms_per_step,
        "step_algorithmic_bytes": ab["total"],
        "step_hbm_gbps": ab["total"] / (ms_per_step * 1e-3) / 1e9,
        "build_landmarks_ms": build_ms,
        "device_copy_gbps": copy_gbps,
        "append_chunk_ms": append_ms,
        "factorize_keys": factorize,
        "setup_s": setup_s,
    }
    if wl.value_location == "host":
        res["value_gather_pcie_bytes"] = ab["values"]
        res["pinned_h2d_copy_gbps"] = h2d_gbps
        res["value_gather_pcie_gbps"] = ab["values"] / (prof["ms"]["gather_values"] * 1e-3) / 1e9
    if wl.value_location == "host":
        # the paper's model with this machine's own rates: measured device copy and pinned-host copy, measured hit rate
        res["paper_model_equivalent_bandwidth_gbps"] = equivalent_bandwidth(
            wl.ctx_len, wl.chunk_size, wl.topk_chunks, wl.n_outlier_chunks, hit_rate or 0.0, copy_gbps, h2d_gbps)
    if cache is not None:
        res["config"]["chunk_cache"] = True
        res["config"]["cache_slots"] = cache.slots
        res["config"]["rho_q"] = args.rho_q
        res["cache_hit_rate"] = hit_rate
        if wl.value_location == "host":
            res["value_gather_pcie_bytes"] = ab["values"] * (1.0 - hit_rate)
            res["value_gather_pcie_gbps"] = res["value_gather_pcie_bytes"] / (prof["ms"]["gather_values"] * 1e-3) / 1e9

    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl, t, args.cpu_seconds, 1 if fp8 else 0)
    print(json.dumps(res), flush=True)
    return 0


def cpu_baseline(wl, t, budget_s: float, kv_dtype: int = 0) -> dict:
    """The CPU oracle, as it stands, on the first sequences of the same workload."""
    import numpy as np
    from oracle import shadowkv_oracle as O

    bs = min(wl.batch, 4)
    sub = wl.scaled(batch=bs)
    op = O.OracleParams(bs, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ctx_len, wl.chunk_size, wl.rank,
                        wl.n_outlier_chunks, wl.topk_chunks, wl.local_len, rope_theta=wl.rope_theta, kv_dtype=kv_dtype)

    def bits(x):
        return O.as_bits(x[:bs].detach().cpu(), kv_dtype)

    s_len = wl.ctx_len      # the oracle gets the dense layout (the arrays may have room to grow)
    t = dict(t, A=t["A"][:bs, :s_len].contiguous(), v=t["v"][:bs, :, :s_len].contiguous())
    k_rope, v = bits(t["k_rope"]), bits(t["v"])
    bl = O.build_landmarks(op, k_rope, v)
    del k_rope
    a = (bits(t["A"]), bits(t["B"]), bl["landmarks"], bl["landmark_chunk_ids"], bl["k_outlier"], bl["v_outlier"],
         bits(t["k_local"]), bits(t["v_local"]), v, t["pos_offset"][:bs].cpu().numpy())
    pool = t["q_pool"]
    def one_step(i):
        q = O.as_bits(pool[i % pool.shape[0]][:bs].detach().cpu())
        t0 = time.perf_counter()
        O.decode_step(op, q, *a, diagnostics=False)
        return time.perf_counter() - t0

    # all cores: at least 5 steps, then until two thirds of the budget are spent
    times = []
    while len(times) < 5 or (sum(times) < budget_s * 2 / 3 and len(times) < 1000):
        times.append(one_step(len(times)))
    reps, spent = len(times), sum(times)
    res = {"value": bs * reps / spent, "unit": "tokens/s", "cores": O.num_threads(), "kind": "oracle",
           "sample": f"first {bs} of {wl.batch} sequences of {sub.name}, {reps} decode steps on {O.num_threads()} threads, {spent:.1f} s",
           "ms_per_step": spent / reps * 1e3, "ms_per_step_median": sorted(times)[reps // 2] * 1e3, "steps": reps,
           "host_cores": os.cpu_count()}
    # the same oracle held to one thread (at least 3 steps), for a per-core figure
    try:
        import ctypes
        gomp = ctypes.CDLL("libgomp.so.1")
        n_thr = O.num_threads()
        gomp.omp_set_num_threads(1)
        one = []
        while len(one) < 3 or (sum(one) < budget_s / 3 and len(one) < 100):
            one.append(one_step(len(one)))
        gomp.omp_set_num_threads(n_thr)
        res["one_thread"] = {"value": bs * len(one) / sum(one), "unit": "tokens/s", "cores": 1, "steps": len(one),
                             "ms_per_step": sum(one) / len(one) * 1e3}
    except OSError:
        pass
    return res


if __name__ == "__main__":
    sys.exit(main())
