#!/usr/bin/env python3
"""Benchmark of the boundary layout transform on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
hp_forward (source layout -> destination layout) followed by hp_backward
(destination gradients -> source layout) on the long-context workload (vision
DP8 -> LLM TP4 x CP8 zigzag, one 131072-token sample, hidden 5120, ~30 % image
tokens).  All buffers are resident in HBM before the timed region.  The metric
is effective HBM GB/s: algorithmic bytes of the two calls divided by their time.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def read_traffic(workload: str):
    """HBM bytes per launch measured with rocprofv3 counters, if a summary for
    this workload has been committed under profiles/ (key = value lines)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    out = {}
    if os.path.exists(path):
        for line in open(path):
            if "=" in line and not line.lstrip().startswith("#"):
                k, v = line.split("=", 1)
                try:
                    out[k.strip()] = float(v.split()[0])
                except (ValueError, IndexError):
                    pass
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=15)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="long_context",
                    choices=["tiny", "colocated4", "colocated4_dense", "long_context", "non_colocated", "large_scale"])
    ap.add_argument("--graph", action="store_true",
                    help="record one step into a HIP graph and time its replays (wall clock); kernel "
                         "durations still come from eager launches carrying events")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tune", action="store_true",
                    help="call hp_plan_tune (measured launch-shape search, ~0.5 s) before the warm-up instead of "
                         "keeping the launch shapes a new plan starts from")
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f32"], help="payload element type")
    ap.add_argument("--seq-shard", action="store_true",
                    help="destination TP ranks hold sequence shards instead of replicas (sequence parallelism)")
    ap.add_argument("--row-order", default="bsh", choices=["bsh", "sbh"],
                    help="destination buffers as [B,S,H] or [S,B,H] (row-strided when a rank holds several samples)")
    ap.add_argument("--accumulate", action="store_true",
                    help="backward adds into fp32 source accumulators (hp_backward_accumulate)")
    ap.add_argument("--per-microbatch", action="store_true",
                    help="one plan and one launch per microbatch instead of one batched plan")
    ap.add_argument("--option", action="append", default=[], metavar="KEY=INT",
                    help="library tuning knob, e.g. tile_bytes_fwd=4096 (see hp_set_option)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on ONE GPU: every source and destination rank is a buffer "
            "in one GPU's HBM and there is no multi-GPU path. Re-run with --gpus 1.")
        return 2

    import torch
    import paper_2605_27678_amd as hp
    from paper_2605_27678_amd import workloads as wl

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the transform has no CPU path")
        return 3
    torch.cuda.set_device(0)
    dev = "cuda:0"
    for kv in args.option:
        key, val = kv.split("=", 1)
        hp.hp_set_option(key, int(val))

    from dataclasses import replace
    w = wl.CONFIGS[args.workload]()
    if args.seq_shard:
        w = replace(w, dst=replace(w.dst, tp_mode=wl.TP_SEQ_SHARD))
    if args.row_order == "sbh":
        w = replace(w, dst=replace(w.dst, row_order=wl.ROW_SBH))
    if args.dtype == "f32":
        w = replace(w, maps=[replace(m, dtype=wl.DT_F32) for m in w.maps])
    tdtype = torch.float32 if args.dtype == "f32" else torch.bfloat16
    maps = w.maps
    H = maps[0].hidden
    log(f"[bench] workload {w.name}: {len(maps)} microbatch(es), hidden {H}")

    # ---- plans and resident buffers (one batched plan, or one plan per microbatch) ----
    torch.zeros(1, device=dev)                 # HIP context up before the plan build is timed
    t0 = time.perf_counter()
    if len(maps) > 1 and not args.per_microbatch:
        plans = [hp.hp_plan_create_batched(w.src, w.dst, maps)]
    else:
        plans = [hp.hp_plan_create(w.src, w.dst, m) for m in maps]
    plan_ms = (time.perf_counter() - t0) * 1e3 / len(plans)
    sets = []
    for i, p in enumerate(plans):
        rows = p.src_rows()
        src = [wl.random_bf16((r, H), w.seed * 100 + i * 7 + k, dev).to(tdtype) for k, r in enumerate(rows)]
        dst = [wl.random_bf16((p.info.dst_rows_per_buf, H), w.seed * 100 + 50 + j, dev).to(tdtype)
               for j in range(p.info.n_dst_bufs)]
        grad = [wl.random_bf16((p.info.dst_rows_per_buf, H), w.seed * 100 + 90 + j, dev).to(tdtype)
                for j in range(p.info.n_dst_bufs)]
        sgrad = [torch.zeros((r, H), dtype=torch.float32 if args.accumulate else tdtype, device=dev) for r in rows]
        ps, pd = p.pointer_arrays(src, dst)
        pgs, pgd = p.pointer_arrays_accum(sgrad, grad) if args.accumulate else p.pointer_arrays(sgrad, grad)
        sets.append(dict(plan=p, src=src, dst=dst, grad=grad, sgrad=sgrad, ps=ps, pd=pd, pgs=pgs, pgd=pgd))
    fwd_bytes = sum(p.info.fwd_bytes for p in plans)
    bwd_bytes = sum(p.info.bwd_accum_bytes if args.accumulate else p.info.bwd_bytes for p in plans)
    boundary = sum(p.info.boundary_bytes for p in plans)
    log(f"[bench] boundary {boundary / 1e6:.1f} MB, fwd {fwd_bytes / 1e9:.3f} GB, bwd {bwd_bytes / 1e9:.3f} GB, "
        f"{sum(p.info.n_tiles for p in plans)} tiles, plan build {plan_ms:.2f} ms")

    stream = torch.cuda.Stream()
    n_launch = len(sets)

    # ---- one-time launch-shape search on the resident buffers (not part of a step) ----
    tune_ms = None
    if args.tune:
        t0 = time.perf_counter()
        s = sets[0]                      # plans of one workload share their grids: tune one, copy its shapes
        if args.accumulate:              # tune on scratch accumulators: every candidate launch adds into them
            tmp = [torch.zeros((r, H), dtype=torch.float32, device=dev) for r in s["plan"].src_rows()]
            s["plan"].tune(s["src"], s["dst"], None, None, stream)
            s["plan"].tune_accumulate(s["grad"], tmp, stream)
            del tmp
        else:
            s["plan"].tune(s["src"], s["dst"], s["grad"], s["sgrad"], stream)
        for other in sets[1:]:
            for d in (0, 1, 2):
                other["plan"].set_launch(d, **s["plan"].get_launch(d))
        tune_ms = (time.perf_counter() - t0) * 1e3
    shapes = {"fwd": sets[0]["plan"].get_launch(0), "bwd": sets[0]["plan"].get_launch(2 if args.accumulate else 1)}
    log(f"[bench] launch shapes: fwd {shapes['fwd']}  bwd {shapes['bwd']}  (tune {tune_ms} ms)")

    def step():
        for s in sets:
            s["plan"].forward_raw(s["ps"], s["pd"], stream)
        for s in sets:
            if args.accumulate:
                s["plan"].backward_accumulate_raw(s["pgd"], s["pgs"], stream)
            else:
                s["plan"].backward_raw(s["pgd"], s["pgs"], stream)

    timed_step = step
    if args.graph:
        step()                                   # first launches outside the capture
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            step()
        timed_step = graph.replay
    for _ in range(args.warmup):
        timed_step()
    stream.synchronize()
    torch.cuda.synchronize()
    rehearsal = 0
    if n_launch > 1 and not args.graph:
        # A step of many launches queues hundreds of dispatches before the closing
        # synchronisation.  The first device-wide synchronisation after the first
        # queue that deep has been seen to take 35-40 ms once per process (host
        # side: the GPU trace shows the kernels back to back and long finished),
        # so one untimed pass of the same length goes first.
        rehearsal = args.steps
        for _ in range(rehearsal):
            timed_step()
        stream.synchronize()
        torch.cuda.synchronize()
    # Timed region: EXACTLY `steps` steps between two synchronisations -> `value`.
    t0 = time.perf_counter()
    for _ in range(args.steps):
        timed_step()
    enqueue_s = time.perf_counter() - t0       # host time to submit the steps (inside the timed region)
    stream.synchronize()
    stream_sync_s = time.perf_counter() - t0
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    log(f"[bench] timed region: submitted after {enqueue_s * 1e3:.3f} ms, stream synchronised after "
        f"{stream_sync_s * 1e3:.3f} ms, device synchronised after {total_s * 1e3:.3f} ms")
    # The same `steps` steps again, now with a HIP event pair attached to every
    # launch (stamped by the dispatch itself on the stream it runs on) -> kernel
    # durations for the roofline.  Kept out of the region above because the
    # runtime handles event-carrying dispatches one by one, which costs tens of
    # microseconds per launch when a step is many short launches.
    hp.hp_profile_enable(2 * n_launch * args.steps)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    stream.synchronize()
    torch.cuda.synchronize()
    total_events_s = time.perf_counter() - t0
    launches = hp.hp_profile_read(2 * n_launch * args.steps)
    hp.hp_profile_enable(0)
    assert len(launches) == 2 * n_launch * args.steps
    per_step = [launches[i * 2 * n_launch:(i + 1) * 2 * n_launch] for i in range(args.steps)]
    fwd_ms = [sum(ms for kind, ms in st if kind == 0) for st in per_step]     # kernel time per step
    bwd_ms = [sum(ms for kind, ms in st if kind != 0) for st in per_step]
    ms_per_step = total_s * 1e3 / args.steps
    value = (fwd_bytes + bwd_bytes) / (total_s / args.steps) / 1e9
    f_avg, b_avg = statistics.fmean(fwd_ms), statistics.fmean(bwd_ms)
    f_med, b_med = statistics.median(fwd_ms), statistics.median(bwd_ms)
    log(f"[bench] kernel time per step: fwd median {f_med:.4f} ms ({fwd_bytes / f_med / 1e6:.0f} GB/s), "
        f"bwd median {b_med:.4f} ms ({bwd_bytes / b_med / 1e6:.0f} GB/s); wall {ms_per_step:.4f} ms/step "
        f"({value:.0f} GB/s), of which the host spent {enqueue_s * 1e3 / args.steps:.4f} submitting; "
        f"wall with per-launch events {total_events_s * 1e3 / args.steps:.4f} ms/step")

    # ---- rebuilding the plan at step rate (token maps change every step): warm create + destroy ----
    t0 = time.perf_counter()
    for _ in range(20):
        q = hp.hp_plan_create_batched(w.src, w.dst, maps) if len(plans) == 1 and len(maps) > 1 \
            else hp.hp_plan_create(w.src, w.dst, maps[0])
        q.close()
    plan_rebuild_ms = (time.perf_counter() - t0) * 1e3 / 20
    log(f"[bench] plan create+destroy, warm: {plan_rebuild_ms:.3f} ms")

    # ---- plain device copy of the same byte count: practical ceiling ----
    n_copy = (fwd_bytes // 2) // 2
    a = torch.empty(n_copy, dtype=torch.bfloat16, device=dev)
    b = torch.empty_like(a)
    with torch.cuda.stream(stream):
        for _ in range(3):
            b.copy_(a)
        ce = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ce[0].record(stream)
        for _ in range(10):
            b.copy_(a)
        ce[1].record(stream)
    stream.synchronize()
    copy_gbps = 10 * 2 * n_copy * 2 / (ce[0].elapsed_time(ce[1]) * 1e-3) / 1e9
    del a, b
    log(f"[bench] plain copy of {2 * n_copy * 2 / 1e9:.2f} GB traffic: {copy_gbps:.0f} GB/s")

    # ---- the access pattern's own ceiling: plain linear arrays, same lanes and launch search, no tables ----
    p0i = sets[0]["plan"].info
    arr = max(int(min(boundary, 1 << 30)) // 4096 * 4096, 1 << 20)
    ceil_f, shape_f = hp.hp_probe_stream(1, min(p0i.dst_copies, 8), arr)
    ceil_b, shape_b = hp.hp_probe_stream(min(p0i.dst_copies, 8), min(p0i.src_copies, 8), arr)   # (overwriting backward)
    log(f"[bench] pattern ceilings: 1R:{p0i.dst_copies}W {ceil_f:.0f} GB/s {shape_f}; "
        f"{p0i.dst_copies}R:{p0i.src_copies}W {ceil_b:.0f} GB/s {shape_b}")

    # ---- roofline of the dominant (slower) kernel: algorithmic bytes per launch / average launch duration ----
    dominant = "hp_backward_kernel" if b_avg >= f_avg else "hp_forward_kernel"
    dom_bytes = (bwd_bytes if dominant == "hp_backward_kernel" else fwd_bytes) / n_launch
    dom_ms = (b_avg if dominant == "hp_backward_kernel" else f_avg) / n_launch
    # the committed counter summary describes the workload's plain configuration only
    plain = args.dtype == "bf16" and not (args.accumulate or args.seq_shard or args.per_microbatch) \
        and args.row_order == "bsh"
    traffic = read_traffic(w.name) if plain else {}
    tkey = "backward_bytes_per_launch" if dominant == "hp_backward_kernel" else "forward_bytes_per_launch"
    roofline = {
        "bound": "hbm", "kernel": dominant,
        "achieved": dom_bytes / dom_ms / 1e6, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": dom_bytes / dom_ms / 1e6 / HBM_PEAK_GBPS,
        "traffic": traffic.get(tkey),
        "bytes_moved_per_boundary_byte": traffic.get(tkey.replace("_bytes_per_launch", "_bytes_per_boundary_byte")),
        "algorithmic_bytes_per_boundary_byte": dom_bytes * n_launch / boundary if boundary else None,
        "algorithmic_bytes_per_launch": dom_bytes,
        "avg_launch_ms": dom_ms,
    }

    # ---- the CPU oracle on the same workload, host cores of this machine ----
    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import oracle
        import numpy as np
        log("[bench] timing the CPU oracle on the same workload (first microbatch) ...")
        s, m = sets[0], maps[0]
        prob = oracle.Problem(w.src, w.dst, m)
        if args.dtype == "f32":
            host = lambda t: t.cpu().contiguous().numpy()
            same = lambda a, b: np.array_equal(a.view(np.uint32), b.view(np.uint32))
            ndt = np.float32
        else:
            host = lambda t: t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
            same = np.array_equal
            ndt = np.uint16
        n_s, n_d = w.src.n_ranks, w.dst.n_ranks            # microbatch 0 = the first buffers of the set
        if args.accumulate:
            # the accumulators have been added to an unknown number of times: start them from zero
            # and run one more hp_backward_accumulate, the call the oracle is compared with
            for t in s["sgrad"]:
                t.zero_()
            torch.cuda.synchronize()
            s["plan"].backward_accumulate_raw(s["pgd"], s["pgs"], stream)
            stream.synchronize()
        h_src = [host(t) for t in s["src"][:n_s]]
        h_dst = [host(t) for t in s["dst"][:n_d]]
        h_grad = [host(t) for t in s["grad"][:n_d]]
        ncores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
        ncores = min(ncores, int(os.environ.get("OMP_NUM_THREADS", ncores)))
        res = {}
        for nt in (ncores, 1):
            h_sg = [np.zeros((r, H), np.float32 if args.accumulate else ndt) for r in prob.src_rows()]
            oracle.set_threads(nt)
            t0 = time.perf_counter()
            prob.forward(h_src, h_dst)
            t1 = time.perf_counter()
            if args.accumulate:
                prob.backward_accumulate(h_grad, h_sg)
            elif args.dtype == "f32":
                prob.backward_f32(h_grad, h_sg)
            else:
                prob.backward_bf16(h_grad, h_sg)
            t2 = time.perf_counter()
            res[nt] = (t1 - t0, t2 - t1)
            log(f"[bench] oracle {nt} thread(s): fwd {t1 - t0:.3f} s, bwd {t2 - t1:.3f} s")
        p0 = s["plan"].info
        ob = (1 + p0.dst_copies) * m.n_rows * p0.row_bytes + (
            p0.dst_copies * m.n_rows * p0.row_bytes + p0.src_copies * 2 * m.n_rows * H * 4 if args.accumulate
            else (p0.dst_copies + p0.src_copies) * m.n_rows * p0.row_bytes)
        cpu_baseline = {
            "value": ob / sum(res[ncores]) / 1e9, "unit": "GB/s", "cores": ncores, "kind": "oracle",
            "sample": f"one full forward+backward pass of {w.name} (microbatch 0), {ob / 1e9:.2f} GB algorithmic",
            "fwd_s": res[ncores][0], "bwd_s": res[ncores][1],
            "one_thread_value": ob / sum(res[1]) / 1e9, "one_thread_fwd_s": res[1][0], "one_thread_bwd_s": res[1][1],
        }
        # The GPU results of the last step must equal what the oracle just computed: the source
        # gradients everywhere, the destination buffers on every image-token row (the oracle's
        # forward has just rewritten those rows of the GPU's own output; text rows are whatever
        # the random prefill was).
        if args.accumulate:                                    # binary32 accumulators whatever the gradients' dtype
            ok_b = all(np.array_equal(t.cpu().numpy().view(np.uint32), h.view(np.uint32))
                       for t, h in zip(s["sgrad"][:n_s], h_sg))
        else:
            ok_b = all(same(host(t), h) for t, h in zip(s["sgrad"][:n_s], h_sg))
        ok_f = all(same(host(t), h) for t, h in zip(s["dst"][:n_d], h_dst))
        cpu_baseline["gpu_matches_oracle"] = bool(ok_b and ok_f)
        cpu_baseline["gpu_matches_oracle_forward"] = bool(ok_f)
        cpu_baseline["gpu_matches_oracle_backward"] = bool(ok_b)

    out = {
        "metric": "boundary fwd+bwd effective HBM GB/s and % of MI355X HBM peak, 1 GPU",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": w.name, "src": f"tp{w.src.tp}dp{w.src.dp}",
                   "dst": f"tp{w.dst.tp}cp{w.dst.cp}dp{w.dst.dp}",
                   "batch": maps[0].batch, "seq": maps[0].seq, "hidden": H, "microbatches": len(maps),
                   "tp_mode": "seq_shard" if args.seq_shard else "replicate", "row_order": args.row_order,
                   "backward": "accumulate_f32" if args.accumulate else "overwrite",
                   "accumulate_dtype": "f32", "launches_per_direction": n_launch, "launch_shapes": shapes, "tuned": args.tune,
                   "submission": "hip_graph_replay" if args.graph else "eager",
                   "image_rows": int(sum(m.n_rows for m in maps)), "boundary_bytes": boundary,
                   },
        "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBPS,
        "forward": {"bytes": fwd_bytes, "median_ms": f_med, "min_ms": min(fwd_ms), "max_ms": max(fwd_ms),
                    "GBps": fwd_bytes / f_med / 1e6, "pct_of_hbm_peak": fwd_bytes / f_med / 1e6 / HBM_PEAK_GBPS * 100},
        "backward": {"bytes": bwd_bytes, "median_ms": b_med, "min_ms": min(bwd_ms), "max_ms": max(bwd_ms),
                     "GBps": bwd_bytes / b_med / 1e6, "pct_of_hbm_peak": bwd_bytes / b_med / 1e6 / HBM_PEAK_GBPS * 100},
        "ms_per_step_with_kernel_events": total_events_s * 1e3 / args.steps,
        "host_submit_ms_per_step": enqueue_s * 1e3 / args.steps,
        "ms_per_step_to_stream_sync": stream_sync_s * 1e3 / args.steps,
        "untimed_rehearsal_steps": rehearsal,
        "plan_build_ms": plan_ms, "plan_rebuild_ms": plan_rebuild_ms, "plan_tune_ms": tune_ms,
        "device_copy_GBps": copy_gbps,
        "pattern_ceiling": {"forward_GBps": ceil_f, "backward_GBps": ceil_b, "array_bytes": arr,
                            "forward_shape": shape_f, "backward_shape": shape_b},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
