#!/usr/bin/env python3
"""Benchmark of the tiered sequence-embedding lookup on one MI355X.

One step = one pass of the whole hot path over one synthetic batch resident in HBM:
  fs_plan_replication (histogram of the batch + top-k under a budget)
  -> fs_route_bucketize -> fs_sort_lookups (the batch's lookups in row order, once)
  -> fs_seq_gather_fwd (all buckets) -> fs_seq_grad_bwd_sorted (all buckets).
Prints ONE JSON line: lookups/s over the whole step on c3 (the configuration the bandwidth target is
stated on), the roofline of the dominant kernel (timed live with HIP events around each launch), the
roofline of every entry point as a whole call (`roofline.calls`), the CPU oracle timed on a bounded
sample, and -- when no --config is given -- the same step on c4 (the largest single-GPU shard) and the
c5 planning pass (10^9 sampled ids through the histogram, then the top-k) under `also_configs`.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c3] [--variant 0|1]
"""
from __future__ import annotations

import argparse
import ctypes
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default=None,
                    help="c1..c5; default: c3 (the configuration the target is stated on), followed by c4 and the "
                         "c5 planning pass under also_configs")
    ap.add_argument("--variant", type=int, default=0, help="backward: 0 sort/bit-exact, 1 atomic partials")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step in a HIP graph and time its replays (for small, launch-bound batches); the "
                         "per-kernel events of the roofline then come from an eager pass after the timed region")
    ap.add_argument("--overlap-plan", action="store_true",
                    help="run the plan on a second stream beside the lookup path (1-2 %% faster per step, but the "
                         "gather then shares the chip and its own duration grows)")
    ap.add_argument("--gather-order", default="auto", choices=("auto", "bucket", "row"),
                    help="order in which the forward gather takes the lookups: as routed, as sorted, or whichever is "
                         "faster on this workload (timed once before the warm-up)")
    ap.add_argument("--no-exchange", action="store_true", help="skip the untimed send / unbucketize / replica-store report")
    ap.add_argument("--no-also", action="store_true", help="skip c4 and the c5 planning pass of the default run")
    ap.add_argument("--c5-chunk", type=int, default=0,
                    help="ids per fs_plan_replication call of the c5 planning pass (0 = the whole sample in one call)")
    ap.add_argument("--cpu-tables", type=int, default=0, help="tables in the oracle's sample (0 = automatic)")
    ap.add_argument("--scale-rows", type=int, default=1, help="divide E by this (debugging only; reported)")
    return ap.parse_args()


def frac_of_peak(nbytes: float, ms: float) -> dict:
    gbs = nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
    return {"ms": round(ms, 4), "algorithmic_bytes": int(nbytes), "achieved": round(gbs, 1),
            "frac": round(gbs / HBM_PEAK_GBS, 4)}


def traffic_from_profiles(key: str):
    """HBM bytes per launch of one kernel as the committed rocprofv3 counter runs measured them
    (profiles/hbm_traffic.json: FETCH_SIZE and WRITE_SIZE, each scaled by a plain copy of known size).
    Returns (bytes or None, provenance or None): a figure of those profile runs, not of this run."""
    tfile = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        table = json.load(open(tfile))
    except Exception:
        return None, None
    entry = table.get(key)
    if entry is None:
        return None, None
    if isinstance(entry, dict):
        return entry.get("bytes"), {k: v for k, v in entry.items() if k != "bytes"}
    return entry, {"file": "profiles/hbm_traffic.json"}


def run_step_config(cfg, args, steps: int, warmup: int, full_report: bool):
    """The step on one configuration.  Returns (result fields, tensors the cpu baseline needs)."""
    import torch
    import fs_inputs
    import paper_2301_02959_amd as fs

    dev = "cuda:0"
    # ---------------------------------------------------------------- inputs, resident in HBM
    t_gen = time.time()
    batch = fs_inputs.make_batch(cfg, dev, keep_perms=False)
    placement = fs_inputs.make_placement(cfg, batch["perms"], dev)
    batch["perms"] = None
    n = batch["n"]
    ids, offsets, row_base = batch["ids"], batch["offsets"], batch["row_base"]
    weights = fs_inputs.make_table(cfg, dev)
    grad_out = fs_inputs.make_grad(cfg, n, dev)
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen
    R, D, U, W, T, B = cfg.R, cfg.D, cfg.U, cfg.W, cfg.T, cfg.B
    self_b = cfg.self_bucket
    row_bytes = cfg.row_bytes

    # ---------------------------------------------------------------- outputs and workspaces
    bucket_offsets = torch.zeros(U + 1, dtype=torch.int64, device=dev)
    out_rows = torch.zeros(n, dtype=torch.int64, device=dev)
    out_pos = torch.zeros(n, dtype=torch.int32, device=dev)
    tier_counts = torch.zeros(3, dtype=torch.int64, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    out = torch.empty(n, D, dtype=cfg.torch_dtype, device=dev)
    num_unique = torch.zeros(1, dtype=torch.int64, device=dev)
    counts = torch.zeros(R, dtype=torch.int32, device=dev)
    budget_rows = max(1, int((cfg.f_global if cfg.f_global > 0 else 0.01) * R))
    sel_rows = torch.zeros(budget_rows, dtype=torch.int64, device=dev)
    num_selected = torch.zeros(1, dtype=torch.int64, device=dev)
    plan_flags = fs.FS_PLAN_ACCUMULATE | fs.FS_PLAN_SELECT

    def ws_for(query):
        size = ctypes.c_size_t(0)
        query(size)
        return torch.empty(max(int(size.value), 256), dtype=torch.uint8, device=dev)

    L = fs.lib()
    z = ctypes.c_void_p(0)
    ws_route = torch.empty(max(fs.route_workspace_bytes(T, B, n, U, W, self_b), 256), dtype=torch.uint8, device=dev)

    def q_bwd(size):
        rc = L.fs_seq_grad_bwd(z, ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int(fs_inputs.DTYPE_CODE[cfg.dtype]),
                               z, z, ctypes.c_int64(0), ctypes.c_int64(n), ctypes.c_int64(R), ctypes.c_int32(args.variant),
                               z, z, ctypes.c_int64(cap_unique), z, z, ctypes.byref(size), z, z)
        assert rc == 0, rc

    def q_plan(size):
        rc = L.fs_plan_replication(z, z, ctypes.c_int32(T), ctypes.c_int32(B), z, ctypes.c_int64(n), ctypes.c_int64(R),
                                   z, ctypes.c_int32(plan_flags), ctypes.c_int64(budget_rows * row_bytes),
                                   ctypes.c_int64(row_bytes), z, z, z, z, ctypes.byref(size), z, z)
        assert rc == 0, rc

    def q_sort(size):
        rc = L.fs_sort_lookups(z, z, ctypes.c_int64(0), ctypes.c_int64(n), ctypes.c_int64(R), ctypes.c_int64(n), z, z,
                               z, ctypes.byref(size), z, z)
        assert rc == 0, rc

    def q_bwd_sorted(size):
        rc = L.fs_seq_grad_bwd_sorted(z, ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int(fs_inputs.DTYPE_CODE[cfg.dtype]),
                                      z, z, ctypes.c_int64(n), ctypes.c_int64(R), ctypes.c_int32(args.variant),
                                      z, z, ctypes.c_int64(cap_unique), z, z, ctypes.byref(size), z, z)
        assert rc == 0, rc

    cap_unique = 0
    ws_bwd = ws_for(q_bwd)
    ws_plan = ws_for(q_plan)
    ws_sort = ws_for(q_sort)
    ws_bwd_sorted = ws_for(q_bwd_sorted)
    sorted_rows = torch.zeros(n, dtype=torch.int32, device=dev)        # 32-bit words (uint32 on the C side)
    sorted_pos = torch.zeros(n, dtype=torch.int32, device=dev)

    # size row_grads to the batch: a first call with capacity 0 only counts the distinct rows
    fs.fs_route_bucketize(ids, offsets, T, B, row_base, placement, n, U, W, self_b, bucket_offsets, out_rows,
                          out_pos, tier_counts, status, workspace=ws_route)
    fs.fs_seq_grad_bwd(grad_out, out_rows, out_pos, 0, n, R, args.variant, None, None, 0, num_unique, None,
                       workspace=ws_bwd)
    torch.cuda.synchronize()
    cap_unique = int(num_unique.item())
    uniq_rows = torch.zeros(max(cap_unique, 1), dtype=torch.int64, device=dev)
    row_grads = torch.empty(max(cap_unique, 1), D, dtype=torch.float32, device=dev)

    # The plan (profiling histogram + top-k) neither reads nor writes anything the lookup path touches, so
    # with --overlap-plan it runs on a second stream beside route -> gather -> backward and joins at the
    # end of the step.  Default: everything on one stream, so that each kernel's duration is its own.
    main_stream = torch.cuda.current_stream()
    plan_stream = torch.cuda.Stream() if args.overlap_plan else main_stream
    plan_calls = [0]

    def plan():
        fs.fs_plan_replication(ids, offsets, T, B, row_base, n, R, counts, plan_flags, budget_rows * row_bytes,
                               row_bytes, sel_rows, num_selected, None, status, workspace=ws_plan)

    def route():
        fs.fs_route_bucketize(ids, offsets, T, B, row_base, placement, n, U, W, self_b, bucket_offsets, out_rows,
                              out_pos, tier_counts, status, workspace=ws_route)

    def gather():
        fs.fs_seq_gather_fwd(weights, out_rows, out_pos, 0, n, out, status)

    def backward():                                      # the backward that sorts for itself (not in the step)
        fs.fs_seq_grad_bwd(grad_out, out_rows, out_pos, 0, n, R, args.variant, uniq_rows, row_grads, cap_unique,
                           num_unique, status, workspace=ws_bwd)

    def sort_lookups():                                  # one sort per batch, in row order, for whoever wants it
        fs.fs_sort_lookups(out_rows, out_pos, 0, n, R, n, sorted_rows, sorted_pos, status, workspace=ws_sort)

    def backward_sorted():
        fs.fs_seq_grad_bwd_sorted(grad_out, sorted_rows, sorted_pos, n, R, args.variant, uniq_rows, row_grads,
                                  cap_unique, num_unique, status, workspace=ws_bwd_sorted)

    def gather_sorted():                                 # the gather in row order (not in the step)
        fs.fs_seq_gather_fwd_sorted(weights, sorted_rows, sorted_pos, n, out, status)

    # The forward gather may take the lookups in bucket order (as routed) or in row order (as sorted for the
    # backward).  Which is faster depends on the workload (whether the repeated rows fit the caches in bucket
    # order), so both are timed once, before the warm-up, and the step uses the faster one.
    gather_order = "bucket"
    fwd = gather
    if args.gather_order != "bucket":
        route(); sort_lookups()
        t_order = {}
        for name, fn in (("bucket", gather), ("row", gather_sorted)):
            fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(3):
                fn()
            e1.record()
            torch.cuda.synchronize()
            t_order[name] = e0.elapsed_time(e1) / 3
        if args.gather_order == "row" or (args.gather_order == "auto" and t_order["row"] < 0.98 * t_order["bucket"]):
            gather_order, fwd = "row", gather_sorted

    def step():
        plan_calls[0] += 1
        if plan_stream is not main_stream:
            plan_stream.wait_stream(main_stream)
            with torch.cuda.stream(plan_stream):
                plan()
        else:
            plan()                                       # on whatever stream is current (a graph capture's, too)
        route()
        sort_lookups()
        fwd()
        backward_sorted()
        if plan_stream is not main_stream:
            main_stream.wait_stream(plan_stream)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()

    # ---------------------------------------------------------------- timed region
    # HIP events bracket only the three bandwidth kernels the roofline is about (two event records per
    # timed launch are not free: with all launches of a step timed, the step is 4 % slower).
    gather_kernel = "gather_rows" if gather_order == "bucket" else "gather_sorted"
    roof_kernels = f"{gather_kernel},bwd_segreduce,bwd_singletons"
    records_per_step = 64
    if args.graph:
        # one step captured, replayed K times; HIP events recorded under capture do not yield times, so the
        # three bandwidth kernels are event-timed in K eager steps right after the timed replays
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()                                   # untimed: the first launch of a graph uploads it
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        fs.fs_prof_begin(records_per_step * steps, only=roof_kernels)
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
    else:
        fs.fs_prof_begin(records_per_step * steps, only=roof_kernels)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    roof_records = fs.fs_prof_end(records_per_step * steps)
    ms_per_step = (t1 - t0) * 1e3 / steps
    assert int(status.item()) == 0, f"device status {int(status.item())}"
    n_u = int(num_unique.item())

    # the same steps once more with an event between the entry points: each call as a whole, its launches
    # and the gaps between them included (not part of `value`)
    call_names = ("fs_plan_replication", "fs_route_bucketize", "fs_sort_lookups", "fs_seq_gather_fwd",
                  "fs_seq_grad_bwd_sorted", "fs_seq_grad_bwd", "fs_seq_gather_fwd_sorted")
    call_fns = (plan, route, sort_lookups, gather, backward_sorted, backward, gather_sorted)    # the last two: not in the step
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(len(call_fns) + 1)] for _ in range(steps)]
    for s in range(steps):
        marks[s][0].record()
        for k, fn in enumerate(call_fns):
            fn()
            marks[s][k + 1].record()
        plan_calls[0] += 1
    torch.cuda.synchronize()
    call_ms = {name: sum(marks[s][k].elapsed_time(marks[s][k + 1]) for s in range(steps)) / steps
               for k, name in enumerate(call_names)}

    # and once more with every launch timed, for the per-kernel breakdown
    fs.fs_prof_begin(records_per_step * steps)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    records = fs.fs_prof_end(records_per_step * steps)

    per_kernel = {}
    for name, ms in records:
        tot, cnt = per_kernel.get(name, (0.0, 0))
        per_kernel[name] = (tot + ms, cnt + 1)
    kernel_ms = {k: v[0] / steps for k, v in per_kernel.items()}                # per step (summed launches)
    launches_per_step = len(records) / steps
    roof = {}
    for name, ms in roof_records:
        tot, cnt = roof.get(name, (0.0, 0))
        roof[name] = (tot + ms, cnt + 1)
    kernel_avg = {k: v[0] / v[1] for k, v in roof.items()}                      # per launch, from the timed region
    stage_ms = {
        "plan": sum(v for k, v in kernel_ms.items() if k.startswith("plan_")),
        "route": sum(v for k, v in kernel_ms.items() if k.startswith("route_")),
        "gather": kernel_ms.get(gather_kernel, 0.0),
        "bwd": sum(v for k, v in kernel_ms.items() if k.startswith("bwd_")),
        "sort": sum(v for k, v in kernel_ms.items() if k.startswith("sort_")),
    }

    # algorithmic bytes per launch of the bandwidth kernels.  The backward's runs of one lookup (n_1 of
    # them, counted here with torch outside the timed region) are moved by bwd_singletons, the rest by
    # bwd_segreduce; both read the sorted (key, position) pairs.
    _, run_len = torch.unique(out_rows, return_counts=True)
    n_1 = int((run_len == 1).sum().item())
    del run_len
    k_sel = int(num_selected.item())
    alg = {
        gather_kernel: n * row_bytes + n_u * row_bytes + n * (12 if gather_order == "bucket" else 8),   # write out, read each distinct row once, indices
        "bwd_segreduce": (n - n_1) * row_bytes + (n_u - n_1) * D * 4 + n * 8,   # read grad_out once, write row_grads, sorted pairs
        "bwd_singletons": n_1 * row_bytes + n_1 * D * 4 + n * 4,                # one row in, one fp32 row out, the sorted keys
    }
    # algorithmic bytes of each entry point as a whole: what the operation must move, whatever the
    # kernels do on the way (the backward's sort traffic, the router's intermediate arrays and the plan's
    # candidate sort are overhead and count for nothing here)
    alg_calls = {
        "fs_seq_gather_fwd": n * row_bytes + n_u * row_bytes + n * 12,
        "fs_seq_grad_bwd": n * row_bytes + n_u * D * 4 + n * 12 + n_u * 8,      # grad_out once, row_grads once, (row, pos) in, uniq_rows out
        "fs_seq_grad_bwd_sorted": n * row_bytes + n_u * D * 4 + n * 8 + n_u * 8,
        "fs_seq_gather_fwd_sorted": n * row_bytes + n_u * row_bytes + n * 8,
        "fs_sort_lookups": n * (12 + 8),                                        # pairs in, pairs out: all of it overhead of the path
        "fs_route_bucketize": n * (8 + 4 + 8 + 4) + (T * B + 1) * 8,           # id and placement entry in, out_rows and out_pos out, offsets
        "fs_plan_replication": n * 8 + n_u * 8 + R * 4 + k_sel * 8,            # ids, one counter update per distinct row, counts once, selection out
    }
    dominant = max(alg, key=lambda k: kernel_avg.get(k, 0.0))
    achieved = alg[dominant] / (kernel_avg[dominant] * 1e-3) / 1e9
    traffic, traffic_source = traffic_from_profiles(f"{cfg.name}:{dominant}")
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_source": traffic_source,
                "algorithmic_bytes": alg[dominant], "avg_ms": round(kernel_avg[dominant], 4)}
    roofline["also"] = [{"kernel": k, "achieved": round(alg[k] / (kernel_avg[k] * 1e-3) / 1e9, 1),
                         "frac": round(alg[k] / (kernel_avg[k] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                         "algorithmic_bytes": alg[k], "avg_ms": round(kernel_avg[k], 4),
                         "traffic": traffic_from_profiles(f"{cfg.name}:{k}")[0]}
                        for k in alg if k != dominant and k in kernel_avg]
    roofline["calls"] = {name: frac_of_peak(alg_calls[name], call_ms[name]) for name in call_names}
    for name in ("fs_seq_grad_bwd", "fs_seq_gather_fwd_sorted" if gather_order == "bucket" else "fs_seq_gather_fwd"):
        roofline["calls"][name]["in_step"] = False       # timed beside the step's calls, for comparison

    result = {
        "ms_per_step": round(ms_per_step, 4),
        "value": round(n / (ms_per_step * 1e-3), 1),
        "config": {"workload": f"{cfg.name}: {T} tables x {cfg.E} rows x D={D} {cfg.dtype}, batch {B}, "
                               f"{cfg.length_law} lengths, Zipf({cfg.alpha}), {U} buckets (W={W})",
                   "lookups": n, "distinct_rows": n_u, "single_lookup_rows": n_1, "bwd_variant": args.variant,
                   "gather_order": gather_order,
                   "schedule": ("plan on a second stream beside route, gather, backward" if args.overlap_plan else "one stream")
                               + (", replayed from a HIP graph" if args.graph else ""),
                   "tier_counts": [int(x) for x in tier_counts.tolist()], "scale_rows": args.scale_rows},
        "roofline": roofline,
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        "launches_per_step": round(launches_per_step, 1),
        "kernel_ms_per_step": {k: round(v, 4) for k, v in sorted(kernel_ms.items())},
        "input_gen_s": round(t_gen, 1),
    }
    if not full_report:
        return result, None

    # what the tiers of this batch mean for the row exchange (the paper's headline quantity, its Section 6.2)
    _, traffic_report = fs.fs_tier_traffic(tier_counts.tolist(), D, cfg.row_bytes // D)
    result["row_exchange"] = {"bytes_if_all_sharded": int(traffic_report[0]), "global_all_to_all_bytes": int(traffic_report[1]),
                              "intra_group_all_to_all_bytes": int(traffic_report[2]),
                              "global_all_to_all_avoided": round(traffic_report[3], 4)}

    # ---------------------------------------------------------------- the box's plain-copy bandwidth, for context
    copy_bytes = min(out.numel() * out.element_size(), grad_out.numel() * grad_out.element_size()) // 16 * 16
    if copy_bytes > 0:
        for _ in range(2):
            fs.fs_util_copy(out, grad_out, copy_bytes)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            fs.fs_util_copy(out, grad_out, copy_bytes)
        e1.record()
        torch.cuda.synchronize()
        copy_ms = e0.elapsed_time(e1) / 5
        result["plain_copy"] = {"bytes_each_way": copy_bytes, "ms": round(copy_ms, 4),
                                "GBps_read_plus_write": round(2 * copy_bytes / (copy_ms * 1e-3) / 1e9, 1)}

    # the same for the backward's traffic shape: a read stream of 512-byte pieces with one 1 KB write per
    # run of the batch's average length (and with no writes at all), without any of the kernel's arithmetic
    src_bytes = grad_out.numel() * grad_out.element_size() // 512 * 512
    dst_elems = row_grads.numel() // 256 * 256                       # whole 1 KB rows of the fp32 buffer
    if src_bytes > 0 and dst_elems > 0:
        avg_run = max(1, min(256, int(round((n - n_1) / max(n_u - n_1, 1)))))
        mix = {}
        mix_src = grad_out.view(-1)[:src_bytes // grad_out.element_size()]
        mix_dst = row_grads.view(-1)[:dst_elems]
        for label, w in (("read_only", 0), ("read_with_writes", avg_run)):
            for _ in range(2):
                fs.fs_util_read_write_mix(mix_src, w, mix_dst if w else None)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                fs.fs_util_read_write_mix(mix_src, w, mix_dst if w else None)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 5
            moved = src_bytes + (src_bytes // 512 // 256 * (256 // w) * 1024 if w else 0)   # a group of 256 pieces writes 256 // w rows
            mix[label] = {"ms": round(ms, 4), "GBps": round(moved / (ms * 1e-3) / 1e9, 1),
                          **({"pieces_per_write": w, "write_share": round(1 - src_bytes / moved, 4)} if w else {})}
        result["reference_streams"] = mix

    # ---------------------------------------------------------------- the exchange halves and the replica store
    # Not part of the step or of `value`: the same lookups once more through fs_seq_gather_send +
    # fs_seq_unbucketize (the two sides of the row exchange) and through fs_seq_gather_fwd_replica (popular
    # rows served from the dense store that fs_replica_build fills from the plan's selection).
    need = n * row_bytes + budget_rows * row_bytes + R * 4
    if not args.no_exchange and torch.cuda.mem_get_info()[0] > 1.1 * need + (1 << 30):
        send = torch.empty(n, D, dtype=cfg.torch_dtype, device=dev)
        store = torch.empty(budget_rows, D, dtype=cfg.torch_dtype, device=dev)
        slots = torch.empty(R, dtype=torch.int32, device=dev)
        # ... and through the slot hand-over: the placement's tier-0 entries carry the replica slots
        # (fs_replica_tag_slots), the router hands each lookup's slot on (fs_route_bucketize_slots) and the gather
        # reads it beside the row and the position (fs_seq_gather_fwd_slots) instead of looking the row up in the
        # slot map
        placement_tagged = placement.clone()
        out_slots = torch.empty(n, dtype=torch.int32, device=dev)

        def q_route_slots(size):
            rc = L.fs_route_bucketize_slots(z, z, ctypes.c_int32(T), ctypes.c_int32(B), z, z, ctypes.c_int64(n),
                                            ctypes.c_int32(U), ctypes.c_int32(W), ctypes.c_int32(self_b), z, z, z, z, z, z,
                                            ctypes.byref(size), z, z)
            assert rc == 0, rc
        ws_route_slots = ws_for(q_route_slots)

        def xstep():
            fs.fs_replica_build(weights, sel_rows, budget_rows, num_selected, store, slots, status)
            fs.fs_seq_gather_send(weights, out_rows, 0, n, send, status)
            fs.fs_seq_unbucketize(send, out_pos, 0, n, out, status)
            fs.fs_seq_gather_fwd_replica(weights, store, budget_rows, slots, out_rows, out_pos, 0, n, out, status)
            fs.fs_replica_tag_slots(placement_tagged, slots, status)
            fs.fs_route_bucketize_slots(ids, offsets, T, B, row_base, placement_tagged, n, U, W, self_b, bucket_offsets,
                                        out_rows, out_pos, out_slots, tier_counts, status, workspace=ws_route_slots)
            fs.fs_seq_gather_fwd_slots(weights, store, budget_rows, out_rows, out_slots, out_pos, 0, n, out, status)

        for _ in range(2):
            xstep()
        reps = 5
        fs.fs_prof_begin(16 * reps)
        for _ in range(reps):
            xstep()
        torch.cuda.synchronize()
        xrec = {}
        for name, ms in fs.fs_prof_end(16 * reps):
            xrec[name] = xrec.get(name, 0.0) + ms / reps
        assert int(status.item()) == 0, f"device status {int(status.item())}"
        xalg = {"gather_send": n * row_bytes + n_u * row_bytes + n * 8,
                "unbucketize": 2 * n * row_bytes + n * 4,
                "gather_replica": n * row_bytes + n_u * row_bytes + n * 16,
                "gather_slots": n * row_bytes + n_u * row_bytes + n * 16}
        result["exchange_path"] = {
            "replica_rows": k_sel,
            "lookups_with_a_slot": int((out_slots >= 0).sum().item()),
            "kernels": {(k + " (with slots)" if k.startswith("route_") else k): {"ms": round(v, 4),
                            **({"GBps": round(xalg[k] / (v * 1e-3) / 1e9, 1),
                                "frac": round(xalg[k] / (v * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)} if k in xalg else {})}
                        for k, v in sorted(xrec.items())}}
        # the optimizer step that follows the backward: row-wise Adagrad on the deduplicated gradients,
        # mirrored into the replica store (lr = 0 keeps the table's bits for the legs below; the traffic is the same)
        opt_state = torch.zeros(R, dtype=torch.float32, device=dev)
        for i in range(2 + reps):
            if i == 2:
                fs.fs_prof_begin(4 * reps)
            fs.fs_sparse_update(weights, uniq_rows, row_grads, cap_unique, num_unique, fs.FS_OPT_ADAGRAD_ROWWISE, 0.0,
                                1e-8, opt_state, store, slots, budget_rows, status)
        torch.cuda.synchronize()
        upd_ms = sum(ms for _, ms in fs.fs_prof_end(4 * reps)) / reps
        upd_bytes = n_u * (D * 4 + 2 * row_bytes + 16)
        result["exchange_path"]["kernels"]["sparse_update"] = {
            "ms": round(upd_ms, 4), "GBps": round(upd_bytes / (upd_ms * 1e-3) / 1e9, 1),
            "frac": round(upd_bytes / (upd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "rule": "row-wise Adagrad"}
        # the backward and the optimizer step as two calls and as the one call that applies the step to rows
        # looked up once straight from grad_out (same bits in the table; lr = 0 again)
        def q_bwd_update(size):
            rc = L.fs_seq_grad_bwd_update(z, ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int(fs_inputs.DTYPE_CODE[cfg.dtype]),
                                          z, z, ctypes.c_int64(n), ctypes.c_int64(R), z, ctypes.c_int32(fs.FS_OPT_ADAGRAD_ROWWISE),
                                          ctypes.c_float(0.0), ctypes.c_float(1e-8), z, z, z, ctypes.c_int64(0), z, z,
                                          ctypes.c_int64(cap_unique), z, z, ctypes.byref(size), z, z)
            assert rc == 0, rc
        ws_fused = ws_for(q_bwd_update)

        def two_calls():
            backward_sorted()
            fs.fs_sparse_update(weights, uniq_rows, row_grads, cap_unique, num_unique, fs.FS_OPT_ADAGRAD_ROWWISE, 0.0,
                                1e-8, opt_state, store, slots, budget_rows, status)

        def one_call():
            fs.fs_seq_grad_bwd_update(grad_out, sorted_rows, sorted_pos, n, R, weights, fs.FS_OPT_ADAGRAD_ROWWISE, 0.0, 1e-8,
                                      opt_state, store, slots, budget_rows, uniq_rows, row_grads, cap_unique, num_unique,
                                      status, workspace=ws_fused)

        fused = {}
        for name, fn in (("fs_seq_grad_bwd_sorted + fs_sparse_update", two_calls), ("fs_seq_grad_bwd_update", one_call)):
            for _ in range(2):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            fused[name] = round(e0.elapsed_time(e1) / reps, 4)
        assert int(status.item()) == 0, f"device status {int(status.item())}"
        result["backward_with_optimizer_step_ms"] = fused
        del send, store, slots, opt_state, ws_fused

        # the tier planner on the counts accumulated so far (the one batch, profiled once per step run so
        # far, so the sample count is B times that); bandwidth ratios as in the paper's Figure 3
        # (all-reduce = 3 x all-to-all)
        tp = dict(num_samples=B * plan_calls[0], B=B, U=U, W=W, dp_multiplier=6, granule=32,
                  a2a_global=1, a2a_intra=6, ar_global=3, ar_cross=2)
        cuts = torch.zeros(fs.FS_TIER_CUTS, dtype=torch.int64, device=dev)
        tier_rows = torch.empty(R, dtype=torch.int64, device=dev)
        for tiers in (3, 3, 2):
            fs.fs_prof_begin(64)
            fs.fs_plan_tiers(counts, R, tp, tiers, tier_rows, R, cuts, None, status)
            torch.cuda.synchronize()
            trec = fs.fs_prof_end(64)
        c = [int(x) for x in cuts.tolist()]
        result["tier_plan"] = {
            "ms": round(sum(ms for _, ms in trec), 4),
            "kernels_ms": {k: round(sum(ms for nm, ms in trec if nm == k), 4) for k in sorted({nm for nm, _ in trec})},
            "params": tp, "two_tier": {"candidates": c[0], "A": c[1], "B": c[2], "C": c[3], "flex_breakpoint": c[4],
                                       "n_dp": c[5], "dp_share": round(c[8] / max(c[7], 1), 4)}}
        del tier_rows

    keep = (ids, offsets, placement, weights, grad_out)
    return result, keep


def run_c5_planning(args):
    """The planning configuration: 10^9 sampled ids (4 tables x 250 M, one segment per table) through
    fs_plan_replication's histogram in ONE call (the ids, 8 GB, are drawn on the GPU and resident when the
    timed region starts), then the top-k under a 4 GB budget at 256 bytes per row.  The call is timed with
    HIP events on its stream; `--c5-chunk N` splits the pass into calls of at most N ids instead."""
    import torch
    import fs_inputs
    import paper_2301_02959_amd as fs

    dev = "cuda:0"
    cfg = fs_inputs.CONFIGS["c5"]
    R, T = cfg.R, cfg.T
    per_table = 250_000_000
    counts = torch.zeros(R, dtype=torch.int32, device=dev)
    row_base = torch.arange(T + 1, dtype=torch.int64, device=dev) * cfg.E
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    budget, bpr = 4_000_000_000, 256
    cap = min(R, budget // bpr)
    sel = torch.zeros(cap, dtype=torch.int64, device=dev)
    nsel = torch.zeros(1, dtype=torch.int64, device=dev)

    def ws_of(flags, n):
        size = ctypes.c_size_t(0)
        z = ctypes.c_void_p(0)
        rc = fs.lib().fs_plan_replication(z, z, ctypes.c_int32(T), ctypes.c_int32(1), z, ctypes.c_int64(n),
                                          ctypes.c_int64(R), z, ctypes.c_int32(flags), ctypes.c_int64(budget),
                                          ctypes.c_int64(bpr), z, z, z, z, ctypes.byref(size), z, z)
        assert rc == 0, rc
        return torch.empty(max(int(size.value), 256), dtype=torch.uint8, device=dev)

    t_wall = time.time()
    parts = [ids for _, ids in fs_inputs.make_profile_sample(cfg, per_table, dev, chunk=per_table)]
    all_ids = torch.cat(parts)
    del parts
    seen = all_ids.numel()
    table_start = torch.arange(T + 1, dtype=torch.int64, device=dev) * per_table
    chunk = args.c5_chunk if args.c5_chunk > 0 else seen
    # the calls: [lo, hi) of the sample with the offsets of the tables inside it (one segment per table)
    calls = []
    for lo in range(0, seen, chunk):
        hi = min(seen, lo + chunk)
        calls.append((all_ids[lo:hi], (table_start.clamp(lo, hi) - lo).contiguous(), hi - lo))
    ws_acc = ws_of(fs.FS_PLAN_ACCUMULATE, max(c[2] for c in calls))
    ws_sel = ws_of(fs.FS_PLAN_SELECT, 0)

    def accumulate(into):
        for ids, offsets, m in calls:
            fs.fs_plan_replication(ids, offsets, T, 1, row_base, m, R, into, fs.FS_PLAN_ACCUMULATE, dev_status=status,
                                   workspace=ws_acc)

    warm = torch.zeros(R, dtype=torch.int32, device=dev)   # untimed: loads the kernels, on counters of its own
    accumulate(warm)
    del warm
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    accumulate(counts)
    e1.record()
    torch.cuda.synchronize()
    hist_ms = e0.elapsed_time(e1)
    del all_ids
    sel_ms = []
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fs.fs_plan_replication(None, None, 1, 1, None, 0, R, counts, fs.FS_PLAN_SELECT, budget, bpr, sel, nsel, None, status,
                               workspace=ws_sel)
        e1.record()
        torch.cuda.synchronize()
        sel_ms.append(e0.elapsed_time(e1))
    assert int(status.item()) == 0, f"device status {int(status.item())}"
    assert int(counts.to(torch.int64).sum().item()) == seen == T * per_table
    k = int(nsel.item())
    distinct = int((counts != 0).sum().item())
    assert k == min(cap, distinct)
    hist_bytes = seen * 8 + distinct * 8                 # every id once, one counter update per distinct row
    sel_bytes = R * 4 + k * 8                            # counts once, the selection out
    total_ms = hist_ms + min(sel_ms)
    return {
        "config": {"workload": f"c5 planning: {seen} sampled ids over {T} tables x {cfg.E} rows, Zipf({cfg.alpha}), "
                               f"histogram in {len(calls)} call(s) of up to {chunk} ids, then top-k under {budget} bytes at {bpr} "
                               f"bytes per row",
                   "ids": seen, "distinct_rows": distinct, "selected": k, "budget_rows": cap},
        "metric": "sampled ids/sec through fs_plan_replication (histogram, then top-k)", "unit": "ids/s",
        "value": round(seen / (total_ms * 1e-3), 1), "ms": round(total_ms, 3),
        "roofline": {"bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "calls": {"fs_plan_replication[ACCUMULATE]": {**frac_of_peak(hist_bytes, hist_ms), "launch_calls": len(calls)},
                               "fs_plan_replication[SELECT]": frac_of_peak(sel_bytes, min(sel_ms))}},
        "wall_s_with_id_generation": round(time.time() - t_wall, 1),
    }


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU only (owner buckets are output partitions, no "
              f"collectives); --gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    import fs_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    main_name = args.config or "c3"
    cfg = fs_inputs.CONFIGS[main_name]
    if args.scale_rows > 1:
        cfg = cfg.scaled(E=cfg.E // args.scale_rows)

    fields, keep = run_step_config(cfg, args, args.steps, args.warmup, full_report=True)
    result = {
        "metric": "embedding lookups/sec and achieved HBM GB/s (% of peak), fwd+bwd, 1 GPU",
        "value": fields.pop("value"), "unit": "lookups/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": fields.pop("ms_per_step"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"f32": "f32", "f16": "f16", "bf16": "bf16"}[cfg.dtype] + " rows, f32 accumulation, int64/int32 indices",
        "data": "synthetic",
    }
    result.update(fields)

    # ---------------------------------------------------------------- CPU oracle on a bounded sample
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args, cfg, *keep)
    del keep, fields
    gc.collect()
    torch.cuda.empty_cache()

    # ---------------------------------------------------------------- the other single-GPU workloads
    # Only in the default run: c4 (the largest shard, 164 GB of tables: the same step, fewer repetitions)
    # and the c5 planning pass.  Reported beside the headline, never part of `value`.
    if args.config is None and not args.no_also:
        also = []
        free_b = torch.cuda.mem_get_info()[0]
        if free_b > 262e9:
            c4_fields, _ = run_step_config(fs_inputs.CONFIGS["c4"], args, max(3, args.steps // 4), 2, full_report=False)
            c4_fields["unit"] = "lookups/s"
            also.append(c4_fields)
            gc.collect()
            torch.cuda.empty_cache()
        else:
            also.append({"config": {"workload": "c4"}, "skipped": f"needs ~262 GB of free HBM, {free_b / 1e9:.0f} GB free"})
        also.append(run_c5_planning(args))
        result["also_configs"] = also

    print(json.dumps(result), flush=True)


def cpu_baseline(args, cfg, ids, offsets, placement, weights, grad_out):
    """The oracle as it stands (one thread) on the first tables of the same batch: plan + route +
    gather + backward on the host copy of exactly those inputs."""
    import numpy as np
    import fs_inputs
    import oracle

    B, E, D = cfg.B, cfg.E, cfg.D
    tables = args.cpu_tables
    if tables <= 0:                                   # aim at ~16M lookups (about 10 s of one core)
        per_table = max(1, int(offsets[B].item()))
        tables = max(1, min(cfg.T, -(-16_000_000 // per_table)))
        while tables > 1 and tables * E * cfg.row_bytes > 48e9:      # keep the host copy of the table modest
            tables -= 1
    n_s = int(offsets[tables * B].item())
    ids_h = ids[:n_s].cpu().numpy()
    off_h = offsets[:tables * B + 1].cpu().numpy()
    rb_h = (np.arange(tables + 1) * E).astype(np.int64)
    pl_h = placement[:tables * E].cpu().numpy().view(np.uint32)
    w_h = fs_inputs.as_numpy_bits(weights[:tables * E])
    g_h = fs_inputs.as_numpy_bits(grad_out[:n_s])
    code = {"f32": oracle.F32, "f16": oracle.F16, "bf16": oracle.BF16}[cfg.dtype]
    R_s = tables * E
    counts = np.zeros(R_s, np.uint32)
    budget_rows = max(1, int((cfg.f_global if cfg.f_global > 0 else 0.01) * R_s))
    out_h = np.zeros((n_s, D), w_h.dtype)
    oracle.lib()
    t0 = time.perf_counter()
    rc0, _, _ = oracle.plan_replication(ids_h, off_h, tables, B, rb_h, R_s, counts,
                                        oracle.PLAN_ACCUMULATE | oracle.PLAN_SELECT, budget_rows * cfg.row_bytes,
                                        cfg.row_bytes)
    rc1, st, bo, rows, pos, tc = oracle.route_bucketize(ids_h, off_h, tables, B, rb_h, pl_h, cfg.U, cfg.W,
                                                        cfg.self_bucket)
    rc2, _ = oracle.seq_gather_fwd(w_h, rows, pos, 0, n_s, out_h, dtype=code)
    rc3, _, u, g32, _, nu = oracle.seq_grad_bwd(g_h, rows, pos, 0, n_s, R_s, dtype=code, want64=False,
                                                cap_unique=min(n_s, R_s))
    dt = time.perf_counter() - t0
    assert rc0 == rc1 == rc2 == rc3 == 0
    return {"value": round(n_s / dt, 1), "unit": "lookups/s", "cores": 1, "kind": "oracle",
            "sample": f"first {tables} of {cfg.T} tables of the same batch ({n_s} lookups, {nu} distinct rows), "
                      f"plan + route + gather + backward, single-threaded C oracle, {dt:.2f} s",
            "host_cores_available": os.cpu_count()}


if __name__ == "__main__":
    main()
