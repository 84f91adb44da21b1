#!/usr/bin/env python3
"""Benchmark of the re-layout hot path on one MI355X.

A step is one pass of the whole path over one synthetic rollout batch that is already resident
in HBM: earl_plan_build (source offsets, padded geometry, rank assignment, packing,
micro-batches, segment table) followed by earl_dispatch (every field, every destination shard,
position ids, cu_seqlens).  The default workload is "heavy" (2048 sequences, about 12.4 M tokens,
2065 bytes per token, DP8 x SP4 zigzag: the largest of the five workloads by bytes moved);
`--workload longctx` is the largest by tokens.

Prints ONE JSON line:  value = real tokens re-laid-out per second over the timed steps
(plan + dispatch, whole job); `roofline` prices the re-layout kernel alone against the 8 TB/s
HBM peak with algorithmic bytes (each real source row read once, each destination row written
once, 4 bytes of position id per destination row) over its HIP-event duration; `cpu_baseline`
is the CPU oracle timed on a bounded sample of the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM traffic of one re-layout kernel launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (scaled by a plain copy kernel of known size, see profiles/), keyed by the sha256 of the kernel
# source the counters were taken on.  A changed kernel reports null until re-measured.
MEASURED_TRAFFIC = {
    "a9b49484a65209c256c1d856cd49a6200fdd70b18845382e075c7d8e5bf33e1b":
        {"heavy": 52882838527, "longctx": 47518212261},
}

WORKLOAD_NOTES = {
    "tiny": "c1 tiny: 64 seqs U[16,512], 4 src shards, 4 fields (13 B/token), DP2 SP1, budget 4096",
    "mid": "c2 mid: 1024 seqs lognormal(2048,0.8) in [64,8192], 8 src shards, 5 fields (17 B/token), "
           "DP8 SP2 zigzag, pad 64, budget 16384",
    "agentic": "c3 agentic multi-turn: 512 episodes x 2-12 turns, TP4xDP2 replicated source "
               "(8 shards), 5 fields (17 B/token), DP4 SP4, budget 65536",
    "heavy": "c4 heavy intermediates: 2048 seqs lognormal(4096,0.9) in [128,32768] (~12.4M tokens), "
             "8 src shards, 5 scalar fields + bf16[1024] (2065 B/token), DP8 SP4 zigzag, budget 131072",
    "longctx": "c5 long-context: 256 seqs U[32768,131072] (~21.9M tokens), 8 src shards, 5 scalar "
               "fields + bf16[512] (1041 B/token), DP2 SP8 zigzag, pad 128, budget 262144",
}


def kernel_source_hash() -> str:
    """sha256 over the sources the re-layout kernels are built from (kernel file + constants)."""
    h = hashlib.sha256()
    for name in ("earl_copy.hip", "earl_internal.h"):
        with open(os.path.join(ROOT, "paper_2510_05943_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


class HipEvents:
    """hipEvent_t handles through ctypes (the HIP runtime is already loaded by torch)."""

    def __init__(self):
        import ctypes
        self.c = ctypes
        self.lib = ctypes.CDLL("libamdhip64.so")
        self.lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.lib.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                                 ctypes.c_void_p]

    def create(self) -> int:
        ev = self.c.c_void_p()
        if self.lib.hipEventCreate(self.c.byref(ev)) != 0:
            raise RuntimeError("hipEventCreate failed")
        return ev.value

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = self.c.c_float()
        if self.lib.hipEventElapsedTime(self.c.byref(ms), a, b) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return float(ms.value)

    def destroy(self, ev: int) -> None:
        self.lib.hipEventDestroy(ev)


def run_gpu(args, torch, B, synth):
    w = synth.make_workload(args.workload, seed=args.seed)
    t0 = time.time()
    src = {f.name: w.device_shard_buffers(f, torch) for f in w.fields}
    torch.cuda.synchronize()
    stage_s = time.time() - t0

    stream = torch.cuda.current_stream()
    src_l = B.SrcLayout(w.n_groups, w.replication)
    dst_l = B.DstLayout(w.dp, w.sp, w.zigzag, w.pad_multiple, w.mb_token_budget, args.balance_policy)
    lengths = torch.from_numpy(w.lengths.astype(np.int32)).cuda()
    ws = torch.empty(B.plan_workspace_bytes(w.n_seqs, src_l, dst_l), dtype=torch.uint8, device="cuda")

    # sizes of the destination shards come from a first plan
    plan0 = B.plan_build(lengths, w.n_seqs, src_l, dst_l, ws, stream=stream)
    sm = B.plan_get_summary(plan0)
    shard_rows = [int(r) for r in sm["shard_rows"]]
    fields = []
    for f in w.fields:
        dsts = [torch.empty((r * f.row_bytes,), dtype=torch.uint8, device="cuda") for r in shard_rows]
        fields.append(B.Field(f.scalar_bytes, f.width, f.pad_scalar, src[f.name], dsts))
    pos = [torch.empty((r,), dtype=torch.int32, device="cuda") for r in shard_rows]
    cu = torch.empty((sm["cu_seqlens_len"],), dtype=torch.int32, device="cuda")

    scratch = torch.empty(B.dispatch_workspace_bytes(plan0, fields), dtype=torch.uint8, device="cuda")
    B.plan_destroy(plan0)

    row_bytes = sum(f.row_bytes for f in w.fields)
    algo_bytes = (row_bytes * sm["total_real_rows"] + row_bytes * sm["total_dst_rows"]
                  + 4 * sm["total_dst_rows"])
    if args.inverse:
        # training layout -> rollout layout: every real row read once and written once
        algo_bytes = 2 * row_bytes * sm["total_real_rows"]
        p1 = B.plan_build(lengths, w.n_seqs, src_l, dst_l, ws, stream=stream)
        B.dispatch(p1, fields, position_ids=pos, cu_seqlens=cu, workspace=scratch, stream=stream)
        torch.cuda.synchronize()        # the destination shards now hold a real training layout
        B.plan_destroy(p1)

    hip = HipEvents()

    def step(ev=None):
        p = B.plan_build(lengths, w.n_seqs, src_l, dst_l, ws, stream=stream)
        if args.async_dispatch:
            # buffers are pre-allocated: the dispatch goes in right behind the plan, the summary
            # and the device-side verdict are fetched afterwards
            if ev is not None:
                B.plan_set_dispatch_events(p, ev[0], ev[1])
            B.dispatch_async(p, fields, position_ids=pos, cu_seqlens=cu, workspace=scratch, stream=stream)
            B.plan_get_summary(p)
            return p
        B.plan_get_summary(p)          # the consumer needs the shard sizes before it can dispatch
        if ev is not None:
            B.plan_set_dispatch_events(p, ev[0], ev[1])
        if args.inverse:
            B.dispatch_inverse(p, fields, workspace=scratch, stream=stream)
        else:
            B.dispatch(p, fields, position_ids=pos, cu_seqlens=cu, workspace=scratch, stream=stream)
        return p

    if args.reference_copy:
        # a plain copy of known size on the same stream: the yardstick for the HBM counters
        n = 4 << 30
        a = torch.empty(n, dtype=torch.uint8, device="cuda")
        b = torch.empty(n, dtype=torch.uint8, device="cuda")
        a.view(torch.int32).fill_(1)
        for _ in range(3):
            b.view(torch.int32).copy_(a.view(torch.int32))
        torch.cuda.synchronize()
        del a, b

    plans = [step() for _ in range(args.warmup)]
    torch.cuda.synchronize()
    for p in plans:
        if args.async_dispatch and B.dispatch_async_status(p) != B.EARL_OK:
            raise RuntimeError("asynchronous dispatch was refused on the device")
        B.plan_destroy(p)

    # HIP events recorded by the library on the dispatch stream, right around the re-layout kernel
    events = [(hip.create(), hip.create()) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plans = [step(events[k]) for k in range(args.steps)]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for p in plans:
        if args.async_dispatch and B.dispatch_async_status(p) != B.EARL_OK:
            raise RuntimeError("asynchronous dispatch was refused on the device")
        B.plan_destroy(p)

    # the two halves on their own (outside the timed region): plan = build + summary (ends with
    # the library's own stream synchronisation), dispatch = enqueue + stream synchronisation
    plan_ms, dispatch_ms = [], []
    for _ in range(10):
        ta = time.perf_counter()
        p = B.plan_build(lengths, w.n_seqs, src_l, dst_l, ws, stream=stream)
        B.plan_get_summary(p)
        tb = time.perf_counter()
        if args.inverse:
            B.dispatch_inverse(p, fields, workspace=scratch, stream=stream)
        else:
            B.dispatch(p, fields, position_ids=pos, cu_seqlens=cu, workspace=scratch, stream=stream)
        torch.cuda.synchronize()
        tc = time.perf_counter()
        B.plan_destroy(p)
        plan_ms.append((tb - ta) * 1e3)
        dispatch_ms.append((tc - tb) * 1e3)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kern_ms = [hip.elapsed_ms(a, b) for a, b in events]
    for a, b in events:
        hip.destroy(a)
        hip.destroy(b)
    kern_avg_ms = float(np.mean(kern_ms))
    achieved = algo_bytes / (kern_avg_ms * 1e-3) / 1e9
    traffic = None if (args.inverse or args.balance_policy) else MEASURED_TRAFFIC.get(kernel_source_hash(), {}).get(args.workload)
    return dict(w=w, sm=sm, ms_per_step=ms_per_step, kern_avg_ms=kern_avg_ms,
                kern_min_ms=float(np.min(kern_ms)), kern_median_ms=float(np.median(kern_ms)),
                achieved=achieved, algo_bytes=algo_bytes,
                traffic=traffic, stage_s=stage_s, row_bytes=row_bytes,
                plan_ms=float(np.median(plan_ms)), dispatch_ms=float(np.median(dispatch_ms)))


def run_gpu_two_pass(args, torch, B, synth):
    """The single-controller pattern the paper argues against (Section 1: all intermediate data is
    aggregated in one place before it is redistributed), done with the same library on one GPU:
    pass 1 gathers every field into one canonical buffer (plan with dp = sp = 1), pass 2 scatters
    it from there into the training layout.  Same result as the direct dispatch, twice the bytes."""
    w = synth.make_workload(args.workload, seed=args.seed)
    t0 = time.time()
    src = {f.name: w.device_shard_buffers(f, torch) for f in w.fields}
    torch.cuda.synchronize()
    stage_s = time.time() - t0
    stream = torch.cuda.current_stream()
    lengths = torch.from_numpy(w.lengths.astype(np.int32)).cuda()
    lay_a = (B.SrcLayout(w.n_groups, w.replication), B.DstLayout(1, 1, 0, 1, 1 << 40))
    lay_b = (B.SrcLayout(1, 1), B.DstLayout(w.dp, w.sp, w.zigzag, w.pad_multiple, w.mb_token_budget,
                                            args.balance_policy))
    ws_a = torch.empty(B.plan_workspace_bytes(w.n_seqs, *lay_a), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(B.plan_workspace_bytes(w.n_seqs, *lay_b), dtype=torch.uint8, device="cuda")
    pa = B.plan_build(lengths, w.n_seqs, *lay_a, ws_a, stream=stream)
    pb = B.plan_build(lengths, w.n_seqs, *lay_b, ws_b, stream=stream)
    sm_a, sm = B.plan_get_summary(pa), B.plan_get_summary(pb)
    total = int(sm_a["shard_rows"][0])
    shard_rows = [int(r) for r in sm["shard_rows"]]
    fields_a, fields_b = [], []
    for f in w.fields:
        canon = torch.empty((total * f.row_bytes,), dtype=torch.uint8, device="cuda")
        dsts = [torch.empty((r * f.row_bytes,), dtype=torch.uint8, device="cuda") for r in shard_rows]
        fields_a.append(B.Field(f.scalar_bytes, f.width, f.pad_scalar, src[f.name], [canon]))
        fields_b.append(B.Field(f.scalar_bytes, f.width, f.pad_scalar, [canon], dsts))
    pos = [torch.empty((r,), dtype=torch.int32, device="cuda") for r in shard_rows]
    cu = torch.empty((sm["cu_seqlens_len"],), dtype=torch.int32, device="cuda")
    scr_a = torch.empty(B.dispatch_workspace_bytes(pa, fields_a, False, False), dtype=torch.uint8, device="cuda")
    scr_b = torch.empty(B.dispatch_workspace_bytes(pb, fields_b), dtype=torch.uint8, device="cuda")
    B.plan_destroy(pa)
    B.plan_destroy(pb)
    row_bytes = sum(f.row_bytes for f in w.fields)
    algo_bytes = (2 * row_bytes * total
                  + row_bytes * (sm["total_real_rows"] + sm["total_dst_rows"]) + 4 * sm["total_dst_rows"])
    hip = HipEvents()

    def step(ev=None):
        a = B.plan_build(lengths, w.n_seqs, *lay_a, ws_a, stream=stream)
        B.plan_get_summary(a)
        if ev is not None:
            B.plan_set_dispatch_events(a, ev[0], ev[1])
        B.dispatch(a, fields_a, workspace=scr_a, stream=stream)
        b = B.plan_build(lengths, w.n_seqs, *lay_b, ws_b, stream=stream)
        B.plan_get_summary(b)
        if ev is not None:
            B.plan_set_dispatch_events(b, ev[2], ev[3])
        B.dispatch(b, fields_b, position_ids=pos, cu_seqlens=cu, workspace=scr_b, stream=stream)
        return [a, b]

    plans = [p for _ in range(args.warmup) for p in step()]
    torch.cuda.synchronize()
    for p in plans:
        B.plan_destroy(p)
    events = [tuple(hip.create() for _ in range(4)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plans = [p for k in range(args.steps) for p in step(events[k])]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for p in plans:
        B.plan_destroy(p)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kern_ms = [hip.elapsed_ms(e[0], e[1]) + hip.elapsed_ms(e[2], e[3]) for e in events]
    for e in events:
        for x in e:
            hip.destroy(x)
    kern_avg_ms = float(np.mean(kern_ms))
    return dict(w=w, sm=sm, ms_per_step=ms_per_step, kern_avg_ms=kern_avg_ms,
                kern_min_ms=float(np.min(kern_ms)), achieved=algo_bytes / (kern_avg_ms * 1e-3) / 1e9,
                algo_bytes=algo_bytes, traffic=None, stage_s=stage_s, row_bytes=row_bytes)


def run_cpu_baseline(args, synth):
    """The oracle as it stands (single thread: Python loops + numpy slice copies) on a bounded
    sample of the workload: a reduced sequence count with the same length distribution, fields
    and layouts, forward path only (plan, all fields, all shards, position ids), repeated until
    about ten seconds of CPU time have been spent."""
    from oracle import earl_oracle as O
    scale = {"tiny": 1.0, "mid": 1.0, "agentic": 1.0, "heavy": 1.0 / 8, "longctx": 1.0 / 8}[args.workload]
    w = synth.make_workload(args.workload, seed=args.seed, scale=scale)
    host = {f.name: [w.group_buffer(f, s // w.replication) for s in range(w.n_shards)]
            for f in w.fields}
    passes = 0
    t0 = time.perf_counter()
    while True:
        plan = O.build_plan(w.lengths, n_groups=w.n_groups, replication=w.replication,
                            seq_group=w.seq_group, dp=w.dp, sp=w.sp, zigzag=w.zigzag,
                            pad_multiple=w.pad_multiple, mb_token_budget=w.mb_token_budget)
        for q in range(w.dp * w.sp):
            O.position_ids_shard(plan, q)
            for f in w.fields:
                O.dispatch_field_shard(plan, q, host[f.name], f.np_dtype, f.width, f.pad_scalar)
        passes += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or passes >= 200:
            break
    row_bytes = sum(f.row_bytes for f in w.fields)
    algo = row_bytes * (plan.total_real_rows + plan.total_dst_rows) + 4 * plan.total_dst_rows
    return {"value": passes * w.total_tokens / dt, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "GBps": passes * algo / dt / 1e9,
            "sample": f"{w.n_seqs} sequences drawn like the workload ({w.total_tokens} tokens, "
                      f"{algo / 1e9:.2f} GB moved per pass), all fields, all {w.dp * w.sp} destination "
                      f"shards, plan + dispatch, {passes} passes in {dt:.1f} s on one core "
                      f"(host reports {os.cpu_count()} logical cpus)"}


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="heavy", choices=list(WORKLOAD_NOTES))
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--two-pass", action="store_true",
                    help="gather into one canonical buffer, then scatter (single-controller pattern)")
    ap.add_argument("--balance-policy", type=int, default=0, choices=[0, 1, 2],
                    help="0 longest-first list scheduling (default), 1 sorted snake deal, "
                         "2 list scheduling on squared padded lengths")
    ap.add_argument("--async-dispatch", action="store_true",
                    help="step = earl_plan_build + earl_dispatch_async + earl_plan_get_summary "
                         "(no host wait between plan and dispatch)")
    ap.add_argument("--inverse", action="store_true",
                    help="time the reverse direction (earl_dispatch_inverse) instead of earl_dispatch")
    ap.add_argument("--reference-copy", action="store_true",
                    help="also run three plain 4 GiB device copies (for scaling profiler counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the re-layout (all destination shards in one "
              "HBM); this library has no multi-GPU path: run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2510_05943_amd import binding as B
    from paper_2510_05943_amd import synth
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    B.load_library()
    torch.cuda.set_device(0)

    r = run_gpu_two_pass(args, torch, B, synth) if args.two_pass else run_gpu(args, torch, B, synth)
    w, sm = r["w"], r["sm"]
    line = {
        "metric": "re-layout throughput: tokens/s and achieved HBM GB/s (% of peak) at 1 GPU",
        "value": sm["total_real_rows"] / (r["ms_per_step"] * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_NOTES[args.workload], "name": args.workload,
                   "seed": args.seed, "n_seqs": w.n_seqs, "real_tokens": sm["total_real_rows"],
                   "dst_rows": sm["total_dst_rows"], "bytes_per_token_row": r["row_bytes"],
                   "dst_shards": w.dp * w.sp, "src_shards": w.n_shards,
                   "balance_policy": args.balance_policy,
                   "step": ("two passes (gather to one buffer, scatter from it), each " if args.two_pass
                            else "") + ("earl_plan_build + earl_dispatch_async + earl_plan_get_summary"
                                        if args.async_dispatch else
                                        "earl_plan_build + earl_plan_get_summary + " +
                                        ("earl_dispatch_inverse" if args.inverse else "earl_dispatch"))},
        "whole_path_GBps": r["algo_bytes"] / (r["ms_per_step"] * 1e-3) / 1e9,
        "roofline": {"bound": "hbm", "achieved": r["achieved"], "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": r["achieved"] / HBM_PEAK_GBPS, "traffic": r["traffic"],
                     "kernel": ("inverse_kernel" if args.inverse else
                                "relayout_kernel (both passes)" if args.two_pass else "relayout_kernel"),
                     "algorithmic_bytes_per_launch": r["algo_bytes"],
                     "kernel_ms_avg": r["kern_avg_ms"], "kernel_ms_min": r["kern_min_ms"],
                     "kernel_ms_median": r.get("kern_median_ms")},
        "input_staging_s": r["stage_s"],
    }
    if "plan_ms" in r:
        # the two calls on their own, each ending with a stream synchronisation (medians of 10)
        line["plan_ms"] = r["plan_ms"]
        line["dispatch_ms"] = r["dispatch_ms"]
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = run_cpu_baseline(args, synth)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
